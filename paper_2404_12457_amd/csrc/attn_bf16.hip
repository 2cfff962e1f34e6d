// bf16 prefix-cached paged prefill attention on gfx950 matrix cores.
//
// out[t,h,:] = softmax_j(scale * q[t,h,:].K_j) V_j over j = 0..prefix+i: the first
// `prefix` keys come from 16-token pool blocks through the request's block table
// (paper Sec. 5.1: K/V of cached documents lives in non-contiguous blocks referenced
// by tree nodes), the rest are the request's own fresh K/V (Sec. 3.2: only the
// request tokens are computed), and the same pass can store that fresh K/V into its
// paged slots (Sec. 4: tensors are cached after the first token).
//
// Mapping.  One workgroup = (request, kv head, 128 rows); a row is a (new token,
// q head of the group) pair, token-major, so the G q heads of a GQA group share
// every K/V tile and a tile's causal frontier stays narrow.  4 waves x 32 rows.
// Keys stream through LDS in tiles of 64 (four pool blocks).
//
// The products are computed transposed so that a lane owns ONE query row:
//   S^T[key][row] = K . Q^T      A = K tile (LDS, 16-byte reads), B = Q (registers)
//   O^T[d][row]  += V^T . P^T    A = V tile read with the transposing LDS load,
//                                B = P^T, which is exactly the accumulator layout of
//                                S^T after conversion to bf16 -- no data movement.
// With v_mfma_f32_32x32x16_bf16 a lane holds 16 of the 32 keys of a sub-tile for its
// row; the other 16 sit in lane+32, so row max / row sum cost one half-swap each.
#include "ragc_internal.h"

namespace ragc {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int TM = 128;  // rows per workgroup
constexpr int TN = 64;   // keys per tile

__device__ __forceinline__ float other_half(float x) {
    // value held by lane ^ 32
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

template <int D>
struct Smem {
    static constexpr int KS = D + 8;   // K row stride (elements): 16-byte reads of 16 rows hit distinct banks
    static constexpr int VS = D + 32;  // V row stride: 4 rows x 64 bytes of a transposing read hit distinct banks
    __bf16 k[TN][KS];
    __bf16 v[TN][VS];
};

template <int D>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(AttnLaunch a) {
    constexpr int CPR = D / 8;               // 16-byte chunks per K/V row
    constexpr int LD = TN * CPR / 256;       // chunks per thread per tile and plane
    constexpr int KSTEPS = D / 16;
    constexpr int DT = D / 32;
    __shared__ Smem<D> sm;

    const int r = blockIdx.z;
    const int g = blockIdx.y;
    const int tile = gridDim.x - 1 - blockIdx.x;  // long key ranges first
    const int G = a.group;
    const int N = a.b.new_len[r];
    const int rows_total = N * G;
    const int row0 = tile * TM;
    if (row0 >= rows_total) return;
    const int P = a.b.prefix_len[r];
    const int s0 = a.b.new_start[r];
    const int Hkv = a.b.kv_heads;
    const int Hq = a.q_heads;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;

    const __bf16* __restrict__ q = static_cast<const __bf16*>(a.q);
    const __bf16* __restrict__ k_new = static_cast<const __bf16*>(a.k_new);
    const __bf16* __restrict__ v_new = static_cast<const __bf16*>(a.v_new);
    const __bf16* __restrict__ pool_k = static_cast<const __bf16*>(a.b.pool_k);
    const __bf16* __restrict__ pool_v = static_cast<const __bf16*>(a.b.pool_v);
    const int32_t* __restrict__ table = a.b.block_table + (long long)r * a.b.table_stride;

    const int last_row = min(row0 + TM, rows_total) - 1;
    const int kv_limit = P + last_row / G + 1;  // keys [0, kv_limit) are visible to some row of the tile
    const int ntiles = (kv_limit + TN - 1) / TN;

    // fused append: this workgroup owns the tokens whose first row (head 0 of the group) it holds
    if (a.fused_append) {
        const int tok_lo = (row0 + G - 1) / G;
        const int tok_hi = min(N - 1, (row0 + TM - 1) / G);
        __bf16* wk = static_cast<__bf16*>(a.pool_k_w);
        __bf16* wv = static_cast<__bf16*>(a.pool_v_w);
        const int n = (tok_hi - tok_lo + 1) * CPR;
        for (int idx = tid; idx < n; idx += 256) {
            const int tok = tok_lo + idx / CPR, ch = idx % CPR;
            const int pos = P + tok;
            const long long src = ((long long)(s0 + tok) * Hkv + g) * D + ch * 8;
            const long long dst = (long long)table[pos >> 4] * a.b.block_stride + ((long long)g * kBlock + (pos & 15)) * D + ch * 8;
            *reinterpret_cast<u32x4*>(wk + dst) = *reinterpret_cast<const u32x4*>(k_new + src);
            *reinterpret_cast<u32x4*>(wv + dst) = *reinterpret_cast<const u32x4*>(v_new + src);
        }
    }

    // this lane's query row
    const int my_row = min(row0 + w * 32 + l32, rows_total - 1);  // clamped: rows past the end repeat the last one
    const int my_tok = my_row / G;
    const int my_head = g * G + (my_row - my_tok * G);
    const int my_vis = P + my_tok + 1;  // keys [0, my_vis) are visible to this row
    const bool wave_active = row0 + w * 32 < rows_total;
    const int wave_vis_min = P + (row0 + w * 32) / G + 1;
    const int wave_vis_max = P + min(row0 + w * 32 + 31, rows_total - 1) / G + 1;

    bf16x8 qreg[KSTEPS];
    {
        const __bf16* qp = q + ((long long)(s0 + my_tok) * Hq + my_head) * D + hf * 8;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    }

    f32x16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.f;
    float m_run = -INFINITY;  // running max of scaled scores (log2 domain)
    float l_run = 0.f;        // this lane's partial of the running sum (other half in lane^32)
    const float c = a.scale_log2e;

    // global -> registers for one tile (zero beyond kv_limit: stale pool slots may hold anything)
    u32x4 kbuf[LD], vbuf[LD];
    auto prefetch = [&](int t) {
#pragma unroll
        for (int it = 0; it < LD; ++it) {
            const int idx = tid + it * 256;
            const int row = idx / CPR, ch = idx % CPR;
            const int kj = t * TN + row;
            u32x4 kk = {0u, 0u, 0u, 0u}, vv = {0u, 0u, 0u, 0u};
            if (kj < kv_limit) {
                if (kj < P) {
                    const long long off = (long long)table[kj >> 4] * a.b.block_stride + ((long long)g * kBlock + (kj & 15)) * D + ch * 8;
                    kk = *reinterpret_cast<const u32x4*>(pool_k + off);
                    vv = *reinterpret_cast<const u32x4*>(pool_v + off);
                } else {
                    const long long off = ((long long)(s0 + kj - P) * Hkv + g) * D + ch * 8;
                    kk = *reinterpret_cast<const u32x4*>(k_new + off);
                    vv = *reinterpret_cast<const u32x4*>(v_new + off);
                }
            }
            kbuf[it] = kk;
            vbuf[it] = vv;
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int it = 0; it < LD; ++it) {
            const int idx = tid + it * 256;
            const int row = idx / CPR, ch = idx % CPR;
            *reinterpret_cast<u32x4*>(&sm.k[row][ch * 8]) = kbuf[it];
            *reinterpret_cast<u32x4*>(&sm.v[row][ch * 8]) = vbuf[it];
        }
    };

    prefetch(0);
    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();  // every wave is done reading the previous tile
        stash();
        __syncthreads();
        if (t + 1 < ntiles) prefetch(t + 1);  // in flight while this tile is computed
        const int base = t * TN;
        if (!wave_active || base >= wave_vis_max) continue;

        // S^T = K Q^T
        f32x16 sacc[2];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[sub][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const bf16x8 ka = *reinterpret_cast<const bf16x8*>(&sm.k[sub * 32 + l32][ks * 16 + hf * 8]);
                sacc[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[ks], sacc[sub], 0, 0, 0);
            }
        }
        // causal frontier / end of sequence: only tiles that reach past the first row's horizon
        if (base + TN > wave_vis_min) {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int kidx = base + sub * 32 + (i >> 2) * 8 + hf * 4 + (i & 3);
                    if (kidx >= my_vis) sacc[sub][i] = -INFINITY;
                }
        }
        // online softmax, one row per lane pair (lane, lane^32)
        float mx = sacc[0][0];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[sub][i]);
        mx = fmaxf(mx, other_half(mx));
        const float m_new = fmaxf(m_run, mx * c);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
        bf16x8 pb[2][2];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float p = __builtin_amdgcn_exp2f(sacc[sub][i] * c - m_new);
                psum += p;
                pb[sub][i >> 3][i & 7] = (__bf16)p;
            }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[dt][i] *= alpha;

        // O^T += V^T P^T ; V rows fetched with the transposing LDS read
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const int vrow = sub * 32 + kk * 16 + hf * 4 + ((lane & 15) >> 2);
                const int vcol = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4*)(&sm.v[vrow][dt * 32 + vcol]));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4*)(&sm.v[vrow + 8][dt * 32 + vcol]));
                    const bf16x4 lo_b = __builtin_bit_cast(bf16x4, lo);
                    const bf16x4 hi_b = __builtin_bit_cast(bf16x4, hi);
                    const bf16x8 va = __builtin_shufflevector(lo_b, hi_b, 0, 1, 2, 3, 4, 5, 6, 7);
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[sub][kk], oacc[dt], 0, 0, 0);
                }
            }
    }

    // normalise and store: lane holds 4 consecutive d per (dt, i/4)
    if (!wave_active) return;
    const float l_tot = l_run + other_half(l_run);
    const float inv = 1.f / l_tot;
    if (row0 + w * 32 + l32 < rows_total) {
        __bf16* op = static_cast<__bf16*>(a.out) + ((long long)(s0 + my_tok) * Hq + my_head) * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                bf16x4 o4;
#pragma unroll
                for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[dt][i4 * 4 + e] * inv);
                *reinterpret_cast<bf16x4*>(op + dt * 32 + i4 * 8 + hf * 4) = o4;
            }
    }
}

}  // namespace

hipError_t launch_attn_bf16(const AttnLaunch& a, hipStream_t s) {
    if (a.max_new <= 0 || a.b.num_reqs <= 0) return hipSuccess;
    dim3 grid(((long long)a.max_new * a.group + TM - 1) / TM, a.b.kv_heads, a.b.num_reqs);
    if (a.b.head_dim == 64)
        hipLaunchKernelGGL(attn_bf16_kernel<64>, grid, dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(attn_bf16_kernel<128>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace ragc
