// bf16 prefix-cached paged prefill attention, 64 query rows per wave, one wave per SIMD.
//
// Same mathematics, data layout in LDS and transposed MFMA formulation as attn_bf16.hip
// (S^T = K.Q^T and O^T += V^T.P^T with v_mfma_f32_32x32x16_bf16, a lane owns a query row;
// paper Sec. 3.2 / Sec. 4 / Sec. 5.1 / Sec. 6 for what is computed).  What differs is the
// schedule: a wave owns two 32-row slabs and works in units of one 32-key sub-tile, software
// pipelined so that the matrix cores and the vector ALU run at the same time inside one wave:
//
//   iteration u:   pre  row max of S(u), raise the running max if needed          (VALU)
//                  X    O += P(u-1).V(u-1)   ||  exp2 / sum / bf16 of S(u), slab 0  (MFMA || VALU)
//                  sync one plane (K or V) of a later tile has landed; issue the next copy
//                  Y    S(u+1) = K(u+1).Q    ||  exp2 / sum / bf16 of S(u), slab 1  (MFMA || VALU)
//
// Every K (V) operand read from LDS feeds two MFMAs (one per slab), so LDS traffic per flop is
// half that of the 32-row kernel, and there is one barrier per 32 keys x 64 rows of work.
// K and V travel in separate rings of R tiles each: K(T) dies after S(2T+1) is computed, V(T)
// one iteration later, so with one barrier per iteration a ring of two already gives a full
// tile of lead time; R = 4 keeps three tiles in flight.
//
// NG = 1: four waves x 64 rows = 256 rows per work item.  NG = 2: two groups of two waves work
// on the same 128 rows and on alternating key tiles, merged through LDS at the end (for launches
// with too few rows to fill the chip).
#include "attn_bf16_common.h"

namespace ragc {
namespace {

template <int D, int NG, int R>
__global__ __launch_bounds__(256, 1) void attn_bf16_w64_kernel(AttnLaunch a, AttnWorkList wl) {
    constexpr int WPG = 4 / NG;         // waves per group
    constexpr int TMV = 64 * WPG;       // rows per work item
    constexpr int BPW = 4 / WPG;        // 16-key blocks a wave copies per tile and plane
    constexpr int CPR = D / 8;          // 16-byte chunks per K/V row
    constexpr int ROWB = D * 2;         // bytes per row
    constexpr int PLANEB = TN * ROWB;   // one tile of K (or V)
    constexpr int RPI = 64 / CPR;       // rows covered by one wave-wide 1 KiB DMA instruction
    constexpr int IPB = 16 / RPI;       // DMA instructions per 16-row block
    constexpr int HP = BPW * IPB;       // DMA instructions per wave, tile and plane
    constexpr int KSTEPS = D / 16;
    constexpr int DT = D / 32;
    constexpr int GROUPB = 2 * R * PLANEB;  // K ring then V ring of one group
    static_assert(NG * GROUPB <= 160 * 1024, "LDS");
    __shared__ __attribute__((aligned(1024))) char smem[NG * GROUPB];

    // ---- work item (kv head from the low bits of the workgroup id: one stream, one XCD)
    const int Hkv = a.b.kv_heads;
    int g, item;
    if ((Hkv & 7) == 0) {
        const int x = blockIdx.x & 7, j = blockIdx.x >> 3, hpx = Hkv >> 3;
        g = x + 8 * (j % hpx);
        item = j / hpx;
    } else {
        g = blockIdx.x % Hkv;
        item = blockIdx.x / Hkv;
    }
    const AttnItem it = wl.item[item];
    const int r = it.req_tile >> 16, tile = it.req_tile & 0xffff;

    const int G = a.group;
    const int N = it.new_len;
    const int rows_total = N * G;
    const int row0 = tile * TMV;
    if (row0 >= rows_total) return;
    const int P = it.prefix_len;
    const int s0 = it.new_start;
    const int Hq = a.q_heads;
    const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = NG == 1 ? 0 : w / WPG, wq = w % WPG;

    const __bf16* __restrict__ q = static_cast<const __bf16*>(a.q);
    const __bf16* __restrict__ k_new = static_cast<const __bf16*>(a.k_new);
    const __bf16* __restrict__ v_new = static_cast<const __bf16*>(a.v_new);
    const __bf16* __restrict__ pool_k = static_cast<const __bf16*>(a.b.pool_k);
    const __bf16* __restrict__ pool_v = static_cast<const __bf16*>(a.b.pool_v);
    const int32_t* __restrict__ table = a.b.block_table + (long long)r * a.b.table_stride;

    const int last_row = min(row0 + TMV, rows_total) - 1;
    const int kv_limit = P + last_row / G + 1;  // keys [0, kv_limit) are visible to some row of the item
    const int ntiles = (kv_limit + TN - 1) / TN;
    const int nsteps = (ntiles + NG - 1) / NG;  // group `grp` takes tile T*NG + grp, T = 0 .. nsteps-1

    // ---- this lane's two query rows (slab s = rows wrow0 + 32 s + l32)
    const int wrow0 = row0 + wq * 64;
    const bool wave_active = wrow0 < rows_total;
    const int wave_vis_min = P + min(wrow0, rows_total - 1) / G + 1;
    int my_tok[2], my_head[2], my_vis[2];
    bf16x8 qreg[2][KSTEPS];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int row = min(wrow0 + 32 * s + l32, rows_total - 1);  // rows past the end repeat the last one
        my_tok[s] = row / G;
        my_head[s] = g * G + (row - my_tok[s] * G);
        my_vis[s] = P + my_tok[s] + 1;  // keys [0, my_vis) are visible to this row
        const __bf16* qp = q + ((long long)(s0 + my_tok[s]) * Hq + my_head[s]) * D + hf * 8;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) qreg[s][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    }
    // The compiler waits for the Q registers here, not at their first use inside the pipeline.
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) asm volatile("" ::"v"(qreg[s][ks]));
    wait_vmcnt<0>();

    // ---- DMA: wave (grp, wq) copies blocks wq*BPW .. +BPW-1 (16 keys each) of a tile, one plane at a time
    uint32_t pool_loff[IPB], new_loff[IPB];  // this lane's chunk inside a pool block / a run of fresh rows (bytes)
#pragma unroll
    for (int c = 0; c < IPB; ++c) {
        const int row16 = RPI * c + lane / CPR;
        const int chunk = (lane % CPR) ^ swz<D>(row16);
        pool_loff[c] = (row16 * D + chunk * 8) * 2;
        new_loff[c] = (row16 * Hkv * D + chunk * 8) * 2;
    }
    const uint32_t smem_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem + grp * GROUPB;
    // block ids: lane i holds the table entry of logical block (base + i); refilled every 16 tiles
    int blkvec[2] = {0, 0}, blkbase[2] = {-(1 << 20), -(1 << 20)};
    auto issue = [&](int T, auto plane_c) __attribute__((always_inline)) {  // plane 0 = K, 1 = V; T = tile index within the group
        constexpr int plane = decltype(plane_c)::value;
        const int tg = min(T * NG + grp, ntiles - 1);  // past the end: re-read the last tile (same number of loads)
        if (tg * 4 + 3 - blkbase[plane] >= 64) {
            blkbase[plane] = tg * 4;
            const int e = tg * 4 + lane;
            blkvec[plane] = (e << 4) < P ? table[e] : 0;
            asm volatile("" ::"v"(blkvec[plane]));  // the compiler's wait for this load stays inside the branch
        }
        const __bf16* pool = plane ? pool_v : pool_k;
        const __bf16* fresh = plane ? v_new : k_new;
        const uint32_t slot = smem_addr + (plane * R + T % R) * PLANEB;
#pragma unroll
        for (int bb = 0; bb < BPW; ++bb) {
            const int b16 = wq * BPW + bb;  // block within the tile
            const int kbase = tg * TN + b16 * 16;
            const int blk = __builtin_amdgcn_readlane(blkvec[plane], tg * 4 + b16 - blkbase[plane]);
            const uint32_t dst = slot + b16 * 16 * ROWB;
            if (kbase + 16 <= P) {
                // whole block cached: one pool block, uniform base + per-lane constant
                const uint64_t sb = uniform_u64(reinterpret_cast<const char*>(pool) +
                                                ((long long)blk * a.b.block_stride + (long long)g * kBlock * D) * 2);
#pragma unroll
                for (int c = 0; c < IPB; ++c) dma_16B_per_lane(sb, pool_loff[c], dst + RPI * c * ROWB);
            } else if (kbase >= P && kbase + 16 <= kv_limit) {
                // 16 fresh rows, all inside the horizon
                const uint64_t sb = uniform_u64(reinterpret_cast<const char*>(fresh) +
                                                (((long long)(s0 + kbase - P)) * Hkv + g) * D * 2);
#pragma unroll
                for (int c = 0; c < IPB; ++c) dma_16B_per_lane(sb, new_loff[c], dst + RPI * c * ROWB);
            } else {
                // the block straddles the prefix end or the horizon: choose the source per row;
                // rows past the horizon re-read the last visible one (they are masked later)
#pragma unroll
                for (int c = 0; c < IPB; ++c) {
                    const int row16 = RPI * c + lane / CPR;
                    const int chunk = (lane % CPR) ^ swz<D>(row16);
                    const int kj = kbase + row16;
                    long long off;
                    if (kj < P) {
                        off = (long long)blk * a.b.block_stride + ((long long)g * kBlock + row16) * D + chunk * 8;
                    } else {
                        const int kn = min(kj, kv_limit - 1) - P;
                        off = ((long long)(s0 + kn) * Hkv + g) * D + chunk * 8;
                    }
                    dma_16B_per_lane((kj < P ? pool : fresh) + off, dst + RPI * c * ROWB);
                }
            }
        }
    };

    // ---- per-lane LDS read offsets (bytes); slot and sub-tile parts are immediates
    typedef __attribute__((address_space(3))) char lds_char;
    lds_char* const lds0 = (lds_char*)smem;
    int koff[KSTEPS];  // K, A operand of S^T: row l32 (+32 sub), chunk 2*ks+hf
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
        koff[ks] = grp * GROUPB + l32 * ROWB + (((2 * ks + hf) ^ swz<D>(l32)) << 4);
        asm volatile("" : "+v"(koff[ks]));  // keep it one register: address = this + immediate
    }
    int voff[2][DT];  // V, A operand of O^T (transposing read): row 8*h2 + 4*hf + (lane&15)/4 (+16 kk +32 sub)
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const int row = 8 * h2 + 4 * hf + ((lane & 15) >> 2);
            const int elem = dt * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
            voff[h2][dt] = grp * GROUPB + R * PLANEB + row * ROWB + ((((elem >> 3)) ^ swz<D>(row)) << 4) + (elem & 7) * 2;
            asm volatile("" : "+v"(voff[h2][dt]));
        }

    f32x16 oacc[2][DT];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[s][dt][i] = 0.f;
    float m_run[2] = {-INFINITY, -INFINITY};  // reference exponent of O and l (log2 domain), at most 2^8 below the row max
    float l_run[2] = {0.f, 0.f};              // this lane's partial of the running sum (other half in lane^32)
    const float c = a.scale_log2e;

    f32x16 s_cur[2], s_nxt[2];  // S^T of sub-tile u and u+1, one 32x32 block per slab
    bf16x8 p_prev[2][2];        // P^T of sub-tile u-1: [slab][kk]
    bf16x8 p_cur[2][2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int e = 0; e < 8; ++e) p_cur[s][kk][e] = (__bf16)0.f;
    float m_sub[2];

    // S(u+1) = K.Q^T for sub-tile SUB of the tile in K slot KSLOT
    auto qk = [&](auto kslot_c, auto sub_c) __attribute__((always_inline)) {
        constexpr int KSLOT = decltype(kslot_c)::value, SUB = decltype(sub_c)::value;
        lds_char* const kst = lds0 + KSLOT * PLANEB + SUB * 32 * ROWB;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const bf16x8 ka = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(kst + koff[ks]);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                if (ks == 0) {
                    const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    s_nxt[s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[s][ks], z, 0, 0, 0);
                } else {
                    s_nxt[s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[s][ks], s_nxt[s], 0, 0, 0);
                }
            }
        }
    };
    // O^T += V^T.P^T for sub-tile SUB of the tile in V slot VSLOT, with the P of the previous iteration
    auto pv = [&](auto vslot_c, auto sub_c) __attribute__((always_inline)) {
        constexpr int VSLOT = decltype(vslot_c)::value, SUB = decltype(sub_c)::value;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            lds_char* const vb = lds0 + VSLOT * PLANEB + (SUB * 32 + kk * 16) * ROWB;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vb + voff[0][dt]));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vb + voff[1][dt]));
                const bf16x8 va = __builtin_shufflevector(__builtin_bit_cast(bf16x4, lo), __builtin_bit_cast(bf16x4, hi), 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int s = 0; s < 2; ++s) oacc[s][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, p_prev[s][kk], oacc[s][dt], 0, 0, 0);
            }
        }
    };
    // row max of S(u), mask on the causal frontier, raise the running max when a tile exceeds it by > 2^8
    auto pre = [&](int key0) __attribute__((always_inline)) {  // key0 = logical index of the sub-tile's first key
        if (__builtin_expect(key0 + 32 > wave_vis_min, 0)) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int kidx = key0 + (i >> 2) * 8 + hf * 4 + (i & 3);
                    if (kidx >= my_vis[s]) s_cur[s][i] = -INFINITY;
                }
        }
        float m_tile[2];
        bool raise[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            float mx = s_cur[s][0];
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s_cur[s][i]);
            mx = fmaxf(mx, other_half(mx));
            m_tile[s] = mx * c;
            raise[s] = m_tile[s] > m_run[s] + kRescaleThreshold;  // true on a row's first visible keys (m_run = -inf)
        }
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(raise[0] || raise[1]) != 0, 0)) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                // 1 where nothing changes, 0 on a row's first visible keys (exp2(-inf))
                const float alpha = raise[s] ? __builtin_amdgcn_exp2f(m_run[s] - m_tile[s]) : 1.f;
                m_run[s] = raise[s] ? m_tile[s] : m_run[s];
                l_run[s] *= alpha;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[s][dt][i] *= alpha;
                // P(u-1) was formed with the old exponent and is added to O after this point
#pragma unroll
                for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                    for (int e = 0; e < 8; ++e) p_prev[s][kk][e] = (__bf16)((float)p_prev[s][kk][e] * alpha);
            }
        }
        // a row that has seen no key yet has m_run = -inf and only masked scores: subtract 0 so
        // that exp2(-inf - 0) = 0 and not NaN
#pragma unroll
        for (int s = 0; s < 2; ++s) m_sub[s] = m_run[s] == -INFINITY ? 0.f : m_run[s];
    };
    // exp2 / partial row sum / bf16 of S(u) for one slab
    auto softmax_slab = [&](auto slab_c) __attribute__((always_inline)) {
        constexpr int S = decltype(slab_c)::value;
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float p = __builtin_amdgcn_exp2f(s_cur[S][i] * c - m_sub[S]);
            psum += p;
            p_cur[S][i >> 3][i & 7] = (__bf16)p;
        }
        l_run[S] += psum;
    };
    auto rotate = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            s_cur[s] = s_nxt[s];
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) p_prev[s][kk] = p_cur[s][kk];
        }
    };

    // ---- prologue: K(0..R-1), V(0..R-2) in flight, S(0)
#pragma unroll
    for (int T = 0; T < R; ++T) issue(T, std::integral_constant<int, 0>{});
#pragma unroll
    for (int T = 0; T < R - 1; ++T) issue(T, std::integral_constant<int, 1>{});
    wait_vmcnt<0>();
    block_barrier();
    qk(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    rotate();

    // one tile of the group = two iterations; J = T % R is a compile-time constant
    auto tile_step = [&](int T, auto j_c) __attribute__((always_inline)) {
        constexpr int J = decltype(j_c)::value;
        const int key0 = (T * NG + grp) * TN;
        // ---- iteration u = 2T: S(u) is sub-tile 0 of tile T
        pre(key0);
        if (T > 0) pv(std::integral_constant<int, (J + R - 1) % R>{}, std::integral_constant<int, 1>{});  // P(2T-1), V of tile T-1
        softmax_slab(std::integral_constant<int, 0>{});
        wait_vmcnt<(2 * R - 3) * HP>();  // V(T) has landed
        block_barrier();                 // ... for every wave; V(T-1) is dead
        issue(T + R - 1, std::integral_constant<int, 1>{});
        qk(std::integral_constant<int, J>{}, std::integral_constant<int, 1>{});  // S(2T+1): sub-tile 1 of tile T
        softmax_slab(std::integral_constant<int, 1>{});
        rotate();
        // ---- iteration u = 2T+1
        pre(key0 + 32);
        pv(std::integral_constant<int, J>{}, std::integral_constant<int, 0>{});  // P(2T), V of tile T
        softmax_slab(std::integral_constant<int, 0>{});
        wait_vmcnt<(2 * R - 3) * HP>();  // K(T+1) has landed
        block_barrier();                 // ... for every wave; K(T) is dead
        issue(T + R, std::integral_constant<int, 0>{});
        qk(std::integral_constant<int, (J + 1) % R>{}, std::integral_constant<int, 0>{});  // S(2T+2): sub-tile 0 of tile T+1
        softmax_slab(std::integral_constant<int, 1>{});
        rotate();
    };
    for (int T0 = 0; T0 < nsteps; T0 += R) {
        tile_step(T0, std::integral_constant<int, 0>{});
        if (T0 + 1 < nsteps) tile_step(T0 + 1, std::integral_constant<int, 1 % R>{});
        if (R > 2) {
            if (T0 + 2 < nsteps) tile_step(T0 + 2, std::integral_constant<int, 2 % R>{});
            if (T0 + 3 < nsteps) tile_step(T0 + 3, std::integral_constant<int, 3 % R>{});
        }
    }
    // ---- epilogue: the last P.V (sub-tile 1 of the last tile), then drain the ring
    {
        const int jl = (nsteps - 1) % R;
        if (jl == 0) pv(std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{});
        else if (jl == 1) pv(std::integral_constant<int, 1 % R>{}, std::integral_constant<int, 1>{});
        else if (jl == 2) pv(std::integral_constant<int, 2 % R>{}, std::integral_constant<int, 1>{});
        else pv(std::integral_constant<int, 3 % R>{}, std::integral_constant<int, 1>{});
    }
    wait_vmcnt<0>();

    // ---- fused append (after the key loop: nothing waits for it, and the fresh rows are L2-hot
    // because the loop has just read them as keys).  This work item owns the tokens whose first
    // row (head 0 of the group) it holds; 16-byte chunks, four per thread in flight.
    if (a.fused_append) {
        const int tok_lo = (row0 + G - 1) / G;
        const int tok_hi = min(N - 1, (row0 + TMV - 1) / G);
        __bf16* wk = static_cast<__bf16*>(a.pool_k_w);
        __bf16* wv = static_cast<__bf16*>(a.pool_v_w);
        const int n = (tok_hi - tok_lo + 1) * CPR;
        constexpr int UNR = 4;
        for (int i0 = tid; i0 < n; i0 += 256 * UNR) {
            int blk[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int idx = min(i0 + u * 256, n - 1);
                blk[u] = table[(P + tok_lo + idx / CPR) >> 4];
            }
            u32x4 kk[UNR], vv[UNR];
            long long dst[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int idx = min(i0 + u * 256, n - 1);
                const int tok = tok_lo + idx / CPR, ch = idx % CPR;
                const int pos = P + tok;
                const long long src = ((long long)(s0 + tok) * Hkv + g) * D + ch * 8;
                dst[u] = (long long)blk[u] * a.b.block_stride + ((long long)g * kBlock + (pos & 15)) * D + ch * 8;
                kk[u] = *reinterpret_cast<const u32x4*>(k_new + src);
                vv[u] = *reinterpret_cast<const u32x4*>(v_new + src);
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                if (i0 + u * 256 < n) {
                    *reinterpret_cast<u32x4*>(wk + dst[u]) = kk[u];
                    *reinterpret_cast<u32x4*>(wv + dst[u]) = vv[u];
                }
            }
        }
    }

    // ---- merge the wave groups through LDS (the rings are idle now)
    if (NG > 1) {
        float* xf = reinterpret_cast<float*>(smem);
        constexpr int WSTRIDE = 2 * (DT * 16 + 2) * 64;  // floats per wave
        block_barrier();
        if (grp == 1) {
            float* dst = xf + wq * WSTRIDE + lane;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) dst[((s * DT + dt) * 16 + i) * 64] = oacc[s][dt][i];
                dst[(2 * DT * 16 + 2 * s) * 64] = m_run[s];
                dst[(2 * DT * 16 + 2 * s + 1) * 64] = l_run[s];
            }
        }
        block_barrier();
        if (grp == 1) return;
        const float* src = xf + wq * WSTRIDE + lane;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const float m1 = src[(2 * DT * 16 + 2 * s) * 64], l1 = src[(2 * DT * 16 + 2 * s + 1) * 64];
            const float m = fmaxf(m_run[s], m1);  // group 0 always saw key 0: finite
            const float f0 = __builtin_amdgcn_exp2f(m_run[s] - m), f1 = __builtin_amdgcn_exp2f(m1 - m);
            l_run[s] = l_run[s] * f0 + l1 * f1;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[s][dt][i] = oacc[s][dt][i] * f0 + src[((s * DT + dt) * 16 + i) * 64] * f1;
        }
    }

    // ---- normalise and store: lane holds 4 consecutive d per (dt, i/4)
    if (!wave_active) return;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const float l_tot = l_run[s] + other_half(l_run[s]);
        const float inv = 1.f / l_tot;
        if (wrow0 + 32 * s + l32 < rows_total) {
            __bf16* op = static_cast<__bf16*>(a.out) + ((long long)(s0 + my_tok[s]) * Hq + my_head[s]) * D;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    bf16x4 o4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[s][dt][i4 * 4 + e] * inv);
                    *reinterpret_cast<bf16x4*>(op + dt * 32 + i4 * 8 + hf * 4) = o4;
                }
        }
    }
}

template <int D, int NG, int R>
void launch_w64(const AttnLaunch& a, const AttnWorkList& wl, hipStream_t s) {
    hipLaunchKernelGGL((attn_bf16_w64_kernel<D, NG, R>), dim3(wl.n * a.b.kv_heads), dim3(256), 0, s, a, wl);
}

}  // namespace

hipError_t launch_attn_bf16_w64(const AttnLaunch& a, const AttnWorkList& wl, int variant, hipStream_t s) {
    if (wl.n <= 0) return hipSuccess;
    const bool d64 = a.b.head_dim == 64;
    if (variant == kAttnVariantW64TwoGroups)
        d64 ? launch_w64<64, 2, 2>(a, wl, s) : launch_w64<128, 2, 2>(a, wl, s);
    else
        d64 ? launch_w64<64, 1, 4>(a, wl, s) : launch_w64<128, 1, 4>(a, wl, s);
    return hipGetLastError();
}

}  // namespace ragc
