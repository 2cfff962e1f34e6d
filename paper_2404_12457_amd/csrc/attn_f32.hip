// fp32 prefix-cached paged prefill attention (no matrix cores: the fp32 variant
// must hold 1e-4 against an fp64 reference, so products are plain fp32 FMAs).
//
// out[t,h,:] = softmax_j(scale * q[t,h,:].K_j) V_j over j = 0..prefix+i, where the
// first `prefix` keys are gathered from 16-token pool blocks through the request's
// block table (paper Sec. 5.1: non-contiguous blocks referenced by tree nodes) and
// the rest are the request's own fresh K/V (Sec. 3.2: only the request tokens are
// computed).  One workgroup = (request, q head, 16 new tokens); keys stream through
// LDS in chunks of 32; each wave owns 4 token rows and keeps an online softmax
// (running max, running sum, rescaled accumulator) per row.
#include "ragc_internal.h"

namespace ragc {
namespace {

constexpr int TR = 16;  // new tokens per workgroup
constexpr int KC = 32;  // keys per LDS chunk

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

template <int D>
__global__ __launch_bounds__(256) void attn_f32_kernel(AttnLaunch a) {
    __shared__ __attribute__((aligned(16))) float Ks[KC][D + 4];  // rows padded by one 16-byte chunk: 16-byte reads of 16 keys hit all banks
    __shared__ __attribute__((aligned(16))) float Vs[KC][D];
    __shared__ __attribute__((aligned(16))) float Qs[TR][D];
    __shared__ __attribute__((aligned(16))) float Ps[4][KC][4];  // per wave: p of its 4 rows, per key

    const int r = blockIdx.z;
    const int h = blockIdx.y;
    const int tile = gridDim.x - 1 - blockIdx.x;  // long key ranges first
    const int N = a.b.new_len[r];
    const int t0 = tile * TR;
    if (t0 >= N) return;
    const int P = a.b.prefix_len[r];
    const int s0 = a.b.new_start[r];
    const int g = h / a.group;
    const int rows = min(TR, N - t0);
    const int kv_limit = P + t0 + rows;  // keys [0, kv_limit) are visible to some row
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int Hkv = a.b.kv_heads;

    const float* __restrict__ q = static_cast<const float*>(a.q);
    const float* __restrict__ k_new = static_cast<const float*>(a.k_new);
    const float* __restrict__ v_new = static_cast<const float*>(a.v_new);
    const float* __restrict__ pool_k = static_cast<const float*>(a.b.pool_k);
    const float* __restrict__ pool_v = static_cast<const float*>(a.b.pool_v);
    const int32_t* __restrict__ table = a.b.block_table + (long long)r * a.b.table_stride;

    constexpr int C4 = D / 4;  // float4 chunks per row
    for (int idx = tid; idx < TR * C4; idx += 256) {
        const int row = idx / C4, c4 = idx % C4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < rows) v = *reinterpret_cast<const float4*>(q + ((long long)(s0 + t0 + row) * a.q_heads + h) * D + c4 * 4);
        *reinterpret_cast<float4*>(&Qs[row][c4 * 4]) = v;
    }

    // fused append: the first q head of each group stores this tile's fresh K/V rows
    if (a.fused_append && h % a.group == 0) {
        float* wk = static_cast<float*>(a.pool_k_w);
        float* wv = static_cast<float*>(a.pool_v_w);
        for (int idx = tid; idx < rows * C4; idx += 256) {
            const int row = idx / C4, c4 = idx % C4;
            const int pos = P + t0 + row;
            const long long src = ((long long)(s0 + t0 + row) * Hkv + g) * D + c4 * 4;
            const long long dst = (long long)table[pos >> 4] * a.b.block_stride + ((long long)g * kBlock + (pos & 15)) * D + c4 * 4;
            *reinterpret_cast<float4*>(wk + dst) = *reinterpret_cast<const float4*>(k_new + src);
            *reinterpret_cast<float4*>(wv + dst) = *reinterpret_cast<const float4*>(v_new + src);
        }
    }

    float m[4], l[4], o[4][D / 64];
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        m[rr] = -INFINITY;
        l[rr] = 0.f;
#pragma unroll
        for (int dd = 0; dd < D / 64; ++dd) o[rr][dd] = 0.f;
    }

    for (int c0 = 0; c0 < kv_limit; c0 += KC) {
        __syncthreads();
        for (int idx = tid; idx < KC * C4; idx += 256) {
            const int row = idx / C4, c4 = idx % C4;
            const int kj = c0 + row;
            float4 kk = make_float4(0.f, 0.f, 0.f, 0.f), vv = kk;
            if (kj < kv_limit) {
                if (kj < P) {
                    const long long off = (long long)table[kj >> 4] * a.b.block_stride + ((long long)g * kBlock + (kj & 15)) * D + c4 * 4;
                    kk = *reinterpret_cast<const float4*>(pool_k + off);
                    vv = *reinterpret_cast<const float4*>(pool_v + off);
                } else {
                    const long long off = ((long long)(s0 + kj - P) * Hkv + g) * D + c4 * 4;
                    kk = *reinterpret_cast<const float4*>(k_new + off);
                    vv = *reinterpret_cast<const float4*>(v_new + off);
                }
            }
            *reinterpret_cast<float4*>(&Ks[row][c4 * 4]) = kk;
            *reinterpret_cast<float4*>(&Vs[row][c4 * 4]) = vv;
        }
        __syncthreads();

        // scores of the wave's 4 rows at once: lane = (key, half of the head dim); every K chunk read
        // from LDS serves the 4 rows.  Rows past the end carry q = 0 and are never stored; a row
        // whose visible keys all lie in earlier chunks gets p = 0 and alpha = 1 below.
        const int key = lane & 31, dh = lane >> 5;
        float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int d4 = 0; d4 < D / 8; ++d4) {
            const float4 kk = *reinterpret_cast<const float4*>(&Ks[key][dh * (D / 2) + d4 * 4]);
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const float4 qq = *reinterpret_cast<const float4*>(&Qs[w * 4 + rr][dh * (D / 2) + d4 * 4]);
                part[rr] += qq.x * kk.x + qq.y * kk.y + qq.z * kk.z + qq.w * kk.w;
            }
        }
        float alpha[4];
        float4 p4;
        float* pp = reinterpret_cast<float*>(&p4);
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int visible = P + t0 + w * 4 + rr + 1;  // keys [0, visible): prefix, earlier new tokens, itself
            float sc = (part[rr] + __shfl_xor(part[rr], 32, 64)) * a.scale_log2e;
            if (c0 + key >= visible) sc = -INFINITY;
            const float m_new = fmaxf(m[rr], wave_max(sc));
            alpha[rr] = exp2f(m[rr] - m_new);  // first chunk: exp2(-inf) = 0
            pp[rr] = exp2f(sc - m_new);
            l[rr] = l[rr] * alpha[rr] + wave_sum(dh == 0 ? pp[rr] : 0.f);
            m[rr] = m_new;
        }
        __builtin_amdgcn_wave_barrier();
        if (dh == 0) *reinterpret_cast<float4*>(&Ps[w][key][0]) = p4;
        __builtin_amdgcn_wave_barrier();
        // O += P V: lane = column of V; every V element read from LDS serves the 4 rows
#pragma unroll
        for (int dd = 0; dd < D / 64; ++dd) {
            float acc[4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) acc[rr] = o[rr][dd] * alpha[rr];
#pragma unroll 8
            for (int j = 0; j < KC; ++j) {
                const float v = Vs[j][lane + 64 * dd];
                const float4 pj = *reinterpret_cast<const float4*>(&Ps[w][j][0]);
                acc[0] += pj.x * v;
                acc[1] += pj.y * v;
                acc[2] += pj.z * v;
                acc[3] += pj.w * v;
            }
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) o[rr][dd] = acc[rr];
        }
    }

    float* __restrict__ out = static_cast<float*>(a.out);
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int il = w * 4 + rr;
        if (il >= rows) continue;
        const float inv = 1.f / l[rr];
#pragma unroll
        for (int dd = 0; dd < D / 64; ++dd)
            out[((long long)(s0 + t0 + il) * a.q_heads + h) * D + lane + 64 * dd] = o[rr][dd] * inv;
    }
}

}  // namespace

hipError_t launch_attn_f32(const AttnLaunch& a, hipStream_t s) {
    if (a.max_new <= 0 || a.b.num_reqs <= 0) return hipSuccess;
    dim3 grid((a.max_new + TR - 1) / TR, a.q_heads, a.b.num_reqs);
    if (a.b.head_dim == 64)
        hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace ragc
