// bf16 prefix-cached paged prefill attention on gfx950 matrix cores.
//
// out[t,h,:] = softmax_j(scale * q[t,h,:].K_j) V_j over j = 0..prefix+i: the first
// `prefix` keys come from 16-token pool blocks through the request's block table
// (paper Sec. 5.1: K/V of cached documents lives in non-contiguous blocks referenced
// by tree nodes), the rest are the request's own fresh K/V (Sec. 3.2: only the
// request tokens are computed), and the same pass can store that fresh K/V into its
// paged slots (Sec. 4: tensors are cached after the first token).
//
// Mapping.  One work item = (request, kv head, 128 rows); a row is a (new token,
// q head of the group) pair, token-major, so the G q heads of a GQA group share
// every K/V tile and a tile's causal frontier stays narrow.  A wave owns 32 rows.
// Keys stream through LDS in tiles of 64 (four pool blocks): each wave copies one
// 16-token block of K and of V per tile straight from HBM into LDS
// (global_load_lds, 16 bytes per lane), one tile ahead of the math, into a ring of
// stages.  Rows are stored unpadded with their 16-byte chunks XOR-swizzled so that
// both the 16-byte K reads and the transposing V reads are bank-conflict free.
//
// NG wave groups of 4 waves work on the same 128 rows but on alternating key tiles
// (each with its own online-softmax state, merged through LDS at the end), so that a
// launch with few work items still puts 8 waves on a CU and one group's softmax
// overlaps the other's MFMAs.  With many work items NG = 1 and two workgroups share
// a CU instead.
//
// A launch whose work items all have at most 32 rows (decode steps) is compiled with DEC: the
// first two waves of a group share those rows and take one 32-key half of every tile each.
//
// A batch with few work items is also split along the keys ACROSS workgroups: a work item
// then appears S times in the list, each copy walks 1/S of the key tiles and leaves its
// unnormalised O and its (max, sum) per row in the caller's workspace, and attn_bf16_merge_kernel
// combines the S partial results of every row.  This is what keeps a single request, or a
// decode step, from running on a fraction of the chip.
//
// The products are computed transposed so that a lane owns ONE query row:
//   S^T[key][row] = K . Q^T      A = K tile (LDS, 16-byte reads), B = Q (registers)
//   O^T[d][row]  += V^T . P^T    A = V tile read with the transposing LDS load,
//                                B = P^T, which is exactly the accumulator layout of
//                                S^T after conversion to bf16 -- no data movement.
// With v_mfma_f32_32x32x16_bf16 a lane holds 16 of the 32 keys of a sub-tile for its
// row; the other 16 sit in lane+32, so a row max costs one half-swap.  The running
// max is only raised (and O, l rescaled) when a tile exceeds it by more than 2^8.
#include "attn_bf16_common.h"

namespace ragc {
namespace {

constexpr int TM = kAttnRowsPerItem;  // rows per work item

// SPLIT: the list holds several copies of every item, each with a share of the key tiles (a
// separate instantiation, so that the common unsplit kernel carries none of it).
template <int D, int NG, int RING, bool SPLIT, bool DEC>
__global__ __launch_bounds__(256 * NG, (NG == 1 && RING == 2) ? 2 : 1) void attn_bf16_kernel(AttnLaunch a, AttnWorkList wl) {
    // DEC: every work item of the launch has at most 32 rows (decode steps: one new token times the
    // group's q heads).  The rows then all sit in wave 0's block and three waves of four would only
    // copy; instead waves 0 and 1 of a group both take those 32 rows and one 32-key half of every
    // tile each, with private softmax state merged at the end like the wave groups' -- half the
    // MFMAs and half the softmax per wave and tile, which is what a step costs when nothing overlaps it.
    constexpr int NSUB = DEC ? 1 : 2;   // 32-key halves of a tile per wave
    constexpr int CPR = D / 8;          // 16-byte chunks per K/V row
    constexpr int ROWB = D * 2;         // bytes per row
    constexpr int PLANEB = TN * ROWB;   // one tile of K (or V)
    constexpr int STAGEB = 2 * PLANEB;
    constexpr int RPI = 64 / CPR;       // rows covered by one wave-wide 1 KiB DMA instruction
    constexpr int IPB = 16 / RPI;       // DMA instructions per 16-row block and plane
    constexpr int LPS = 2 * IPB;        // DMA instructions per wave and step
    constexpr int KSTEPS = D / 16;
    constexpr int DT = D / 32;
    constexpr int NSTAGE = NG * RING;
    static_assert(NSTAGE * STAGEB <= 160 * 1024, "LDS");
    __shared__ __attribute__((aligned(1024))) char smem[NSTAGE * STAGEB];

    // ---- work item: consecutive workgroup ids round-robin over the 8 XCDs, so the kv head
    // is taken from the low bits: all row tiles of one (request, kv head) stream share an L2
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
    // x / G for 0 <= x < 2^26 / G without an integer division (the host supplies ceil(2^32 / G), 0 for G = 1)
    const uint32_t g_magic = a.group_magic;
    auto div_g = [&](int x) { return g_magic ? (int)__umulhi((uint32_t)x, g_magic) : x; };
    const int N = it.new_len;
    const int rows_total = N * G;
    const int row0 = tile * TM;
    if (row0 >= rows_total) return;
    const int P = it.prefix_len;
    const int s0 = it.new_start;
    const int Hq = a.q_heads;
    const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = NG == 1 ? 0 : w >> 2, wq = w & 3;

    const __bf16* __restrict__ q = static_cast<const __bf16*>(a.q);
    const __bf16* __restrict__ k_new = static_cast<const __bf16*>(a.k_new);
    const __bf16* __restrict__ v_new = static_cast<const __bf16*>(a.v_new);
    const __bf16* __restrict__ pool_k = static_cast<const __bf16*>(a.b.pool_k);
    const __bf16* __restrict__ pool_v = static_cast<const __bf16*>(a.b.pool_v);
    const int32_t* __restrict__ table = a.b.block_table + (long long)r * a.b.table_stride;

    const int last_row = min(row0 + TM, rows_total) - 1;
    const int kv_limit = P + div_g(last_row) + 1;  // keys [0, kv_limit) are visible to some row of the item
    const int ntiles_all = (kv_limit + TN - 1) / TN;
    // key split across workgroups: copy `sidx` of S takes tiles [t_lo, ntiles)
    const int S = SPLIT ? wl.splits : 1, sidx = SPLIT ? item % S : 0;
    const int t_lo = ntiles_all * sidx / S;
    const int ntiles = ntiles_all * (sidx + 1) / S;  // exclusive end of this copy's tiles
    if (t_lo >= ntiles) return;                      // more copies than tiles: nothing for this one
    const int nsteps = (ntiles - t_lo + NG - 1) / NG;  // group `grp` takes tile t_lo + step*NG + grp

    // ---- this lane's query row
    const int wrow0 = row0 + (DEC ? 0 : wq * 32);
    const int ksub = DEC ? wq * 32 : 0;  // DEC: this wave's half of every tile (waves 2 and 3 only copy)
    const int my_row = min(wrow0 + l32, rows_total - 1);  // rows past the end repeat the last one
    const int my_tok = div_g(my_row);
    const int my_head = g * G + (my_row - my_tok * G);
    const int my_vis = P + my_tok + 1;  // keys [0, my_vis) are visible to this row
    const bool wave_active = wrow0 < rows_total && (!DEC || wq < 2);
    const int wave_vis_min = P + div_g(wrow0) + 1;
    const int wave_vis_max = P + div_g(min(wrow0 + 31, rows_total - 1)) + 1;

    // Block ids are fetched 64 steps at a time, one per lane (entry of step blk_base+lane), and
    // handed out with a lane read: no memory load sits on the issue path of a step.  The first
    // window is requested before Q so that both round trips overlap; it also covers the blocks of
    // this item's new tokens, which warms the table lines the fused append reads at the end.
    const int nblk_item = (kv_limit + 15) >> 4;
    int blk_base = 0;
    int blk_vec;
    {
        const int e = (min(t_lo + lane * NG + grp, ntiles - 1) * TN >> 4) + wq;
        blk_vec = e < nblk_item ? table[e] : 0;
    }
    bf16x8 qreg[KSTEPS];
    {
        const __bf16* qp = q + ((long long)(s0 + my_tok) * Hq + my_head) * D + hf * 8;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    }
    // Every ordinary load above completes here, before the DMA ring starts counting.  The
    // empty asm statements make the compiler itself wait for these registers now; otherwise it
    // would place its vmcnt waits at their first use inside the loop and drain the ring there.
    asm volatile("" ::"v"(blk_vec));
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) asm volatile("" ::"v"(qreg[ks]));
    wait_vmcnt<0>();

    // ---- DMA: wave (grp, wq) copies block wq (16 keys) of tile step*NG+grp, K and V planes.
    // Lane i of DMA instruction c brings row RPI*c + i/CPR of the block, 16-byte chunk
    // (i%CPR) ^ swz(row): the swizzle is applied on the global side, LDS is written linearly.
    uint32_t pool_loff[IPB], new_loff[IPB];  // byte offsets of this lane's chunk inside a pool block / a run of fresh rows
#pragma unroll
    for (int c = 0; c < IPB; ++c) {
        const int row16 = RPI * c + lane / CPR;
        const int chunk = (lane % CPR) ^ swz<D>(row16);
        pool_loff[c] = (row16 * D + chunk * 8) * 2;
        new_loff[c] = (row16 * Hkv * D + chunk * 8) * 2;
    }
    const uint32_t smem_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    // The copy of one step is prepared (addresses) right after the barrier and its DMA
    // instructions are then slipped between the MFMAs of S^T = K.Q^T, where their issue cost
    // hides under the matrix pipe; `flush` issues whatever is still pending at once.
    int pend = 0;              // 1: a fast-path copy (uniform base + per-lane constant) waits to be issued
    bool pend_fresh = false;   // source is the run of fresh rows, else one pool block
    uint64_t pend_kb = 0, pend_vb = 0;
    uint32_t pend_dst = 0;
    auto emit = [&](int c) {
        const uint32_t lo = pend_fresh ? new_loff[c] : pool_loff[c];
        dma_16B_per_lane(pend_kb, lo, pend_dst + RPI * c * ROWB);
        dma_16B_per_lane(pend_vb, lo, pend_dst + RPI * c * ROWB + PLANEB);
    };
    auto flush = [&]() {
        if (pend) {
#pragma unroll
            for (int c = 0; c < IPB; ++c) emit(c);
            pend = 0;
        }
    };
    auto prepare = [&](int step) {
        if (step - blk_base >= 64) {
            blk_base = step;
            const int e = (min(t_lo + (step + lane) * NG + grp, ntiles - 1) * TN >> 4) + wq;
            blk_vec = e < nblk_item ? table[e] : 0;
            asm volatile("" ::"v"(blk_vec));  // the compiler's wait for this load stays inside the branch
        }
        const int tg = min(t_lo + step * NG + grp, ntiles - 1);  // a group without a tile re-reads the last one (same count of loads)
        const int kbase = tg * TN + wq * 16;
        const int blk = __builtin_amdgcn_readlane(blk_vec, step - blk_base);
        const uint32_t dst = smem_addr + (grp * RING + step % RING) * STAGEB + wq * 16 * ROWB;
        if (kbase + 16 <= P) {
            // the whole block is cached: one pool block, uniform base + per-lane constant
            const long long boff = ((long long)blk * a.b.block_stride + (long long)g * kBlock * D) * 2;
            pend_kb = uniform_u64(reinterpret_cast<const char*>(pool_k) + boff);
            pend_vb = uniform_u64(reinterpret_cast<const char*>(pool_v) + boff);
            pend_dst = dst;
            pend_fresh = false;
            pend = 1;
        } else if (kbase >= P && kbase + 16 <= kv_limit) {
            // 16 fresh rows, all inside the horizon
            const long long boff = (((long long)(s0 + kbase - P)) * Hkv + g) * D * 2;
            pend_kb = uniform_u64(reinterpret_cast<const char*>(k_new) + boff);
            pend_vb = uniform_u64(reinterpret_cast<const char*>(v_new) + boff);
            pend_dst = dst;
            pend_fresh = true;
            pend = 1;
        } else {
            // the block straddles the prefix end or the horizon: choose the source per row, issue
            // now; rows past the horizon re-read the last visible one (they are masked later)
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
                const __bf16* ksrc = (kj < P ? pool_k : k_new) + off;
                const __bf16* vsrc = (kj < P ? pool_v : v_new) + off;
                dma_16B_per_lane(ksrc, dst + RPI * c * ROWB);
                dma_16B_per_lane(vsrc, dst + RPI * c * ROWB + PLANEB);
            }
            pend = 0;
        }
    };

    // ---- per-lane LDS read offsets (bytes); the stage and sub-tile parts are immediates
    typedef __attribute__((address_space(3))) char lds_char;
    lds_char* const lds0 = (lds_char*)smem;
    const int grp_off = grp * RING * STAGEB;  // folded into the per-lane offsets below
    // K, A operand of S^T: row sub*32+l32, chunk 2*ks+hf
    int koff[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
        koff[ks] = grp_off + (ksub + l32) * ROWB + (((2 * ks + hf) ^ swz<D>(l32)) << 4);
        asm volatile("" : "+v"(koff[ks]));  // keep it one register: address = this + immediate
    }
    // V, A operand of O^T (transposing read): rows kk*16 + 8*h2 + 4*hf + (lane&15)/4 + {sub*32},
    // 8 bytes at element dt*32 + 16*((lane>>4)&1) + 4*(lane&3)
    int voff[2][DT];
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const int row = 8 * h2 + 4 * hf + ((lane & 15) >> 2);
            const int elem = dt * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
            voff[h2][dt] = grp_off + (ksub + row) * ROWB + ((((elem >> 3)) ^ swz<D>(row)) << 4) + (elem & 7) * 2;
            asm volatile("" : "+v"(voff[h2][dt]));
        }

    f32x16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.f;
    float m_run = -INFINITY;  // reference exponent of O and l (log2 domain); at most 2^8 below the true row max
    float l_run = 0.f;        // this lane's partial of the running sum (other half in lane^32)
    const float c = a.scale_log2e;

    // one step with the ring slot as a compile-time constant
    auto do_step = [&](int step, auto slot_c) {
        constexpr int SLOT = decltype(slot_c)::value;
        // loads of this step have landed (later steps may stay in flight)
        if (RING > 2 && step + RING - 2 < nsteps) wait_vmcnt<(RING - 2) * LPS>();
        else wait_vmcnt<0>();
        block_barrier();  // every wave's part is in LDS, and every wave is done with the previous step
        if (step + RING - 1 < nsteps) prepare(step + RING - 1);

        const int tg = t_lo + step * NG + grp;
        const int base = tg * TN + ksub;  // first key this wave looks at
        if (!wave_active || tg >= ntiles || base >= wave_vis_max) {
            flush();
            return;
        }
        lds_char* const kst = lds0 + SLOT * STAGEB;
        lds_char* const vst = kst + PLANEB;

        // S^T = K Q^T
        f32x16 sacc[NSUB];
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[sub][i] = 0.f;
        // K operands are read two k-steps ahead of the MFMAs that consume them (LDS latency is
        // about four MFMAs long)
        bf16x8 kbuf[3][NSUB];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub)
                kbuf[ks][sub] = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(kst + sub * 32 * ROWB + koff[ks]);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            if (ks + 2 < KSTEPS) {
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub)
                    kbuf[(ks + 2) % 3][sub] = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(kst + sub * 32 * ROWB + koff[ks + 2]);
            }
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub)
                sacc[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kbuf[ks % 3][sub], qreg[ks], sacc[sub], 0, 0, 0);
            if (ks < IPB && pend) emit(ks);  // two DMA instructions in the shadow of the MFMAs just issued
        }
        pend = 0;
        // causal frontier / end of sequence: only tiles that reach past the first row's horizon
        if (base + NSUB * 32 > wave_vis_min) {
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int kidx = base + sub * 32 + (i >> 2) * 8 + hf * 4 + (i & 3);
                    if (kidx >= my_vis) sacc[sub][i] = -INFINITY;
                }
        }
        // online softmax, one row per lane pair (lane, lane^32)
        float mx = sacc[0][0];
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[sub][i]);
        mx = fmaxf(mx, other_half(mx));
        const float m_tile = mx * c;
        const bool raise = m_tile > m_run + kRescaleThreshold;  // true on a row's first visible tile (m_run = -inf)
        if (__builtin_amdgcn_ballot_w64(raise) != 0) {
            // 1 where nothing changes, 0 on a row's first visible tile (exp2(-inf))
            const float alpha = raise ? __builtin_amdgcn_exp2f(m_run - m_tile) : 1.f;
            m_run = raise ? m_tile : m_run;
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[dt][i] *= alpha;
        }
        // a row that has not seen a key yet (possible in the second wave group) has m_run = -inf
        // and only masked scores: subtract 0 instead, so that exp2(-inf - 0) = 0 and not NaN
        const float m_sub = m_run == -INFINITY ? 0.f : m_run;
        // The row sum is taken over the bf16-rounded probabilities, the same weights the PV
        // product uses, so that the rounding of P cancels between numerator and denominator.
        float psum = 0.f;
        bf16x8 pb[NSUB][2];
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const float p0 = __builtin_amdgcn_exp2f(sacc[sub][i] * c - m_sub);
                const float p1 = __builtin_amdgcn_exp2f(sacc[sub][i + 1] * c - m_sub);
                const bf16x2 pp = {(__bf16)p0, (__bf16)p1};
                psum = __builtin_amdgcn_fdot2_f32_bf16(pp, kOnes2, psum, false);
                pb[sub][i >> 3][i & 7] = pp[0];
                pb[sub][i >> 3][(i & 7) + 1] = pp[1];
            }
        l_run += psum;

        // O^T += V^T P^T ; V rows fetched with the transposing LDS read
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                lds_char* const vb = vst + (sub * 32 + kk * 16) * ROWB;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vb + voff[0][dt]));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vb + voff[1][dt]));
                    const bf16x4 lo_b = __builtin_bit_cast(bf16x4, lo);
                    const bf16x4 hi_b = __builtin_bit_cast(bf16x4, hi);
                    const bf16x8 va = __builtin_shufflevector(lo_b, hi_b, 0, 1, 2, 3, 4, 5, 6, 7);
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[sub][kk], oacc[dt], 0, 0, 0);
                }
            }
    };

#pragma unroll
    for (int s = 0; s < RING - 1; ++s)
        if (s < nsteps) {
            prepare(s);
            flush();
        }

    for (int step0 = 0; step0 < nsteps; step0 += RING) {
        do_step(step0, std::integral_constant<int, 0>{});
        if (step0 + 1 < nsteps) do_step(step0 + 1, std::integral_constant<int, 1>{});
        if (RING > 2) {
            if (step0 + 2 < nsteps) do_step(step0 + 2, std::integral_constant<int, 2 % RING>{});
            if (step0 + 3 < nsteps) do_step(step0 + 3, std::integral_constant<int, 3 % RING>{});
        }
    }

    // ---- fused append (after the key loop: nothing waits for it, and the fresh rows are L2-hot
    // because the loop has just read them as keys; requested up front, next to Q, the rows cost 1-4 %
    // on the prefill configurations and gain 1-2 % on decode steps).  This work item owns the tokens
    // whose first row (head 0 of the group) it holds; 16-byte chunks, four per thread in flight.
    if (a.fused_append && sidx == S - 1) {  // the last copy always has tiles
        const int tok_lo = div_g(row0 + G - 1);
        const int tok_hi = min(N - 1, div_g(row0 + TM - 1));
        __bf16* wk = static_cast<__bf16*>(a.pool_k_w);
        __bf16* wv = static_cast<__bf16*>(a.pool_v_w);
        const int n = (tok_hi - tok_lo + 1) * CPR;
        constexpr int UNR = 4;
        for (int i0 = tid; i0 < n; i0 += (256 * NG) * UNR) {
            int blk[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int idx = min(i0 + u * (256 * NG), n - 1);
                blk[u] = table[(P + tok_lo + idx / CPR) >> 4];
            }
            u32x4 kk[UNR], vv[UNR];
            long long dst[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int idx = min(i0 + u * (256 * NG), n - 1);
                const int tok = tok_lo + idx / CPR, ch = idx % CPR;
                const int pos = P + tok;
                const long long src = ((long long)(s0 + tok) * Hkv + g) * D + ch * 8;
                dst[u] = (long long)blk[u] * a.b.block_stride + ((long long)g * kBlock + (pos & 15)) * D + ch * 8;
                kk[u] = *reinterpret_cast<const u32x4*>(k_new + src);
                vv[u] = *reinterpret_cast<const u32x4*>(v_new + src);
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                if (i0 + u * (256 * NG) < n) {
                    *reinterpret_cast<u32x4*>(wk + dst[u]) = kk[u];
                    *reinterpret_cast<u32x4*>(wv + dst[u]) = vv[u];
                }
            }
        }
    }

    // ---- merge the wave groups through LDS (the DMA ring is idle now)
    constexpr int WSTRIDE = (DT * 16 + 4) * 64;  // floats per wave in the merge area: [DT*4 + 1 chunks][64 lanes][4]
    if (DEC) {
        // up to 2 * NG waves hold a state for the same 32 rows: wave (grp, wq < 2) is participant
        // p = 2 * grp + wq; everyone but participant 0 leaves its state in area p, participant 0 adds
        // them up one after the other and goes on alone
        static_assert(2 * NG * WSTRIDE * 4 <= NSTAGE * STAGEB, "merge areas fit the ring");
        typedef __attribute__((address_space(3))) f32x4 lds_f32x4;
        const int part_id = 2 * grp + wq;
        block_barrier();
        if (wq < 2 && part_id != 0) {
            lds_f32x4* const xw = reinterpret_cast<lds_f32x4*>(lds0 + part_id * (WSTRIDE * 4)) + lane;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const f32x4 v = {oacc[dt][i4 * 4], oacc[dt][i4 * 4 + 1], oacc[dt][i4 * 4 + 2], oacc[dt][i4 * 4 + 3]};
                    xw[(dt * 4 + i4) * 64] = v;
                }
            const f32x4 ml = {m_run, l_run, 0.f, 0.f};
            xw[DT * 4 * 64] = ml;
        }
        block_barrier();
        if (w != 0) return;
#pragma unroll 1
        for (int other = 1; other < 2 * NG; ++other) {
            lds_f32x4* const xw = reinterpret_cast<lds_f32x4*>(lds0 + other * (WSTRIDE * 4)) + lane;
            const f32x4 ml = xw[DT * 4 * 64];
            const float m1 = ml[0], l1 = ml[1];
            // a participant (or, with a key split, all of them) may have seen no visible key of a row: weight 0
            const float m = fmaxf(m_run, m1);
            const float s0f = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run - m);
            const float s1f = m1 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m1 - m);
            m_run = m;
            l_run = l_run * s0f + l1 * s1f;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const f32x4 v = xw[(dt * 4 + i4) * 64];
#pragma unroll
                    for (int e = 0; e < 4; ++e) oacc[dt][i4 * 4 + e] = oacc[dt][i4 * 4 + e] * s0f + v[e] * s1f;
                }
        }
    } else if (NG > 1) {
        typedef __attribute__((address_space(3))) f32x4 lds_f32x4;
        lds_f32x4* const xw = reinterpret_cast<lds_f32x4*>(lds0 + wq * (WSTRIDE * 4)) + lane;
        block_barrier();
        if (grp == 1) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const f32x4 v = {oacc[dt][i4 * 4], oacc[dt][i4 * 4 + 1], oacc[dt][i4 * 4 + 2], oacc[dt][i4 * 4 + 3]};
                    xw[(dt * 4 + i4) * 64] = v;
                }
            const f32x4 ml = {m_run, l_run, 0.f, 0.f};
            xw[DT * 4 * 64] = ml;
        }
        block_barrier();
        if (grp == 1) return;
        if (wave_active) {
            const f32x4 ml = xw[DT * 4 * 64];
            const float m1 = ml[0], l1 = ml[1];
            // a group (or, with a key split, both) may have seen no visible key of a row: weight 0
            const float m = fmaxf(m_run, m1);
            const float s0f = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run - m);
            const float s1f = m1 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m1 - m);
            m_run = m;
            l_run = l_run * s0f + l1 * s1f;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const f32x4 v = xw[(dt * 4 + i4) * 64];
#pragma unroll
                    for (int e = 0; e < 4; ++e) oacc[dt][i4 * 4 + e] = oacc[dt][i4 * 4 + e] * s0f + v[e] * s1f;
                }
        }
    } else {
        block_barrier();  // every wave is done with the ring: its memory is reused below
    }

    // ---- normalise and store.  A lane holds 4 consecutive d of ONE row per (dt, i/4), so a direct
    // store would touch 32 rows with 16 bytes each per instruction; instead the wave turns its 32
    // rows around in a private LDS patch (rows padded by 16 bytes) and stores whole rows, 16 bytes
    // per lane.  With two groups the patch is the wave's own merge area, which only it reads.
    if (!wave_active) return;
    constexpr int OROWB = ROWB + 16;
    static_assert(32 * OROWB <= WSTRIDE * 4, "output patch fits the merge area");
    lds_char* const patch = lds0 + wq * (NG > 1 ? WSTRIDE * 4 : 32 * OROWB);  // DEC: wave 0 only, area 0 holds no state
    const float l_tot = l_run + other_half(l_run);
    if (SPLIT) {
        // ---- one of S copies of the item: leave O (unnormalised, fp32), max and sum of every row in the
        // workspace; partial (item, copy, kv head) = [TM][D] floats of O, then [TM][2] floats (max, sum).
        // Same turn through LDS as below, in two passes of D/2 floats per row.
        float* const part = static_cast<float*>(a.partial) + ((long long)(wl.part_base + item) * Hkv + g) * (TM * (D + 2));
        const int prow = wq * 32;
        if (hf == 0) {
            const float2 ml = {m_run, l_tot};
            *reinterpret_cast<float2*>(part + TM * D + (prow + l32) * 2) = ml;
        }
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
            for (int dtl = 0; dtl < DT / 2; ++dtl)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const int dt = pass * (DT / 2) + dtl;
                    const f32x4 v = {oacc[dt][i4 * 4], oacc[dt][i4 * 4 + 1], oacc[dt][i4 * 4 + 2], oacc[dt][i4 * 4 + 3]};
                    *reinterpret_cast<__attribute__((address_space(3))) f32x4*>(patch + l32 * OROWB + (dtl * 32 + i4 * 8 + hf * 4) * 4) = v;
                }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int p = 0; p < 32 / RPI; ++p) {
                const int rr = p * RPI + lane / CPR;
                const f32x4 v = *reinterpret_cast<const __attribute__((address_space(3))) f32x4*>(patch + rr * OROWB + (lane % CPR) * 16);
                *reinterpret_cast<f32x4*>(part + (prow + rr) * D + pass * (D / 2) + (lane % CPR) * 4) = v;
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the patch is rewritten by the next pass
        }
        return;
    }
    const float inv = 1.f / l_tot;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            bf16x4 o4;
#pragma unroll
            for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[dt][i4 * 4 + e] * inv);
            *reinterpret_cast<__attribute__((address_space(3))) bf16x4*>(patch + l32 * OROWB + (dt * 32 + i4 * 8 + hf * 4) * 2) = o4;
        }
    // lanes now read what other lanes of the same wave wrote: LDS operations of a wave complete in order
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __bf16* const outp = static_cast<__bf16*>(a.out);
#pragma unroll
    for (int p = 0; p < 32 / RPI; ++p) {
        const int rr = p * RPI + lane / CPR;
        const int row = wrow0 + rr;
        const u32x4 v = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(patch + rr * OROWB + (lane % CPR) * 16);
        if (row < rows_total) {
            const int tok = div_g(row);
            const int head = g * G + (row - tok * G);
            *reinterpret_cast<u32x4*>(outp + ((long long)(s0 + tok) * Hq + head) * D + (lane % CPR) * 8) = v;
        }
    }
}

// Combines the S partial results of every row of a split work item (see the end of
// attn_bf16_kernel for the layout): out = sum_s O_s 2^(m_s - m) / sum_s l_s 2^(m_s - m), m = max_s m_s.
// The list holds one entry per split item (its copy 0); one workgroup per (entry, kv head, run of
// 256 / (D/4) rows): 4 consecutive d of one row per thread.
template <int D>
__global__ __launch_bounds__(256) void attn_bf16_merge_kernel(AttnLaunch a, AttnWorkList wl) {
    constexpr int TPR = D / 4;          // threads per row
    constexpr int RPW = 256 / TPR;      // rows per workgroup
    constexpr int CHUNKS = TM / RPW;    // workgroups per (entry, kv head)
    const int Hkv = a.b.kv_heads;
    const int chunk = blockIdx.x % CHUNKS;
    const int g = (blockIdx.x / CHUNKS) % Hkv;
    const int lead = blockIdx.x / (CHUNKS * Hkv);  // the list holds copy 0 of every split item, in launch order
    const AttnItem it = wl.item[lead];
    const int S = wl.splits;
    const int G = a.group;
    const uint32_t g_magic = a.group_magic;
    auto div_g = [&](int x) { return g_magic ? (int)__umulhi((uint32_t)x, g_magic) : x; };
    const int rows_total = it.new_len * G;
    const int row0 = (it.req_tile & 0xffff) * TM;
    const int rows_here = min(TM, rows_total - row0);
    const int kv_limit = it.prefix_len + div_g(row0 + rows_here - 1) + 1;
    const int ntiles_all = (kv_limit + TN - 1) / TN;
    constexpr int PART = TM * (D + 2);
    const float* const part0 = static_cast<const float*>(a.partial) + ((long long)(wl.part_base + lead * S) * Hkv + g) * PART;
    const long long copy_stride = (long long)Hkv * PART;
    const int d4 = threadIdx.x % TPR;
    __bf16* const outp = static_cast<__bf16*>(a.out);
    const int r = chunk * RPW + threadIdx.x / TPR;
    if (r < rows_here) {
        // one round trip: every copy's (max, sum) and O piece are requested before any is used
        float mc[kAttnMaxSplits], lc[kAttnMaxSplits];
        f32x4 oc[kAttnMaxSplits];
#pragma unroll
        for (int c = 0; c < kAttnMaxSplits; ++c) {
            mc[c] = -INFINITY;  // a copy that does not exist, or had no tiles and wrote nothing, weighs 0
            lc[c] = 0.f;
            oc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (c < S && ntiles_all * c / S < ntiles_all * (c + 1) / S) {
                const float* pc = part0 + c * copy_stride;
                const float2 ml = *reinterpret_cast<const float2*>(pc + TM * D + r * 2);
                mc[c] = ml.x;
                lc[c] = ml.y;
                oc[c] = *reinterpret_cast<const f32x4*>(pc + r * D + d4 * 4);
            }
        }
        float m = -INFINITY;
#pragma unroll
        for (int c = 0; c < kAttnMaxSplits; ++c) m = fmaxf(m, mc[c]);
        float l = 0.f;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < kAttnMaxSplits; ++c) {
            const float wgt = mc[c] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mc[c] - m);  // a copy may hold no visible key of the row
            l += lc[c] * wgt;
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] += oc[c][e] * wgt;
        }
        const float inv = 1.f / l;
        const int row = row0 + r;
        const int tok = div_g(row);
        const int head = g * G + (row - tok * G);
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(acc[e] * inv);
        *reinterpret_cast<bf16x4*>(outp + ((long long)(it.new_start + tok) * a.q_heads + head) * D + d4 * 4) = o4;
    }
}

template <int D, int NG, int RING, bool DEC>
void launch_dec(const AttnLaunch& a, const AttnWorkList& wl, hipStream_t s) {
    if (wl.splits > 1)
        hipLaunchKernelGGL((attn_bf16_kernel<D, NG, RING, true, DEC>), dim3(wl.n * a.b.kv_heads), dim3(256 * NG), 0, s, a, wl);
    else
        hipLaunchKernelGGL((attn_bf16_kernel<D, NG, RING, false, DEC>), dim3(wl.n * a.b.kv_heads), dim3(256 * NG), 0, s, a, wl);
}
template <int D, int NG, int RING>
void launch_one(const AttnLaunch& a, const AttnWorkList& wl, hipStream_t s) {
    if (a.max_new * a.group <= 32) launch_dec<D, NG, RING, true>(a, wl, s);  // every item has at most 32 rows
    else launch_dec<D, NG, RING, false>(a, wl, s);
}

}  // namespace

int attn_bf16_item_cost(int prefix, int new_len, int group, int tile) {
    const int rows = new_len * group;
    const int last_row = (tile + 1) * TM < rows ? (tile + 1) * TM - 1 : rows - 1;
    return (prefix + last_row / group + 1 + TN - 1) / TN;
}

hipError_t launch_attn_bf16(const AttnLaunch& a, const AttnWorkList& wl, int variant, hipStream_t s) {
    if (wl.n <= 0) return hipSuccess;
    const bool d64 = a.b.head_dim == 64;
    if (variant == kAttnVariantTwoGroups)
        d64 ? launch_one<64, 2, 2>(a, wl, s) : launch_one<128, 2, 2>(a, wl, s);
    else
        d64 ? launch_one<64, 1, 2>(a, wl, s) : launch_one<128, 1, 2>(a, wl, s);
    return hipGetLastError();
}

hipError_t launch_attn_bf16_merge(const AttnLaunch& a, const AttnWorkList& wl, hipStream_t s) {
    if (wl.n <= 0) return hipSuccess;
    if (a.b.head_dim == 64)
        hipLaunchKernelGGL((attn_bf16_merge_kernel<64>), dim3(wl.n * a.b.kv_heads * (TM / 16)), dim3(256), 0, s, a, wl);
    else
        hipLaunchKernelGGL((attn_bf16_merge_kernel<128>), dim3(wl.n * a.b.kv_heads * (TM / 8)), dim3(256), 0, s, a, wl);
    return hipGetLastError();
}

}  // namespace ragc
