// Device helpers shared by the bf16 attention kernels (gfx950 only).
#pragma once
#include <type_traits>

#include "ragc_internal.h"

namespace ragc {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int TN = 64;                    // keys per LDS tile
constexpr float kRescaleThreshold = 8.f;  // log2 units
constexpr bf16x2 kOnes2 = {(__bf16)1.0f, (__bf16)1.0f};

// Wave-wide copy of 64 x 16 bytes from global memory straight into LDS: lane i's 16 bytes
// land at lds_addr + 16*i.  Issued as inline assembly on purpose: the compiler's own
// bookkeeping for this instruction drains every outstanding load before the next LDS read,
// which would serialise the ring; the waits are placed by hand (wait_vmcnt + block_barrier).
// The s_nop is required: the LDS address travels in M0, and a scalar write of M0 needs one wait
// state before an LDS-DMA instruction reads it (inside inline assembly nobody inserts it for us;
// without it the copy can land at the previous instruction's LDS address).
__device__ __forceinline__ void dma_16B_per_lane(const void* gptr, uint32_t lds_addr) {
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);  // wave-uniform by construction; make the register class explicit
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory", "m0");
}
// same with a wave-uniform base address and a 32-bit per-lane byte offset
__device__ __forceinline__ void dma_16B_per_lane(uint64_t sbase, uint32_t lane_off, uint32_t lds_addr) {
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
    // a scalar register pair whatever the compiler knows or does not know about the value
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)sbase), hi = __builtin_amdgcn_readfirstlane((uint32_t)(sbase >> 32));
    asm volatile("" : "+s"(lo), "+s"(hi));
    sbase = ((uint64_t)hi << 32) | lo;
    // No "memory" clobber: the slot this copy writes is not read before the next barrier (which has
    // one), and without it the compiler may move the LDS reads of the current tile across the copy.
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(lane_off), "s"(sbase) : "m0");
}
__device__ __forceinline__ uint64_t uniform_u64(const void* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ float other_half(float x) {
    // value held by lane ^ 32
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

// XOR pattern applied to the 16-byte chunk index of row `row` (depends on row & 15).
template <int D>
__device__ __forceinline__ int swz(int row) {
    if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
    return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
}

// wait until at most N vector-memory operations of this wave are outstanding
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ void block_barrier() {
    // hardware barrier without the fence of __syncthreads(): outstanding LDS-DMA loads of
    // later tiles must stay in flight across it
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}


}  // namespace
}  // namespace ragc
