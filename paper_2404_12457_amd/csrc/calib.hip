// Calibration kernels for the benchmark: what this GPU sustains on the two resources the
// roofline fractions are quoted against, measured with plain kernels that do nothing else.
// Built into libragc_calib.so (not part of libragc.so; the product path never calls them).
//
//   ragc_calib_mfma   register-only loop of v_mfma_f32_32x32x16_bf16 with operands read once
//                     from a caller-filled buffer (random values: the matrix cores draw more
//                     power, and clock lower, on random operands than on constants)
//   ragc_calib_copy   streaming device-to-device copy, 16 bytes per lane
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kChains = 4;        // independent accumulators per wave

// Every wave: load 2 A and 2 B operands (16 bytes per lane each), run iters * 8 MFMAs on 4
// independent accumulators, store one value so nothing is dead.  Lane 0 of every wave also
// records the shader-clock and constant-clock counters around the loop.
__global__ __launch_bounds__(256, 2) void mfma_loop(const bf16x8* __restrict__ operands, float* __restrict__ sink,
                                                    int64_t* __restrict__ clocks, int iters) {
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const bf16x8* op = operands + (size_t)(wave & 63) * 256;  // 64 distinct operand sets of 4 KiB
    const bf16x8 a0 = op[lane], a1 = op[64 + lane], b0 = op[128 + lane], b1 = op[192 + lane];
    f32x16 acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
    const int64_t t0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[c], 0, 0, 0);
#pragma unroll
        for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[c], 0, 0, 0);
    }
    const int64_t t1 = clock64(), w1 = wall_clock64();
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[c][i];
    sink[(size_t)wave * 64 + lane] = s;
    if (lane == 0) {
        clocks[2 * wave] = t1 - t0;
        clocks[2 * wave + 1] = w1 - w0;
    }
}

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__global__ __launch_bounds__(256) void copy_stream(u32x4* __restrict__ dst, const u32x4* __restrict__ src, int64_t n16) {
    // each workgroup owns a contiguous run of 4 x 256 chunks per trip, four loads in flight per lane
    const int64_t stride = (int64_t)gridDim.x * 1024;
    for (int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x; base < n16; base += stride) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (base + u * 256 < n16) v[u] = __builtin_nontemporal_load(src + base + u * 256);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (base + u * 256 < n16) __builtin_nontemporal_store(v[u], dst + base + u * 256);
    }
}

}  // namespace

extern "C" {

// operands [device]: at least 64 * 4096 bytes of bf16 values; sink [device]: waves * 64 floats;
// clocks [device]: waves * 2 int64 (shader-clock ticks, 100 MHz ticks).  waves = workgroups * 4.
// Returns the hipError_t of the launch as an int.  Flops done = workgroups * 4 * iters * 8 * 32768.
int ragc_calib_mfma(const void* operands, void* sink, void* clocks, int32_t workgroups, int32_t iters, void* stream) {
    if (!operands || !sink || !clocks || workgroups <= 0 || iters <= 0) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(mfma_loop, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const bf16x8*>(operands), static_cast<float*>(sink), static_cast<int64_t*>(clocks), iters);
    return (int)hipGetLastError();
}

// dst, src [device], 16-byte aligned, bytes a multiple of 16.
int ragc_calib_copy(void* dst, const void* src, int64_t bytes, int32_t workgroups, void* stream) {
    if (!dst || !src || bytes <= 0 || (bytes & 15) || workgroups <= 0) return (int)hipErrorInvalidValue;
    if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15u) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(copy_stream, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<u32x4*>(dst), static_cast<const u32x4*>(src), bytes / 16);
    return (int)hipGetLastError();
}

}  // extern "C"
