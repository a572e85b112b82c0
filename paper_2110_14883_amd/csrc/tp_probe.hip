// Measurement aid for bench.py, NOT part of libtplinear: a register-resident loop of dense bf16
// MFMAs (no LDS, no memory traffic, operands with random-looking bits) on every compute unit.  Timed
// by the caller it gives the dense-bf16 rate the chip sustains at the clock it holds under load, to
// set beside the published 2.5 PFLOP/s.  Built into libtpprobe.so; declared in include/tp_probe.h.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tp_probe.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

__global__ __launch_bounds__(256) void tp_mfma_probe_kernel(float* out, int iters, uint32_t seed) {
    u32x4_t a0, b0;
    uint32_t x = seed ^ (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x = x * 1664525u + 1013904223u; a0[i] = (x & 0x807f807fu) | 0x3f003f00u;     // bf16 pairs in [0.5, 1) with random sign/mantissa
        x = x * 1664525u + 1013904223u; b0[i] = (x & 0x807f807fu) | 0x3c003c00u;
    }
    const bf16x8_t a = __builtin_bit_cast(bf16x8_t, a0), b = __builtin_bit_cast(bf16x8_t, b0);
    f32x16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

constexpr int kWorkgroups = 256;

}  // namespace

extern "C" int tp_mfma_probe(void* scratch, size_t scratch_bytes, int iters, double* flops, void* hip_stream) {
    if (!scratch || !flops) return 1;
    if (iters < 1) return 4;
    if (scratch_bytes < (size_t)kWorkgroups * 256 * sizeof(float) || (reinterpret_cast<uintptr_t>(scratch) & 15u)) return 7;
    // 256 workgroups x 4 waves x iters x 8 MFMAs of 32x32x16 (32768 flops each)
    *flops = (double)kWorkgroups * 4.0 * (double)iters * 8.0 * 32768.0;
    float* out = static_cast<float*>(scratch);
    uint32_t seed = 0x9E3779B9u;
    void* args[] = {&out, &iters, &seed};
    return hipLaunchKernel(reinterpret_cast<const void*>(&tp_mfma_probe_kernel), dim3(kWorkgroups), dim3(256), args, 0,
                           static_cast<hipStream_t>(hip_stream)) == hipSuccess ? 0 : 8;
}
