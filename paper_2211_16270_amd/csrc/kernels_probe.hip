// Measurement support: a loop of nothing but 32x32x16 bf16 (or 32x32x64 fp8) MFMAs on operand fragments the caller chooses.
// The rate this loop reaches depends on the operand values (the chip lowers its clock under its power limit),
// which is what the MFMA-bound kernels of this library can be compared with besides the published peak.
#include "device_common.h"
#include "kernels.h"

namespace rnnt {

namespace {

// 256 threads = 4 waves, one per SIMD; every wave holds 4 A and 4 B fragments in registers (taken from
// frags [32][64 lanes] x 16 bytes: wave w uses fragments 8w .. 8w+7) and multiplies them into 16
// accumulator tiles, iters times: 16 MFMAs per iteration, no memory access inside the loop.
__global__ __launch_bounds__(256) void k_mfma_loop(const bf16x8* __restrict__ frags, float* __restrict__ out, int iters) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = frags[(wave * 8 + i) * 64 + lane];
        b[i] = frags[(wave * 8 + 4 + i) * 64 + lane];
    }
    f32x16 c[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) c[i] = f32x16{0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int n = 0; n < 4; ++n)
                c[m * 4 + n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m], b[n], c[m * 4 + n], 0, 0, 0);
    }
    float r = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) r += c[i][0] + c[i][5];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = r;
}

// The same loop on the fp8 (e4m3) MFMA of gfx950, 32x32x64 with unit scales: fragments of 64 lanes x 32 bytes.
typedef int i32x8 __attribute__((ext_vector_type(8)));
__global__ __launch_bounds__(256) void k_mfma_loop_fp8(const i32x8* __restrict__ frags, float* __restrict__ out, int iters) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    i32x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = frags[(wave * 8 + i) * 64 + lane];
        b[i] = frags[(wave * 8 + 4 + i) * 64 + lane];
    }
    f32x16 c[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) c[i] = f32x16{0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int n = 0; n < 4; ++n)
                c[m * 4 + n] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[m], b[n], c[m * 4 + n], 0, 0, 0, 0, 0, 0);
    }
    float r = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) r += c[i][0] + c[i][5];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = r;
}

}  // namespace

hipError_t launch_mfma_loop_fp8(const void* frags, float* out, int workgroups, int iters, hipStream_t stream) {
    k_mfma_loop_fp8<<<dim3((unsigned)workgroups), dim3(256), 0, stream>>>((const i32x8*)frags, out, iters);
    return hipGetLastError();
}

hipError_t launch_mfma_loop(const void* frags, float* out, int workgroups, int iters, hipStream_t stream) {
    k_mfma_loop<<<dim3((unsigned)workgroups), dim3(256), 0, stream>>>((const bf16x8*)frags, out, iters);
    return hipGetLastError();
}

}  // namespace rnnt
