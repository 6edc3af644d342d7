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

// Every workgroup reads the same n16 16-byte pieces `iters` times, 16 bytes per lane and 1 KB per wave instruction,
// eight instructions in flight per wave (the way the score kernels stream their W_out fragments, which all
// workgroups share): what the path from the L2 (or, for a larger array, from the last-level cache or HBM) to the
// compute units delivers when every compute unit pulls at once.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void k_stream_read(const u32x4* __restrict__ src, size_t n16, int iters,
                                                     u32x4* __restrict__ out) {
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int it = 0; it < iters; ++it) {
        const u32x4* p = src + threadIdx.x;
        asm volatile("" : "+v"(p));              // a new pointer as far as the compiler knows: the loads stay in the loop
        for (size_t i = 0; i < n16; i += 8 * 256) {
            u32x4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = p[i + j * 256];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc ^= v[j];
        }
    }
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = acc;
}

}  // namespace

hipError_t launch_stream_read(const void* src, size_t bytes, void* out, int workgroups, int iters, hipStream_t stream) {
    k_stream_read<<<dim3((unsigned)workgroups), dim3(256), 0, stream>>>((const u32x4*)src, bytes / 16, iters, (u32x4*)out);
    return hipGetLastError();
}

hipError_t launch_mfma_loop_fp8(const void* frags, float* out, int workgroups, int iters, hipStream_t stream) {
    k_mfma_loop_fp8<<<dim3((unsigned)workgroups), dim3(256), 0, stream>>>((const i32x8*)frags, out, iters);
    return hipGetLastError();
}

hipError_t launch_mfma_loop(const void* frags, float* out, int workgroups, int iters, hipStream_t stream) {
    k_mfma_loop<<<dim3((unsigned)workgroups), dim3(256), 0, stream>>>((const bf16x8*)frags, out, iters);
    return hipGetLastError();
}

}  // namespace rnnt
