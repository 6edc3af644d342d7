// Set-up work of one call in a single launch: clears the gradient outputs, writes the tile -> sample
// table and the two fragment-major copies of W_out.  Each workgroup reads its job from its index.
#include "device_common.h"
#include "kernels.h"

namespace rnnt {

namespace {
struct PrepKernelArgs {
    PrepArgs a;
    unsigned zero_end[4];   // cumulative workgroup counts: clear region r is [zero_end[r-1], zero_end[r])
    unsigned ts_end;        // tile -> sample table: one workgroup per sample
    unsigned wp_end;        // W_out^T fragments for the score GEMM
    unsigned wq_end;        // W_out fragments for the dz GEMM
};
}  // namespace

__global__ __launch_bounds__(256) void k_prepare(PrepKernelArgs k) {
    const unsigned b = blockIdx.x;
    const int tid = threadIdx.x;
    if (b < k.zero_end[3]) {
        int r = 0;
        unsigned first = 0;
#pragma unroll
        for (int i = 0; i < 3; ++i)
            if (b >= k.zero_end[i]) { r = i + 1; first = k.zero_end[i]; }
        float* __restrict__ p = k.a.zero_ptr[r];
        const size_t n = k.a.zero_n[r];
        const size_t stride = (size_t)(k.zero_end[r] - first) * 256;
        for (size_t i = (size_t)(b - first) * 256 + tid; i < n; i += stride) p[i] = 0.0f;
    } else if (b < k.ts_end) {
        const int s = (int)(b - k.zero_end[3]);
        const int e = k.a.tile_off[s + 1];
        for (int i = k.a.tile_off[s] + tid; i < e; i += 256) k.a.tile_sample[i] = s;
    } else if (b < k.wp_end) {
        // Wp[((vt*KK + kk)*64 + lane)*8 + j] = W[kk*16 + 8*(lane/32) + j][vt*32 + lane%32]:
        // one A fragment of the score GEMM is a contiguous 1 KiB block
        const int H = k.a.H, V = k.a.V, KK = H >> 4;
        const long long g = (long long)(b - k.ts_end) * 256 + tid;
        if (g >= (long long)(V >> 5) * KK * 64) return;
        const int lane = (int)(g & 63);
        const long long f = g >> 6;
        const int kk = (int)(f % KK), vt = (int)(f / KK);
        const int v = vt * 32 + (lane & 31);
        const int k0 = kk * 16 + 8 * (lane >> 5);
        const bf16_t* __restrict__ W = (const bf16_t*)k.a.W;
        bf16x8 o;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = W[(size_t)(k0 + j) * V + v];
        *reinterpret_cast<bf16x8*>((bf16_t*)k.a.Wp + g * 8) = o;
    } else {
        // Wq[((ht*(V/16) + vk)*64 + lane)*8 + j] = W[ht*32 + lane%32][vk*16 + 8*(lane/32) + j]
        const int H = k.a.H, V = k.a.V, VK = V >> 4;
        const long long g = (long long)(b - k.wp_end) * 256 + tid;
        if (g >= (long long)(H >> 5) * VK * 64) return;
        const int lane = (int)(g & 63);
        const long long f = g >> 6;
        const int vk = (int)(f % VK), ht = (int)(f / VK);
        const bf16_t* src = (const bf16_t*)k.a.W + (size_t)(ht * 32 + (lane & 31)) * V + vk * 16 + 8 * (lane >> 5);
        *reinterpret_cast<bf16x8*>((bf16_t*)k.a.Wq + g * 8) = *reinterpret_cast<const bf16x8*>(src);
    }
}

// dst[i] = bf16(src[i]) (round to nearest even), n a multiple of 8
__global__ __launch_bounds__(256) void k_f32_to_bf16(const float* __restrict__ src, bf16_t* __restrict__ dst, size_t n8) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += stride) {
        const f32x4 lo = *reinterpret_cast<const f32x4*>(src + i * 8);
        const f32x4 hi = *reinterpret_cast<const f32x4*>(src + i * 8 + 4);
        bf16x8 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            o[j] = (bf16_t)lo[j];
            o[4 + j] = (bf16_t)hi[j];
        }
        *reinterpret_cast<bf16x8*>(dst + i * 8) = o;
    }
}

hipError_t launch_f32_to_bf16(const float* src, void* dst, size_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    if (n % 8 != 0) return hipErrorInvalidValue;
    const size_t n8 = n / 8;
    const size_t blocks = (n8 + 255) / 256;
    k_f32_to_bf16<<<dim3((unsigned)(blocks > 16384 ? 16384 : blocks)), dim3(256), 0, stream>>>(src, (bf16_t*)dst, n8);
    return hipGetLastError();
}

hipError_t launch_prepare(const PrepArgs& a, hipStream_t stream) {
    PrepKernelArgs k{};
    k.a = a;
    unsigned end = 0;
    for (int r = 0; r < 4; ++r) {
        if (a.zero_ptr[r] != nullptr && a.zero_n[r] > 0) {
            size_t blocks = (a.zero_n[r] + 2047) / 2048;
            end += (unsigned)(blocks > 8192 ? 8192 : blocks);
        }
        k.zero_end[r] = end;
    }
    if (a.tile_sample != nullptr) end += (unsigned)a.B;
    k.ts_end = end;
    if (a.Wp != nullptr) end += (unsigned)(((long long)(a.V / 32) * (a.H / 16) * 64 + 255) / 256);
    k.wp_end = end;
    if (a.Wq != nullptr) end += (unsigned)(((long long)(a.H / 32) * (a.V / 16) * 64 + 255) / 256);
    k.wq_end = end;
    if (end == 0) return hipSuccess;
    k_prepare<<<dim3(end), dim3(256), 0, stream>>>(k);
    return hipGetLastError();
}

}  // namespace rnnt
