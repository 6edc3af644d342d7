// The two linear maps inside the tanh of the joint network (Eq. 4): enc = hA W_A + b_Z, pred = hL W_L,
// and their backward (Algorithm 1 line 9 for W_A, b_Z, W_L; lines 10-11 continued to hA, hL).
//
// All of them are one GEMM shape family  C[m,n] (+)= sum_k A(m,k) B(k,n)  over row-major arrays whose
// operands differ only in which index is contiguous in memory:
//   forward      enc[r,h]   = sum_k hA[r,k]   W_A[k,h] + b_Z[h]     A k-contiguous, B k-slow
//   d input      d_hA[r,k]  = sum_h d_enc[r,h] W_A[k,h]             A k-contiguous, B k-contiguous
//   d weights    dW_A[k,h] += sum_r hA[r,k]   d_enc[r,h]            A k-slow, B k-slow (split over r)
// Rows r = b*T_max + t beyond a sample's length are padding: their input may hold anything (NaN
// included) and is read as zero.
//
// bf16 path: 128x128 output tile per workgroup, 4 waves x (64x64 = 2x2 MFMA 32x32x16 tiles), K-step 64.
// A k-contiguous operand lies in LDS as [row][k] and gives fragments by plain 16-byte reads; a k-slow
// operand lies there as in memory ([k][row], 16-byte chunks XOR-swizzled) and gives fragments by the
// transposing LDS read.  Global loads run one K-step ahead in registers.  These GEMMs are about 1 % of the path's flops.
// fp32 path: the fp32 MFMA tile GEMM of the fp32 joint path where rows are 16-byte aligned (D, H multiples of 4);
// else one thread per output element.
#include "device_common.h"
#include "kernels.h"

namespace rnnt {

namespace {

constexpr int PT = 128;        // output tile edge
constexpr int PK = 64;         // K-step
constexpr int PP = PK + 8;     // LDS row pitch (bf16 elements): 272 bytes, conflict-free 16-byte reads
constexpr int PQ = PT * PK / 8 / 256;   // 16-byte chunks per thread, operand and step
constexpr int PD = 1;          // K-steps the global loads run ahead

// source row s is real data iff there is no mask or (s % period) < len[s / period] + extra
__device__ __forceinline__ bool row_is_data(const RowMask& m, long long s) {
    if (m.len == nullptr) return true;
    const long long b = s / m.period;
    return (int)(s - b * m.period) < m.len[b] + m.extra;
}

__device__ __forceinline__ bf16x8 load8(const bf16_t* p) { return *reinterpret_cast<const bf16x8*>(p); }
__device__ __forceinline__ bf16x8 load8(const float* p) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 4; ++j) { r[j] = (bf16_t)a[j]; r[4 + j] = (bf16_t)b[j]; }
    return r;
}
__device__ __forceinline__ bf16x8 zero8() {
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = (bf16_t)0.0f;
    return r;
}

// One operand of the tile product.  KSLOW = false: element (i, k) at p[i*ld + k]; true: at p[k*ld + i].
// i runs over the tile's 128 rows (m for A, n for B) starting at i0, k over [k0, k0 + 32).
// Each of the 256 threads fetches PQ x 8 elements along the contiguous index.
template <typename T, bool KSLOW>
struct Operand {
    const T* p;
    long long ld;
    long long n_i;     // extent of i (rows beyond it read as zero)
    long long n_k;
    RowMask mask;      // applies to the source row: i if !KSLOW, k if KSLOW

    __device__ __forceinline__ void fetch(bf16x8 (&v)[PQ], long long i0, long long k0, int tid) const {
        // Branch-free: an element outside the operand, or in a padded source row, is loaded from the
        // operand's first element instead and cleared afterwards (conditional loads would each wait
        // for the one before).
        typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int q = 0; q < PQ; ++q) {
            const int e = tid + 256 * q;                 // PT*PK/8 chunks of 8 elements per tile
            long long i, k, src, off;
            if (!KSLOW) {
                i = i0 + e / (PK / 8);                   // PK/8 chunks of 8 along k per row
                k = k0 + (e % (PK / 8)) * 8;
                src = i;
                off = i * ld + k;
            } else {
                k = k0 + (e >> 4);                       // 16 chunks of 8 along i per k
                i = i0 + (e & 15) * 8;
                src = k;
                off = k * ld + i;
            }
            const bool ok = i < n_i && k < n_k;
            const bool keep = ok && row_is_data(mask, ok ? src : 0);
            const bf16x8 x = load8(p + (ok ? off : 0));
            u32x4_t w = __builtin_bit_cast(u32x4_t, x);
            w &= keep ? ~0u : 0u;
            v[q] = __builtin_bit_cast(bf16x8, w);
        }
    }
    // LDS image of the tile.  !KSLOW: [i][k], pitch PP (k contiguous).  KSLOW: as in memory, [k][i] with
    // 128 elements per row, 16-byte chunk c of row k at position c ^ 4*(k%4) (conflict-free for the
    // transposing read that turns it into MFMA fragments).
    __device__ __forceinline__ void stage(const bf16x8 (&v)[PQ], bf16_t* tile, int tid) const {
#pragma unroll
        for (int q = 0; q < PQ; ++q) {
            const int e = tid + 256 * q;
            if (!KSLOW) {
                *reinterpret_cast<bf16x8*>(tile + (e / (PK / 8)) * PP + (e % (PK / 8)) * 8) = v[q];
            } else {
                const int kk = e >> 4, c = e & 15;
                *reinterpret_cast<bf16x8*>(tile + kk * PT + ((c ^ ((kk & 3) << 2)) << 3)) = v[q];
            }
        }
    }
    // MFMA fragment of rows [i_base, i_base + 32), k16-step kk: lane l holds row i_base + l%32, k = 8*(l/32)..+7
    __device__ __forceinline__ bf16x8 fragment(const bf16_t* tile, int i_base, int kk, int lane) const {
        if (!KSLOW) {
            return *reinterpret_cast<const bf16x8*>(tile + (i_base + (lane & 31)) * PP + kk * 16 + (lane >> 5) * 8);
        } else {
            // transposing read: within 16 lanes, lane 4j+c supplies 4 columns of row j and lane i receives
            // rows 0..3 of column i; lane = 16 g + 4 j + c reads row 8*(g/2) + j, columns 16*(g%2) + 4c .. +3
            typedef short s16x4 __attribute__((ext_vector_type(4)));
            typedef short s16x8 __attribute__((ext_vector_type(8)));
            const int fg = lane >> 4, fj = (lane >> 2) & 3, fc = lane & 3;
            const int row = kk * 16 + 8 * (fg >> 1) + fj;
            const int col = i_base + 16 * (fg & 1) + 4 * fc;
            const bf16_t* p = tile + row * PT + ((((col >> 3) ^ (fj << 2))) << 3) + (col & 7);
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + 4 * PT));
            const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, v);
        }
    }
};

struct Epilogue {
    void* C;
    long long ldc;
    const float* bias;   // per column n, or null
    int out_bf16;        // store bf16 (else fp32)
    int atomic;          // fp32 atomicAdd (split-K) instead of a store
};

template <typename TA, bool AK, typename TB, bool BK>
__global__ __launch_bounds__(256) void k_proj_gemm(Operand<TA, AK> A, Operand<TB, BK> B, Epilogue ep, long long M,
                                                   long long N, long long K, long long k_per_split) {
    extern __shared__ __align__(16) unsigned char proj_smem[];
    bf16_t* As = reinterpret_cast<bf16_t*>(proj_smem);
    bf16_t* Bs = As + PT * PP;             // PT*PP >= PK*PT: either layout fits
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hb = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    static_assert(PT * PP >= PK * PT, "LDS tile size");
    const long long m0 = (long long)blockIdx.x * PT, n0 = (long long)blockIdx.y * PT;
    const long long ks = (long long)blockIdx.z * k_per_split;
    const long long ke = ks + k_per_split < K ? ks + k_per_split : K;
    if (ks >= ke) return;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = f32x16{0};

    // Global loads run PD K-steps ahead of the MFMAs (register sets, rotated by unrolling): a small
    // problem leaves one workgroup per CU, and nothing else hides the memory latency.
    bf16x8 va[PD][PQ], vb[PD][PQ];
    const long long nsteps = (ke - ks + PK - 1) / PK;
#pragma unroll
    for (int u = 0; u < PD; ++u)
        if (u < nsteps) {
            A.fetch(va[u], m0, ks + (long long)u * PK, tid);
            B.fetch(vb[u], n0, ks + (long long)u * PK, tid);
        }
    for (long long s0 = 0; s0 < nsteps; s0 += PD) {
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            const long long st = s0 + u;
            if (st >= nsteps) break;
            __syncthreads();                     // the previous step's fragment reads are done
            A.stage(va[u], As, tid);
            B.stage(vb[u], Bs, tid);
            __syncthreads();
            if (st + PD < nsteps) {
                A.fetch(va[u], m0, ks + (st + PD) * PK, tid);
                B.fetch(vb[u], n0, ks + (st + PD) * PK, tid);
            }
#pragma unroll
            for (int kk = 0; kk < PK / 16; ++kk) {
                bf16x8 fa[2], fb[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) fa[i] = A.fragment(As, wm * 64 + i * 32, kk, lane);
#pragma unroll
                for (int j = 0; j < 2; ++j) fb[j] = B.fragment(Bs, wn * 64 + j * 32, kk, lane);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
        }
    }
    // accumulator register 4q+r of tile (i,j): row 8q + 4hb + r, column l32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const long long n = n0 + wn * 64 + j * 32 + l32;
            if (n >= N) continue;
            const float bv = (ep.bias != nullptr && blockIdx.z == 0) ? ep.bias[n] : 0.0f;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const long long m = m0 + wm * 64 + i * 32 + 8 * (q >> 2) + 4 * hb + (q & 3);
                if (m >= M) continue;
                const float v = acc[i][j][q] + bv;
                if (ep.atomic) atomicAdd(reinterpret_cast<float*>(ep.C) + m * ep.ldc + n, v);
                else if (ep.out_bf16) reinterpret_cast<bf16_t*>(ep.C)[m * ep.ldc + n] = (bf16_t)v;
                else reinterpret_cast<float*>(ep.C)[m * ep.ldc + n] = v;
            }
        }
}

template <typename TA, bool AK, typename TB, bool BK>
hipError_t launch_tile_gemm(const void* A, long long lda, const RowMask& ma, const void* Bm, long long ldb,
                            const RowMask& mb, const Epilogue& ep, long long M, long long N, long long K, int splits,
                            hipStream_t stream) {
    if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
    Operand<TA, AK> a{(const TA*)A, lda, M, K, ma};
    Operand<TB, BK> b{(const TB*)Bm, ldb, N, K, mb};
    long long per = (K + splits - 1) / splits;
    per = (per + PK - 1) / PK * PK;
    const long long nz = (K + per - 1) / per;
    dim3 grid((unsigned)((M + PT - 1) / PT), (unsigned)((N + PT - 1) / PT), (unsigned)nz);
    const size_t smem = (size_t)2 * PT * PP * sizeof(bf16_t);
    static bool configured = false;          // one flag per instantiation
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_proj_gemm<TA, AK, TB, BK>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        configured = true;
    }
    k_proj_gemm<TA, AK, TB, BK><<<grid, dim3(256), smem, stream>>>(a, b, ep, M, N, K, per);
    return hipGetLastError();
}

// ---- fp32: one thread per output element ---------------------------------------------------
// A(m,k) at a[m*sam + k*sak], B(k,n) at b[k*sbk + n*sbn]; mask_on: 0 none, 1 rows m of A, 2 rows k (both operands)
__global__ void k_proj_gemm_f32(const float* __restrict__ a, long long sam, long long sak, const float* __restrict__ b,
                                long long sbk, long long sbn, float* __restrict__ c, long long ldc,
                                const float* __restrict__ bias, long long M, long long N, long long K, RowMask mask,
                                int mask_on, int accumulate) {
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= M * N) return;
    const long long m = idx / N, n = idx - m * N;
    float s = bias ? bias[n] : 0.0f;
    if (mask_on != 1 || row_is_data(mask, m)) {
        for (long long k = 0; k < K; ++k) {
            if (mask_on == 2 && !row_is_data(mask, k)) continue;
            s = fmaf(a[m * sam + k * sak], b[k * sbk + n * sbn], s);
        }
    }
    c[m * ldc + n] = accumulate ? c[m * ldc + n] + s : s;
}

// out[c] (+)= sum over all rows of x[r, c]   (x fp32 [rows, cols]); 256 columns x one slice of rows per workgroup
__global__ __launch_bounds__(256) void k_col_sum(const float* __restrict__ x, long long rows, int cols, long long rows_per,
                                                 float* __restrict__ out) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= cols) return;
    const long long r0 = (long long)blockIdx.y * rows_per;
    const long long r1 = r0 + rows_per < rows ? r0 + rows_per : rows;
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    long long r = r0;
    for (; r + 3 < r1; r += 4) {
        s0 += x[r * cols + c];
        s1 += x[(r + 1) * cols + c];
        s2 += x[(r + 2) * cols + c];
        s3 += x[(r + 3) * cols + c];
    }
    for (; r < r1; ++r) s0 += x[r * cols + c];
    atomicAdd(&out[c], (s0 + s1) + (s2 + s3));
}

}  // namespace

hipError_t launch_proj_forward(int bf16, const void* h, long long rows, int D, const RowMask& mask, const void* W,
                               const float* bias, int H, void* out, hipStream_t stream) {
    if (bf16) {
        Epilogue ep{out, H, bias, 1, 0};
        return launch_tile_gemm<bf16_t, false, bf16_t, true>(h, D, mask, W, H, RowMask{nullptr, 1, 0}, ep, rows, H, D, 1,
                                                             stream);
    }
    if (gemm_f32_edge_fits(h, D, W, H, D, H))
        return launch_gemm_f32_masked(0, 1, (const float*)h, D, mask, (const float*)W, H, RowMask{nullptr, 1, 0},
                                      (float*)out, H, bias, 0, rows, H, D, 1, stream);
    const long long total = rows * H;
    k_proj_gemm_f32<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream>>>(
        (const float*)h, D, 1, (const float*)W, H, 1, (float*)out, H, bias, rows, H, D, mask, 1, 0);
    return hipGetLastError();
}

hipError_t launch_proj_backward_input(int bf16, const float* d_out, long long rows, int H, const void* W, int D,
                                      float* d_in, hipStream_t stream) {
    // padded rows of d_out are zero, so d_in is zero there without a mask
    const RowMask none{nullptr, 1, 0};
    if (bf16) {
        Epilogue ep{d_in, D, nullptr, 0, 0};
        return launch_tile_gemm<float, false, bf16_t, false>(d_out, H, none, W, H, none, ep, rows, D, H, 1, stream);
    }
    if (gemm_f32_edge_fits(d_out, H, W, H, H, H))
        return launch_gemm_f32_masked(0, 0, d_out, H, none, (const float*)W, H, none, d_in, D, nullptr, 0, rows, D, H, 1,
                                      stream);
    const long long total = rows * D;
    k_proj_gemm_f32<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream>>>(
        d_out, H, 1, (const float*)W, 1, H, d_in, D, nullptr, rows, D, H, none, 0, 0);
    return hipGetLastError();
}

hipError_t launch_proj_backward_weight(int bf16, const void* h, long long rows, int D, const RowMask& mask,
                                       const float* d_out, int H, float* dW, hipStream_t stream) {
    if (bf16) {
        // split over the rows: about 512 workgroups in all, at least 256 rows per split; dW is added to
        const long long tiles = (long long)((D + PT - 1) / PT) * ((H + PT - 1) / PT);
        long long splits = (512 + tiles - 1) / tiles;
        const long long max_splits = (rows + 255) / 256;
        if (splits > max_splits) splits = max_splits;
        if (splits < 1) splits = 1;
        Epilogue ep{dW, H, nullptr, 0, 1};
        return launch_tile_gemm<bf16_t, true, float, true>(h, D, mask, d_out, H, mask, ep, D, H, rows, (int)splits, stream);
    }
    if (gemm_f32_edge_fits(h, D, d_out, H, D, H)) {
        // split over the rows as on the bf16 path; dW is added to with float atomics
        const long long tiles = (long long)((D + PT - 1) / PT) * ((H + PT - 1) / PT);
        long long splits = (512 + tiles - 1) / tiles;
        const long long max_splits = (rows + 255) / 256;
        if (splits > max_splits) splits = max_splits;
        if (splits < 1) splits = 1;
        return launch_gemm_f32_masked(1, 1, (const float*)h, D, mask, d_out, H, mask, dW, H, nullptr, 1, D, H, rows,
                                      (int)splits, stream);
    }
    const long long total = (long long)D * H;
    k_proj_gemm_f32<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream>>>(
        (const float*)h, 1, D, d_out, H, 1, dW, H, nullptr, D, H, rows, mask, 2, 1);
    return hipGetLastError();
}

hipError_t launch_col_sum(const float* x, long long rows, int cols, float* out, hipStream_t stream) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    long long slices = (rows + 31) / 32;
    if (slices > 1024) slices = 1024;
    const long long per = (rows + slices - 1) / slices;
    k_col_sum<<<dim3((unsigned)((cols + 255) / 256), (unsigned)((rows + per - 1) / per)), dim3(256), 0, stream>>>(
        x, rows, cols, per, out);
    return hipGetLastError();
}

}  // namespace rnnt
