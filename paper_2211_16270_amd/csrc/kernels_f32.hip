// fp32 path.  Two forms:
//  * plain FMA kernels, one wavefront per lattice node, for any H, V (the small fp32 workloads);
//  * for H and V multiples of 4 from 64 on, the same steps over chunks of lattice nodes as fp32 MFMA GEMMs
//    (v_mfma_f32_32x32x2_f32, full fp32 products and sums) with row kernels between them:
//      Z = tanh(enc_t + pred_u)              (Eq. 4)            k_rows_z_f32
//      S = Z W + b                            (Eq. 6)            k_gemm_f32 <A k-contiguous, B k-slow>
//      lse, lpb, lpy per row                  (f^W_1)            k_rows_stats_f32
//      dh = gamma softmax - posteriors        (f^W_4)            k_rows_dh_f32 (in place of S)
//      db += column sums, dW += Z^T dh        (Alg. 1 line 8)    k_gemm_f32 <A k-slow, B k-slow>, split over the rows
//      dZ = dh W^T                            (Alg. 1 l. 10-11)  k_gemm_f32 <A k-contiguous, B k-contiguous>
//      d_enc, d_pred += dZ (1 - Z^2)                             k_rows_dz_f32
//    The chunk buffers S [rows, V], Z and dZ [rows, H] live in the workspace; rows beyond the chunk's
//    last node (up to the next multiple of 128) are zero.  The throughput path is the bf16 one.
#include <cstdint>

#include "device_common.h"

namespace rnnt {

__global__ void k_copy_f32(const float4* __restrict__ src, float4* __restrict__ dst, size_t n4) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n4; i += stride) dst[i] = src[i];
}

hipError_t launch_copy_f32(const float* src, float* dst, size_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    k_copy_f32<<<dim3(4096), dim3(256), 0, stream>>>((const float4*)src, (float4*)dst, n / 4);
    return hipGetLastError();
}

struct NodePos {
    int s, T, U, t, u;
    long long idx;  // index into the group's lattice arrays
};

__device__ __forceinline__ NodePos locate_node(const SampleTable& st, long long row_base, int s0, int s1,
                                               long long r) {
    NodePos p;
    const long long rg = r + row_base;
    p.s = find_segment<long long>(st.row_off, s0, s1, rg);
    p.T = st.T[p.s];
    p.U = st.U[p.s];
    const int local = (int)(rg - st.row_off[p.s]);
    p.t = local / (p.U + 1);
    p.u = local - p.t * (p.U + 1);
    p.idx = r;
    return p;
}

// Eq. (4), Eq. (6), f^W_1 for one lattice node per wavefront.
__global__ __launch_bounds__(64) void k_fwd_f32(Problem pr, SampleTable st, LatticeState ls, int s0, int s1,
                                                long long rows) {
    extern __shared__ float zs[];  // [H]
    const long long r = blockIdx.x;
    if (r >= rows) return;
    const int lane = threadIdx.x;
    const NodePos p = locate_node(st, ls.row_base, s0, s1, r);
    const int H = pr.H, V = pr.V;
    const float* enc = (const float*)pr.enc + ((size_t)p.s * pr.T_max + p.t) * H;
    const float* prd = (const float*)pr.pred + ((size_t)p.s * (pr.U_max + 1) + p.u) * H;
    for (int k = lane; k < H; k += 64) zs[k] = tanhf(enc[k] + prd[k]);
    __syncthreads();
    const float* W = (const float*)pr.W;
    const int label = (p.u < p.U) ? pr.labels[(size_t)p.s * pr.U_max + p.u] : -1;
    float m = RNNT_NEG_INF, ssum = 0.0f, cap_b = RNNT_NEG_INF, cap_y = RNNT_NEG_INF;
    for (int v = lane; v < V; v += 64) {
        float acc = 0.0f;
        for (int k = 0; k < H; ++k) acc = fmaf(zs[k], W[(size_t)k * V + v], acc);
        acc += pr.b_out[v];
        if (v == pr.blank) cap_b = acc;
        if (v == label) cap_y = acc;
        const float mn = fmaxf(m, acc);
        ssum = ssum * expf(m - mn) + expf(acc - mn);
        m = mn;
    }
    const float M = wave_max(m);
    const float S = wave_sum(m == RNNT_NEG_INF ? 0.0f : ssum * expf(m - M));
    const float lse = M + logf(S);
    cap_b = wave_max(cap_b);
    cap_y = wave_max(cap_y);
    if (lane == 0) {
        ls.lse[p.idx] = lse;
        ls.lpb[p.idx] = cap_b - lse;
        ls.lpy[p.idx] = (p.u < p.U) ? cap_y - lse : 0.0f;
    }
}

// f^W_4 and Algorithm 1 lines 8, 10, 11 for one lattice node per wavefront.
__global__ __launch_bounds__(64) void k_bwd_f32(Problem pr, SampleTable st, LatticeState ls, GradOut go, int s0,
                                                int s1, long long rows) {
    extern __shared__ float sm[];  // z[H], dh[V]
    const long long r = blockIdx.x;
    if (r >= rows) return;
    const int lane = threadIdx.x;
    const NodePos p = locate_node(st, ls.row_base, s0, s1, r);
    const int H = pr.H, V = pr.V;
    float* zs = sm;
    float* dh = sm + H;
    const float* enc = (const float*)pr.enc + ((size_t)p.s * pr.T_max + p.t) * H;
    const float* prd = (const float*)pr.pred + ((size_t)p.s * (pr.U_max + 1) + p.u) * H;
    for (int k = lane; k < H; k += 64) zs[k] = tanhf(enc[k] + prd[k]);
    __syncthreads();
    const float* W = (const float*)pr.W;
    const int label = (p.u < p.U) ? pr.labels[(size_t)p.s * pr.U_max + p.u] : -1;
    const RowPost rp = row_posteriors(ls, p.idx, p.t, p.u, p.T, p.U, p.s);
    const float off = rp.log_gamma - ls.lse[p.idx];
    for (int v = lane; v < V; v += 64) {
        float acc = 0.0f;
        for (int k = 0; k < H; ++k) acc = fmaf(zs[k], W[(size_t)k * V + v], acc);
        acc += pr.b_out[v];
        float d = expf(acc + off);
        if (v == pr.blank) d -= rp.Bk;
        if (v == label) d -= rp.Yk;
        dh[v] = d;
        atomicAdd(&go.db[v], d);
    }
    __syncthreads();
    float* d_enc = go.d_enc + ((size_t)p.s * pr.T_max + p.t) * H;
    float* d_prd = go.d_pred + ((size_t)p.s * (pr.U_max + 1) + p.u) * H;
    for (int k = 0; k < H; ++k) {
        const float zk = zs[k];
        float part = 0.0f;
        for (int v = lane; v < V; v += 64) {
            const float d = dh[v];
            part = fmaf(d, W[(size_t)k * V + v], part);
            atomicAdd(&go.dW[(size_t)k * V + v], zk * d);
        }
        part = wave_sum(part);
        if (lane == 0) {
            const float dx = part * (1.0f - zk * zk);
            atomicAdd(&d_enc[k], dx);
            atomicAdd(&d_prd[k], dx);
        }
    }
}

hipError_t launch_fwd_f32(const Problem& pr, const SampleTable& st, const LatticeState& ls, int s0, int s1,
                          long long rows, hipStream_t stream) {
    if (rows <= 0) return hipSuccess;
    k_fwd_f32<<<dim3((unsigned)rows), dim3(64), (size_t)pr.H * 4, stream>>>(pr, st, ls, s0, s1, rows);
    return hipGetLastError();
}

hipError_t launch_bwd_f32(const Problem& pr, const SampleTable& st, const LatticeState& ls, const GradOut& go,
                          int s0, int s1, long long rows, hipStream_t stream) {
    if (rows <= 0) return hipSuccess;
    k_bwd_f32<<<dim3((unsigned)rows), dim3(64), (size_t)(pr.H + pr.V) * 4, stream>>>(pr, st, ls, go, s0, s1, rows);
    return hipGetLastError();
}

// ---- fp32 MFMA GEMM path ---------------------------------------------------------------------

namespace {

constexpr int FT = 128;       // output tile edge
constexpr int FK = 16;        // K-step (32: 2.7 % slower at H = 1024, V = 4096)
constexpr int FQ = FT * FK / 4 / 256;  // 16-byte pieces per thread, operand and step
constexpr int FP = FT + 4;    // LDS row pitch (floats) of the [k][i] tile images

// One operand of the tile product.  KSLOW = false: element (i, k) at p[i*ld + k]; true: at p[k*ld + i].
// i runs over the tile's 128 rows (m for A, n for B), k over one K-step; every extent is a multiple of the
// tile sizes, so no access needs a guard.  In LDS both layouts become [k][i] (pitch FP): lane l of an MFMA
// operand fragment is element (i_base + l%32, 2 kk + l/32).
template <bool KSLOW>
struct OperandF32 {
    const float* p;
    long long ld;
    __device__ __forceinline__ void fetch(f32x4 (&v)[FQ], long long i0, long long k0, int tid) const {
#pragma unroll
        for (int q = 0; q < FQ; ++q) {
            const int e = tid + 256 * q;
            const long long off = !KSLOW ? (i0 + e / (FK / 4)) * ld + k0 + (e % (FK / 4)) * 4
                                         : (k0 + (e >> 5)) * ld + i0 + (e & 31) * 4;
            v[q] = *reinterpret_cast<const f32x4*>(p + off);
        }
    }
    __device__ __forceinline__ void stage(const f32x4 (&v)[FQ], float* tile, int tid) const {
#pragma unroll
        for (int q = 0; q < FQ; ++q) {
            const int e = tid + 256 * q;
            if (!KSLOW) {
                const int i = e / (FK / 4), k = (e % (FK / 4)) * 4;
#pragma unroll
                for (int j = 0; j < 4; ++j) tile[(k + j) * FP + i] = v[q][j];
            } else {
                *reinterpret_cast<f32x4*>(tile + (e >> 5) * FP + (e & 31) * 4) = v[q];
            }
        }
    }
};

// The same operand with edges: elements with i >= n_i or k >= n_k, and those of a padded source row (the
// row index is i if !KSLOW, k if KSLOW; see RowMask), read as zero.  The extent along the contiguous index
// is a multiple of 4, so a 16-byte piece is inside or outside as a whole.  Branch-free: a piece outside is
// loaded from the operand's first element and cleared.
template <bool KSLOW>
struct OperandF32Edge : OperandF32<KSLOW> {
    long long n_i, n_k;
    RowMask mask;
    __device__ __forceinline__ void fetch(f32x4 (&v)[FQ], long long i0, long long k0, int tid) const {
        typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int q = 0; q < FQ; ++q) {
            const int e = tid + 256 * q;
            const long long i = !KSLOW ? i0 + e / (FK / 4) : i0 + (e & 31) * 4;
            const long long k = !KSLOW ? k0 + (e % (FK / 4)) * 4 : k0 + (e >> 5);
            const long long off = !KSLOW ? i * this->ld + k : k * this->ld + i;
            const bool ok = i < n_i && k < n_k;
            bool keep = ok;
            if (mask.len != nullptr) {
                const long long src = ok ? (!KSLOW ? i : k) : 0, b = src / mask.period;
                keep = ok && (int)(src - b * mask.period) < mask.len[b] + mask.extra;
            }
            u32x4_t w = __builtin_bit_cast(u32x4_t, *reinterpret_cast<const f32x4*>(this->p + (ok ? off : 0)));
            w &= keep ? ~0u : 0u;
            v[q] = __builtin_bit_cast(f32x4, w);
        }
    }
};

// C[m, n] (+)= sum_k A(m, k) B(k, n) (+ bias[n]) in fp32.  128x128 output tile per workgroup, 4 waves x
// (64x64 = 2x2 MFMA 32x32x2 tiles), K-step 16, global loads one K-step ahead in registers.
// grid (M/128, N/128, splits); a split covers k_per_split (a multiple of 16) of K.  atomic != 0: the tile
// is added to C with float atomics (split over K, or C accumulates over calls).
template <class OpA, class OpB>
__global__ __launch_bounds__(256) void k_gemm_f32(OpA A, OpB B, float* __restrict__ C, long long ldc,
                                                  const float* __restrict__ bias, int atomic, long long M,
                                                  long long N, long long K, long long k_per_split) {
    __shared__ __align__(16) float As[FK * FP];
    __shared__ __align__(16) float Bs[FK * FP];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hb = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const long long m0 = (long long)blockIdx.x * FT, n0 = (long long)blockIdx.y * FT;
    const long long ks = (long long)blockIdx.z * k_per_split;
    const long long ke = ks + k_per_split < K ? ks + k_per_split : K;
    if (ks >= ke) return;
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = f32x16{0};
    f32x4 va[FQ], vb[FQ];
    A.fetch(va, m0, ks, tid);
    B.fetch(vb, n0, ks, tid);
    for (long long k0 = ks; k0 < ke; k0 += FK) {
        __syncthreads();                     // the previous step's fragment reads are done
        A.stage(va, As, tid);
        B.stage(vb, Bs, tid);
        __syncthreads();
        if (k0 + FK < ke) {
            A.fetch(va, m0, k0 + FK, tid);
            B.fetch(vb, n0, k0 + FK, tid);
        }
#pragma unroll
        for (int kk = 0; kk < FK / 2; ++kk) {
            float fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) fa[i] = As[(2 * kk + hb) * FP + wm * 64 + i * 32 + l32];
#pragma unroll
            for (int j = 0; j < 2; ++j) fb[j] = Bs[(2 * kk + hb) * FP + wn * 64 + j * 32 + l32];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }
    // accumulator register 4q+r of tile (i,j): row 8q + 4hb + r, column l32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const long long n = n0 + wn * 64 + j * 32 + l32;
            if (n >= N) continue;
            const float bv = (bias != nullptr && blockIdx.z == 0) ? bias[n] : 0.0f;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const long long m = m0 + wm * 64 + i * 32 + 8 * (q >> 2) + 4 * hb + (q & 3);
                if (m >= M) continue;
                const float v = acc[i][j][q] + bv;
                if (atomic) atomicAdd(C + m * ldc + n, v);
                else C[m * ldc + n] = v;
            }
        }
}

template <bool AK, bool BK>
hipError_t launch_gemm_f32(const float* A, long long lda, const float* B, long long ldb, float* C, long long ldc,
                           const float* bias, int atomic, long long M, long long N, long long K, int splits,
                           hipStream_t stream) {
    if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
    if (M % FT != 0 || N % FT != 0 || K % FK != 0 || splits < 1 || (splits > 1 && !atomic)) return hipErrorInvalidValue;
    long long per = (K + splits - 1) / splits;
    per = (per + FK - 1) / FK * FK;
    const long long nz = (K + per - 1) / per;
    if (M / FT > 0x7fffffffLL || N / FT > 65535 || nz > 65535) return hipErrorInvalidValue;
    k_gemm_f32<<<dim3((unsigned)(M / FT), (unsigned)(N / FT), (unsigned)nz), dim3(256), 0, stream>>>(
        OperandF32<AK>{A, lda}, OperandF32<BK>{B, ldb}, C, ldc, bias, atomic, M, N, K, per);
    return hipGetLastError();
}

template <bool AK, bool BK>
hipError_t launch_gemm_f32_edge(const float* A, long long lda, const RowMask& ma, const float* B, long long ldb,
                                const RowMask& mb, float* C, long long ldc, const float* bias, int atomic,
                                long long M, long long N, long long K, int splits, hipStream_t stream) {
    if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
    // 16-byte pieces along each operand's contiguous index
    const bool fits = lda % 4 == 0 && ldb % 4 == 0 && (AK ? M : K) % 4 == 0 && (BK ? N : K) % 4 == 0 &&
                      (uintptr_t)A % 16 == 0 && (uintptr_t)B % 16 == 0;
    if (!fits || splits < 1 || (splits > 1 && !atomic)) return hipErrorInvalidValue;
    long long per = (K + splits - 1) / splits;
    per = (per + FK - 1) / FK * FK;
    const long long nz = (K + per - 1) / per, gm = (M + FT - 1) / FT, gn = (N + FT - 1) / FT;
    if (gm > 0x7fffffffLL || gn > 65535 || nz > 65535) return hipErrorInvalidValue;
    OperandF32Edge<AK> a;
    a.p = A; a.ld = lda; a.n_i = M; a.n_k = K; a.mask = ma;
    OperandF32Edge<BK> b;
    b.p = B; b.ld = ldb; b.n_i = N; b.n_k = K; b.mask = mb;
    k_gemm_f32<<<dim3((unsigned)gm, (unsigned)gn, (unsigned)nz), dim3(256), 0, stream>>>(a, b, C, ldc, bias, atomic, M,
                                                                                        N, K, per);
    return hipGetLastError();
}

// Row i of the chunk is lattice node r0 + i of the group (i < n), or padding (n <= i < gridDim.x).
// Z[i, :] = tanh(enc_t + pred_u), zero in padding rows.
__global__ __launch_bounds__(256) void k_rows_z_f32(Problem pr, SampleTable st, LatticeState ls, int s0, int s1,
                                                    long long r0, long long n, float* __restrict__ Z) {
    const long long i = blockIdx.x;
    const int H = pr.H;
    float* z = Z + i * H;
    if (i >= n) {
        for (int k = threadIdx.x; k < H; k += 256) z[k] = 0.0f;
        return;
    }
    const NodePos p = locate_node(st, ls.row_base, s0, s1, r0 + i);
    const float* enc = (const float*)pr.enc + ((size_t)p.s * pr.T_max + p.t) * H;
    const float* prd = (const float*)pr.pred + ((size_t)p.s * (pr.U_max + 1) + p.u) * H;
    for (int k = threadIdx.x; k < H; k += 256) z[k] = tanhf(enc[k] + prd[k]);
}

// f^W_1 for one row of scores per wavefront (4 rows per workgroup): lse, lpb, lpy of node r0 + i.
__global__ __launch_bounds__(256) void k_rows_stats_f32(Problem pr, SampleTable st, LatticeState ls, int s0, int s1,
                                                        long long r0, long long n, const float* __restrict__ S) {
    const long long i = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n) return;
    const int lane = threadIdx.x & 63, V = pr.V;
    const NodePos p = locate_node(st, ls.row_base, s0, s1, r0 + i);
    const float* row = S + i * V;
    const int label = (p.u < p.U) ? pr.labels[(size_t)p.s * pr.U_max + p.u] : -1;
    const f32x4* row4 = reinterpret_cast<const f32x4*>(row);      // V is a multiple of 4, rows are 16-byte aligned
    float m = RNNT_NEG_INF;
    for (int v = lane; v < V / 4; v += 64) {
        const f32x4 x = row4[v];
        m = fmaxf(fmaxf(m, fmaxf(x[0], x[1])), fmaxf(x[2], x[3]));
    }
    const float M = wave_max(m);
    float ssum = 0.0f;
    for (int v = lane; v < V / 4; v += 64) {
        const f32x4 x = row4[v];
        ssum += (expf(x[0] - M) + expf(x[1] - M)) + (expf(x[2] - M) + expf(x[3] - M));
    }
    const float lse = M + logf(wave_sum(ssum));
    if (lane == 0) {
        ls.lse[p.idx] = lse;
        ls.lpb[p.idx] = row[pr.blank] - lse;
        ls.lpy[p.idx] = (label >= 0) ? row[label] - lse : 0.0f;
    }
}

// f^W_4 for one row per wavefront, in place of the scores: dh = gamma softmax - posteriors; zero in padding rows.
__global__ __launch_bounds__(256) void k_rows_dh_f32(Problem pr, SampleTable st, LatticeState ls, int s0, int s1,
                                                     long long r0, long long n, long long n_padded,
                                                     float* __restrict__ S) {
    const long long i = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n_padded) return;
    const int lane = threadIdx.x & 63, V = pr.V;
    float* row = S + i * V;
    if (i >= n) {
        for (int v = lane; v < V; v += 64) row[v] = 0.0f;
        return;
    }
    const NodePos p = locate_node(st, ls.row_base, s0, s1, r0 + i);
    const int label = (p.u < p.U) ? pr.labels[(size_t)p.s * pr.U_max + p.u] : -1;
    const RowPost rp = row_posteriors(ls, p.idx, p.t, p.u, p.T, p.U, p.s);
    const float off = rp.log_gamma - ls.lse[p.idx];
    f32x4* row4 = reinterpret_cast<f32x4*>(row);
    for (int v = lane; v < V / 4; v += 64) {
        f32x4 x = row4[v];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float d = expf(x[j] + off);
            if (4 * v + j == pr.blank) d -= rp.Bk;
            if (4 * v + j == label) d -= rp.Yk;
            x[j] = d;
        }
        row4[v] = x;
    }
}

// d_enc[s, t, :] += dZ (1 - Z^2), d_pred[s, u, :] += the same, for one node per workgroup.
__global__ __launch_bounds__(256) void k_rows_dz_f32(Problem pr, SampleTable st, LatticeState ls, int s0, int s1,
                                                     long long r0, const float* __restrict__ Z,
                                                     const float* __restrict__ dZ, float* __restrict__ d_enc,
                                                     float* __restrict__ d_pred) {
    const long long i = blockIdx.x;
    const int H = pr.H;
    const NodePos p = locate_node(st, ls.row_base, s0, s1, r0 + i);
    float* de = d_enc + ((size_t)p.s * pr.T_max + p.t) * H;
    float* dp = d_pred + ((size_t)p.s * (pr.U_max + 1) + p.u) * H;
    for (int k = threadIdx.x; k < H; k += 256) {
        const float z = Z[i * H + k];
        const float dx = dZ[i * H + k] * (1.0f - z * z);
        atomicAdd(&de[k], dx);
        atomicAdd(&dp[k], dx);
    }
}

}  // namespace

bool gemm_f32_edge_fits(const void* A, long long lda, const void* B, long long ldb, long long a_contig_extent,
                        long long b_contig_extent) {
    return lda % 4 == 0 && ldb % 4 == 0 && a_contig_extent % 4 == 0 && b_contig_extent % 4 == 0 &&
           (uintptr_t)A % 16 == 0 && (uintptr_t)B % 16 == 0;
}

hipError_t launch_gemm_f32_masked(int a_kslow, int b_kslow, const float* A, long long lda, const RowMask& ma,
                                  const float* B, long long ldb, const RowMask& mb, float* C, long long ldc,
                                  const float* bias, int atomic, long long M, long long N, long long K, int splits,
                                  hipStream_t stream) {
    if (!a_kslow && b_kslow)
        return launch_gemm_f32_edge<false, true>(A, lda, ma, B, ldb, mb, C, ldc, bias, atomic, M, N, K, splits, stream);
    if (!a_kslow && !b_kslow)
        return launch_gemm_f32_edge<false, false>(A, lda, ma, B, ldb, mb, C, ldc, bias, atomic, M, N, K, splits, stream);
    if (a_kslow && b_kslow)
        return launch_gemm_f32_edge<true, true>(A, lda, ma, B, ldb, mb, C, ldc, bias, atomic, M, N, K, splits, stream);
    return hipErrorInvalidValue;
}

namespace {
// The GEMM of the joint path: without edge handling where H and V are multiples of the tile, else with it.
template <bool AK, bool BK>
hipError_t joint_gemm_f32(const float* A, long long lda, const float* B, long long ldb, float* C, long long ldc,
                          const float* bias, int atomic, long long M, long long N, long long K, int splits,
                          hipStream_t stream) {
    if (M % FT == 0 && N % FT == 0 && K % FK == 0)
        return launch_gemm_f32<AK, BK>(A, lda, B, ldb, C, ldc, bias, atomic, M, N, K, splits, stream);
    const RowMask none{nullptr, 1, 0};
    return launch_gemm_f32_edge<AK, BK>(A, lda, none, B, ldb, none, C, ldc, bias, atomic, M, N, K, splits, stream);
}
}  // namespace

hipError_t launch_fwd_f32_gemm(const Problem& pr, const SampleTable& st, const LatticeState& ls, int s0, int s1,
                               long long r0, long long n, float* S, float* Z, hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    const long long np = (n + FT - 1) / FT * FT;
    k_rows_z_f32<<<dim3((unsigned)np), dim3(256), 0, stream>>>(pr, st, ls, s0, s1, r0, n, Z);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = joint_gemm_f32<false, true>(Z, pr.H, (const float*)pr.W, pr.V, S, pr.V, pr.b_out, 0, np, pr.V, pr.H, 1, stream);
    if (e != hipSuccess) return e;
    k_rows_stats_f32<<<dim3((unsigned)((n + 3) / 4)), dim3(256), 0, stream>>>(pr, st, ls, s0, s1, r0, n, S);
    return hipGetLastError();
}

hipError_t launch_bwd_f32_gemm(const Problem& pr, const SampleTable& st, const LatticeState& ls, const GradOut& go,
                               int s0, int s1, long long r0, long long n, float* S, float* Z, float* dZ,
                               hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    const long long np = (n + FT - 1) / FT * FT;
    const int H = pr.H, V = pr.V;
    const float* W = (const float*)pr.W;
    k_rows_z_f32<<<dim3((unsigned)np), dim3(256), 0, stream>>>(pr, st, ls, s0, s1, r0, n, Z);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = joint_gemm_f32<false, true>(Z, H, W, V, S, V, pr.b_out, 0, np, V, H, 1, stream);
    if (e != hipSuccess) return e;
    k_rows_dh_f32<<<dim3((unsigned)(np / 4)), dim3(256), 0, stream>>>(pr, st, ls, s0, s1, r0, n, np, S);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_col_sum(S, np, V, go.db, stream);
    if (e != hipSuccess) return e;
    // dW += Z^T dh: about 512 workgroups in all, at least 128 rows per split
    const long long tiles = (long long)((H + FT - 1) / FT) * ((V + FT - 1) / FT);
    long long splits = (512 + tiles - 1) / tiles;
    if (splits > np / FT) splits = np / FT;
    e = joint_gemm_f32<true, true>(Z, H, S, V, go.dW, V, nullptr, 1, H, V, np, (int)splits, stream);
    if (e != hipSuccess) return e;
    // dZ = dh W^T   (B(k = v, n = h) = W[h, v]: k-contiguous)
    e = joint_gemm_f32<false, false>(S, V, W, V, dZ, H, nullptr, 0, np, H, V, 1, stream);
    if (e != hipSuccess) return e;
    k_rows_dz_f32<<<dim3((unsigned)n), dim3(256), 0, stream>>>(pr, st, ls, s0, s1, r0, Z, dZ, go.d_enc, go.d_pred);
    return hipGetLastError();
}

}  // namespace rnnt
