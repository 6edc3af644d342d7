// fp32 path: plain FMA kernels, one wavefront per lattice node.  Serves the fp32 workloads
// (small shapes, tight tolerance) and any H, V; the throughput path is the bf16 MFMA one.
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

}  // namespace rnnt
