// Forward/backward variables of the transducer lattice (f^W_2) and the loss (f^W_3), fp32 log space.
//
// One workgroup per (sample, direction): blockIdx.y = 0 sweeps alpha from (0,0), blockIdx.y = 1
// sweeps beta from (T-1,U).  Thread u owns label position u and walks its column one
// anti-diagonal per step; the value of the neighbouring column comes through LDS, the value of
// the neighbouring frame is the thread's own previous result.  The emission log-probabilities a
// step needs do not depend on earlier steps, so they are fetched PF steps ahead.
//
// Every alignment emits exactly T blanks and U labels, so adding a constant c to every emission
// log-probability shifts ln P by c*(T+U) and leaves all posteriors unchanged.  c is chosen per
// sample (minus the mean of the larger of the two emission log-probabilities over the lattice)
// so that alpha and beta stay near zero instead of growing to thousands, which keeps fp32
// resolution for the posteriors of long utterances.  The fp32 path's instantiation (k_lattice<double>)
// accumulates in fp64 and takes c = -ln P / (T+U) from a first sweep.
#include "device_common.h"

namespace rnnt {

constexpr int LAT_PF = 8;       // prefetch distance in steps

// Sum over this thread's share (i = first, first + stride, ...) of max(lpb, lpy) over the lattice.  The
// sweep cannot start before this sum is known, and a workgroup has few threads for the size of a lattice:
// 2 x LAT_SUM_DEPTH independent loads are in flight per thread, so that few memory latencies are exposed.
constexpr int LAT_SUM_DEPTH = 24;
__device__ __forceinline__ float emission_max_partial(const float* __restrict__ lpb, const float* __restrict__ lpy,
                                                      int n, int W1, int U, int first, int stride) {
    float acc[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    for (int i0 = first; i0 < n; i0 += LAT_SUM_DEPTH * stride) {
        float b[LAT_SUM_DEPTH], y[LAT_SUM_DEPTH];
#pragma unroll
        for (int j = 0; j < LAT_SUM_DEPTH; ++j) {
            const int i = i0 + j * stride;
            const int ic = (i < n) ? i : first;
            b[j] = lpb[ic];
            y[j] = lpy[ic];
        }
#pragma unroll
        for (int j = 0; j < LAT_SUM_DEPTH; ++j) {
            const int i = i0 + j * stride;
            const float v = (i % W1 < U) ? fmaxf(b[j], y[j]) : b[j];
            acc[j & 7] += (i < n) ? v : 0.0f;
        }
    }
    return ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
}
// The same sum from the per-tile sums the bf16 forward kernels leave behind (a few hundred numbers instead of
// the whole lattice), if there are any.  Both workgroups of a sample add in the same order.
__device__ __forceinline__ float emission_sum_partial(const SampleTable& st, const LatticeState& ls, int s,
                                                      const float* __restrict__ lpb, const float* __restrict__ lpy,
                                                      int n, int W1, int U, int first, int stride) {
    if (ls.tile_esum == nullptr) return emission_max_partial(lpb, lpy, n, W1, U, first, stride);
    float acc = 0.0f;
    for (int i = st.tile_off[s] + first, e = st.tile_off[s + 1]; i < e; i += stride) acc += ls.tile_esum[i];
    return acc;
}
// ln(e^a + e^b) on the hardware exp2/log2 units; one of the two may be -inf (both: NaN, which only lanes
// outside the lattice ever see and never keep).  The argument of the logarithm lies in [1, 2], so no range
// fix-up is needed.  Six dependent instructions: the sweep's step time is the latency of this chain.
__device__ __forceinline__ float log_add_exp_fast(float a, float b) {
    const float m = fmaxf(a, b);
    const float e = __builtin_amdgcn_exp2f(fabsf(a - b) * -1.44269504088896340736f);   // 0 when one is -inf
    return fmaf(__builtin_amdgcn_logf(1.0f + e), 0.69314718055994530942f, m);
}

constexpr int LAT_MAX_T = 1024; // threads per workgroup (label positions 0..U <= 1023)

// R = float: the sweep in fp32 (bf16 path).  R = double: the recursion accumulates in fp64 and alpha, beta are
// rounded to fp32 once, when stored (fp32 path: a sweep of T+U dependent fp32 log-add-exps loses about
// sqrt(T+U) half-ulps of values of the order of 100, 2e-4 relative in the posteriors of a 500 x 100 lattice).
__device__ __forceinline__ float lattice_lae(float a, float b) { return log_add_exp_fast(a, b); }
__device__ __forceinline__ double lattice_lae(double a, double b) {
    const double m = fmax(a, b);
    return m + log1p(exp(-fabs(a - b)));      // one of the two may be -inf
}

template <typename R>
__global__ __launch_bounds__(LAT_MAX_T) void k_lattice(SampleTable st, LatticeState ls, int s0,
                                                       float* __restrict__ loss) {
    __shared__ R xch[2][LAT_MAX_T + 2];
    __shared__ float red[LAT_MAX_T / 64];
    __shared__ float shift_sh;

    const int s = s0 + blockIdx.x;
    const bool is_beta = (blockIdx.y != 0);
    const int tid = threadIdx.x;
    const int T = st.T[s], U = st.U[s], W1 = U + 1;
    const long long base = st.row_off[s] - ls.row_base;
    const float* __restrict__ lpb = ls.lpb + base;
    const float* __restrict__ lpy = ls.lpy + base;
    const int n = T * W1;

    // ---- per-sample offset c (identical in both workgroups of a sample: same code, same order)
    {
        // (read from the emissions themselves although the forward kernels' per-tile sums would do: this pass
        // also brings the sample's emissions into the L2 the sweep then reads them from, and without it the
        // kernel as a whole was 7 % slower on lattices of 1000 x 200)
        float acc = emission_max_partial(lpb, lpy, n, W1, U, tid, (int)blockDim.x);
        acc = wave_sum(acc);
        if ((tid & 63) == 0) red[tid >> 6] = acc;
        __syncthreads();
        if (tid == 0) {
            float tot = 0.0f;
            for (int w = 0; w < (int)(blockDim.x >> 6); ++w) tot += red[w];
            shift_sh = -tot / (float)n;
        }
        xch[0][tid + 1] = (R)RNNT_NEG_INF;
        xch[1][tid + 1] = (R)RNNT_NEG_INF;
        if (tid == 0) {
            xch[0][0] = xch[1][0] = (R)RNNT_NEG_INF;
            xch[0][blockDim.x + 1] = xch[1][blockDim.x + 1] = (R)RNNT_NEG_INF;
        }
        __syncthreads();
    }
    float c = shift_sh;
    const int u = tid;
    const bool col = (u <= U);
    const int nsteps = T + U;   // anti-diagonals 0 .. T+U-1
    if constexpr (sizeof(R) == 8) {
        // fp64 sweep (fp32 path): alpha and beta are still stored as fp32, so their magnitude where the posteriors
        // are not negligible decides the accuracy.  With c = -ln P / (T+U) the offset ln P is zero and alpha, beta
        // stay near zero along the alignments that carry the probability, whatever the emissions look like (flat
        // scores, where the number of alignments adds hundreds to ln P, or peaked ones).  ln P is not known
        // beforehand: both workgroups of the sample first run the alpha sweep without storing anything (the same
        // arithmetic in both, hence the same c), then the sweep proper.
        __shared__ double c_better;
        R o = (R)RNNT_NEG_INF;
        int pr = 0;
        for (int k = 0; k < nsteps; ++k) {
            const int t = k - u;
            const bool act = col && t >= 0 && t < T;
            const R left = xch[pr][u];
            R val = o;
            if (act) {
                if (k == 0) {
                    val = (R)0;
                } else {
                    const R eb = (t > 0) ? (R)lpb[(t - 1) * W1 + u] + (R)c : (R)RNNT_NEG_INF;
                    const R ey = (u > 0) ? (R)lpy[t * W1 + u - 1] + (R)c : (R)RNNT_NEG_INF;
                    val = lattice_lae(o + eb, left + ey);
                }
                o = val;
            }
            xch[pr ^ 1][u + 1] = val;
            __syncthreads();
            pr ^= 1;
        }
        if (u == U) c_better = (double)c - (o + ((R)lpb[(T - 1) * W1 + U] + (R)c)) / (double)(T + U);
        __syncthreads();
        c = (float)c_better;
        xch[0][tid + 1] = (R)RNNT_NEG_INF;
        xch[1][tid + 1] = (R)RNNT_NEG_INF;
        __syncthreads();
    }
    R own = RNNT_NEG_INF;
    int par = 0;
    float pb[LAT_PF], py[LAT_PF];

    if (!is_beta) {
        float* __restrict__ alpha = ls.alpha + base;
        // step k handles node (t = k - u, u): needs lpb[t-1,u] and lpy[t,u-1]
        auto fetch = [&](int k, float& fb, float& fy) {
            const int t = k - u;
            fb = 0.0f;
            fy = 0.0f;
            if (col && t >= 0 && t < T) {
                if (t > 0) fb = lpb[(t - 1) * W1 + u];
                if (u > 0) fy = lpy[t * W1 + u - 1];
            }
        };
#pragma unroll
        for (int i = 0; i < LAT_PF; ++i) fetch(i, pb[i], py[i]);
        for (int k0 = 0; k0 < nsteps; k0 += LAT_PF) {
#pragma unroll
            for (int i = 0; i < LAT_PF; ++i) {
                const int k = k0 + i;
                if (k < nsteps) {
                    const int t = k - u;
                    const bool act = col && t >= 0 && t < T;
                    const R left = xch[par][u];          // column u-1, previous step
                    R val = own;
                    if (act) {
                        if (k == 0) {
                            val = (R)0;
                        } else {
                            // the offset and the boundary conditions go into the emission values, which do not
                            // depend on the step before: the dependent chain is own -> add -> log-add-exp
                            const R eb = (t > 0) ? (R)pb[i] + (R)c : (R)RNNT_NEG_INF;
                            const R ey = (u > 0) ? (R)py[i] + (R)c : (R)RNNT_NEG_INF;
                            val = lattice_lae(own + eb, left + ey);
                        }
                        alpha[t * W1 + u] = (float)val;
                        own = val;
                    }
                    xch[par ^ 1][u + 1] = val;
                    fetch(k + LAT_PF, pb[i], py[i]);
                    __syncthreads();
                    par ^= 1;
                }
            }
        }
        if (u == U) {
            // own = alpha[T-1,U]; ln P (offset) = alpha + final blank
            const R lnP_off = own + ((R)lpb[(T - 1) * W1 + U] + (R)c);
            ls.lnP[s] = (float)lnP_off;
            ls.shift[s] = c;
            loss[s] = (float)-(lnP_off - (R)c * (R)(T + U));
        }
    } else {
        float* __restrict__ beta = ls.beta + base;
        // step k handles node (t = T-1 - (k - (U-u)), u): needs lpb[t,u] and lpy[t,u]
        auto fetch = [&](int k, float& fb, float& fy) {
            const int t = T - 1 - (k - (U - u));
            fb = 0.0f;
            fy = 0.0f;
            if (col && t >= 0 && t < T) {
                fb = lpb[t * W1 + u];
                if (u < U) fy = lpy[t * W1 + u];
            }
        };
#pragma unroll
        for (int i = 0; i < LAT_PF; ++i) fetch(i, pb[i], py[i]);
        for (int k0 = 0; k0 < nsteps; k0 += LAT_PF) {
#pragma unroll
            for (int i = 0; i < LAT_PF; ++i) {
                const int k = k0 + i;
                if (k < nsteps) {
                    const int t = T - 1 - (k - (U - u));
                    const bool act = col && t >= 0 && t < T;
                    const R right = xch[par][u + 2];     // column u+1, previous step
                    R val = own;
                    if (act) {
                        if (k == 0) {
                            val = (R)pb[i] + (R)c;           // beta[T-1,U] = final blank
                        } else {
                            const R eb = (t < T - 1) ? (R)pb[i] + (R)c : (R)RNNT_NEG_INF;
                            const R ey = (u < U) ? (R)py[i] + (R)c : (R)RNNT_NEG_INF;
                            val = lattice_lae(own + eb, right + ey);
                        }
                        beta[t * W1 + u] = (float)val;
                        own = val;
                    }
                    xch[par ^ 1][u + 1] = val;
                    fetch(k + LAT_PF, pb[i], py[i]);
                    __syncthreads();
                    par ^= 1;
                }
            }
        }
    }
}

// Same recursion for lattices with at most 64 label positions (U + 1 <= 64): one wavefront per
// (sample, direction), no barrier; the neighbouring column arrives by a lane shift.
//
// The emission log-probabilities reach the recursion through LDS: a ring of LW_ROWS sweep rows (frames in
// sweep order: upwards for alpha, downwards for beta) of 64 floats each, filled in blocks of LW_RB rows
// by asynchronous global -> LDS copies one block ahead of the block the sweep is in.  The sequential
// steps then wait for LDS reads only, issued one step ahead, and every per-step index advances by an
// addition: with a single wave per SIMD the step time is the issue time of its instructions.
constexpr int LW_RB = 32;                 // sweep rows per staged block
constexpr int LW_ROWS = 128;              // rows in the ring (a step touches its row and the 64 before it)
constexpr int LW_RING = LW_ROWS * 64;     // floats per array

// Value of lane l-1 (lane 0 gets 0) / lane l+1 (lane 63 gets 0): whole-wavefront shifts on the
// data-parallel-primitive path, no LDS round trip.  With nothing to preserve in the lanes that have no
// source the shift can ride on the addition that consumes it instead of taking a move of its own.
__device__ __forceinline__ float lane_from_below(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x138 /* wave_shr:1 */, 0xf, 0xf, true));
}
__device__ __forceinline__ float lane_from_above(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x130 /* wave_shl:1 */, 0xf, 0xf, true));
}
// Makes the compiler finish a value where this stands instead of sinking its arithmetic to the first use
// (for the emission values: into the dependent chain of the next step).
__device__ __forceinline__ void pin(float& a, float& b) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("" : "+v"(a), "+v"(b));
#endif
}

// Asynchronous global -> LDS copy of 4 bytes per lane (global_load_lds_dword): lane l's word lands at LDS
// byte address lds_base + 4*l (lds_base wave-uniform, passed in M0).  The compiler does not see
// these loads; the sweep waits for them explicitly (vmcnt) before the first step that reads them.
__device__ __forceinline__ void lds_dma4(const void* gptr, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off" ::"v"(gptr), "s"(lds_base) : "memory", "m0");
}

// Steps 1 .. nsteps-1 of a sweep.  Step k with (k+1) % LW_RB == 0 is the last one before the sweep enters the
// next staged block: it first waits for that block and sends for the one after it.  Whole blocks of LW_RB
// steps are unrolled (a taken branch costs about as much as the arithmetic of a step); the steps before the
// first whole block and after the last one run in plain loops.
#define SWEEP(step)                                                          \
    {                                                                        \
        int k = 1;                                                           \
        for (; k < nsteps && k < LW_RB; ++k) {                               \
            if (k == LW_RB - 1) {                                            \
                landed();                                                    \
                issue(2);                                                    \
            }                                                                \
            step();                                                          \
        }                                                                    \
        for (; k + LW_RB <= nsteps; k += LW_RB) {                            \
            _Pragma("unroll") for (int j = 0; j < LW_RB - 1; ++j) step();    \
            landed();                                                        \
            issue(k / LW_RB + 2);                                            \
            step();                                                          \
        }                                                                    \
        for (; k < nsteps; ++k) step();                                      \
    }

__global__ __launch_bounds__(64) void k_lattice_wave(SampleTable st, LatticeState ls, int s0,
                                                     float* __restrict__ loss) {
    extern __shared__ __align__(16) float lw_smem[];    // ring_b [LW_ROWS][64], ring_y [LW_ROWS][64]
    const float* ring_b = lw_smem;
    const float* ring_y = lw_smem + LW_RING;
    const unsigned smem_base = (unsigned)(size_t)(__attribute__((address_space(3))) float*)lw_smem;
    const int s = s0 + blockIdx.x;
    const bool is_beta = (blockIdx.y != 0);
    const int u = threadIdx.x;
    const int T = st.T[s], U = st.U[s], W1 = U + 1;
    const long long base = st.row_off[s] - ls.row_base;
    const float* __restrict__ lpb = ls.lpb + base;
    const float* __restrict__ lpy = ls.lpy + base;
    const int n = T * W1;
    const float c = -wave_sum(emission_sum_partial(st, ls, s, lpb, lpy, n, W1, U, u, 64)) / (float)n;
    const int nsteps = T + U;
    const unsigned T_act = (u <= U) ? (unsigned)T : 0u;     // lanes beyond the last label position never act

    // Block q holds sweep rows d = q*LW_RB .. +LW_RB-1, i.e. frame d (alpha) or T-1-d (beta); one copy per
    // row and array, lane = column.  Indices outside the sample (rows past its end, lanes past the row)
    // are clamped to a valid one; such values are never used by an acting lane.
    auto issue = [&](int q) {
        for (int j = 0; j < LW_RB; ++j) {
            const int d = q * LW_RB + j;
            const int t = is_beta ? T - 1 - d : d;
            int idx = t * W1 + u;
            idx = idx < 0 ? 0 : (idx > n - 1 ? n - 1 : idx);
            const unsigned dst = smem_base + (unsigned)(d & (LW_ROWS - 1)) * 256u;
            lds_dma4(lpb + idx, __builtin_amdgcn_readfirstlane(dst));
            lds_dma4(lpy + idx, __builtin_amdgcn_readfirstlane(dst + LW_RING * 4u));
        }
    };
    // waits for the staged copies; the LDS reads already issued must be complete as well, since the
    // next copy overwrites rows that an already fetched operand may have come from
    auto landed = [&]() { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory"); };
    issue(0);
    issue(1);
    landed();

    // Step k computes the node at sweep row d = k - u (alpha, frame t = d) resp. d = k - (U - u) (beta,
    // frame t = T-1-d).  Step 0 has a single node, handled up front; the emission values of step k+1 are
    // read from the ring during step k.
    if (!is_beta) {
        float* __restrict__ alpha = ls.alpha + base;
        float own = RNNT_NEG_INF;
        if (u == 0) {
            alpha[0] = 0.0f;
            own = 0.0f;
        }
        const bool has_left = (u > 0);
        const int du = has_left ? 1 : 0;
        int d = 1 - u;                                              // sweep row of step 1
        unsigned so = (unsigned)(d * W1 + u);                       // index of the node written at step 1
        // blank emission of frame d-1 at column u, label emission of frame d at column u-1
        unsigned rb = (unsigned)((((d - 1) & (LW_ROWS - 1)) << 6) + u);
        unsigned ry = (unsigned)(((d & (LW_ROWS - 1)) << 6) + u - du);
        // The offset c and the two boundary conditions (no frame below row 0, no column left of 0) go into
        // the emission values as soon as they arrive, off the dependent chain own -> val -> own.
        float eb = (d > 0) ? ring_b[rb] + c : RNNT_NEG_INF;
        float ey = has_left ? ring_y[ry] + c : RNNT_NEG_INF;
        auto step = [&]() {
            rb = ry + du;
            ry = (ry + 64u) & (LW_RING - 1);
            const float eb_r = ring_b[rb], ey_r = ring_y[ry];
            const bool act = (unsigned)d < T_act;
            const float left = lane_from_below(own);                // column u-1, previous step
            const float val = log_add_exp_fast(own + eb, left + ey);
            own = act ? val : own;
            if (act) alpha[so] = val;
            so += (unsigned)W1;
            d += 1;
            eb = (d > 0) ? eb_r + c : RNNT_NEG_INF;
            ey = has_left ? ey_r + c : RNNT_NEG_INF;
            pin(eb, ey);
        };
        SWEEP(step)
        if (u == U) {
            const float lnP_off = own + (lpb[(T - 1) * W1 + U] + c);
            ls.lnP[s] = lnP_off;
            ls.shift[s] = c;
            loss[s] = -(lnP_off - c * (float)(T + U));
        }
    } else {
        float* __restrict__ beta = ls.beta + base;
        float own = RNNT_NEG_INF;
        if (u == U) {
            own = ring_b[u] + c;                                    // beta[T-1,U] = final blank
            beta[(T - 1) * W1 + U] = own;
        }
        const bool has_right = (u < U);
        int d = 1 - (U - u);                                        // sweep row of step 1
        unsigned so = (unsigned)((T - 1 - d) * W1 + u);
        unsigned ro = (unsigned)(((d & (LW_ROWS - 1)) << 6) + u);   // both emissions of the node itself
        float eb = (d > 0) ? ring_b[ro] + c : RNNT_NEG_INF;        // d > 0: frame t < T-1
        float ey = has_right ? ring_y[ro] + c : RNNT_NEG_INF;
        auto step = [&]() {
            ro = (ro + 64u) & (LW_RING - 1);
            const float eb_r = ring_b[ro], ey_r = ring_y[ro];
            const bool act = (unsigned)d < T_act;
            const float right = lane_from_above(own);               // column u+1, previous step
            const float val = log_add_exp_fast(own + eb, right + ey);
            own = act ? val : own;
            if (act) beta[so] = val;
            so -= (unsigned)W1;
            d += 1;
            eb = (d > 0) ? eb_r + c : RNNT_NEG_INF;
            ey = has_right ? ey_r + c : RNNT_NEG_INF;
            pin(eb, ey);
        };
        SWEEP(step)
    }
}

hipError_t launch_lattice(const SampleTable& st, const LatticeState& ls, int s0, int s1, int u_max, int wide,
                          float* loss, hipStream_t stream) {
    if (s1 <= s0) return hipSuccess;
    if (wide) {
        const int threads = ((u_max + 1) + 63) / 64 * 64;
        if (threads > LAT_MAX_T) return hipErrorInvalidValue;
        k_lattice<double><<<dim3((unsigned)(s1 - s0), 2), dim3(threads), 0, stream>>>(st, ls, s0, loss);
        return hipGetLastError();
    }
    if (u_max + 1 <= 64) {
        k_lattice_wave<<<dim3((unsigned)(s1 - s0), 2), dim3(64), 2 * LW_RING * sizeof(float), stream>>>(
            st, ls, s0, loss);
        return hipGetLastError();
    }
    int threads = ((u_max + 1) + 63) / 64 * 64;
    if (threads > LAT_MAX_T) return hipErrorInvalidValue;
    k_lattice<float><<<dim3((unsigned)(s1 - s0), 2), dim3(threads), 0, stream>>>(st, ls, s0, loss);
    return hipGetLastError();
}

}  // namespace rnnt
