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
// resolution for the posteriors of long utterances.
#include "device_common.h"

namespace rnnt {

constexpr int LAT_PF = 8;       // prefetch distance in steps

// Sum over this thread's share (i = first, first + stride, ...) of max(lpb, lpy) over the lattice,
// eight independent loads in flight.
__device__ __forceinline__ float emission_max_partial(const float* __restrict__ lpb, const float* __restrict__ lpy,
                                                      int n, int W1, int U, int first, int stride) {
    float acc[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    for (int i0 = first; i0 < n; i0 += 8 * stride) {
        float b[8], y[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = i0 + j * stride;
            const int ic = (i < n) ? i : first;
            b[j] = lpb[ic];
            y[j] = lpy[ic];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = i0 + j * stride;
            if (i < n) acc[j] += (i % W1 < U) ? fmaxf(b[j], y[j]) : b[j];
        }
    }
    return ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
}
constexpr int LAT_MAX_T = 1024; // threads per workgroup (label positions 0..U <= 1023)

__global__ __launch_bounds__(LAT_MAX_T) void k_lattice(SampleTable st, LatticeState ls, int s0,
                                                       float* __restrict__ loss) {
    __shared__ float xch[2][LAT_MAX_T + 2];
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
        float acc = emission_max_partial(lpb, lpy, n, W1, U, tid, (int)blockDim.x);
        acc = wave_sum(acc);
        if ((tid & 63) == 0) red[tid >> 6] = acc;
        __syncthreads();
        if (tid == 0) {
            float tot = 0.0f;
            for (int w = 0; w < (int)(blockDim.x >> 6); ++w) tot += red[w];
            shift_sh = -tot / (float)n;
        }
        xch[0][tid + 1] = RNNT_NEG_INF;
        xch[1][tid + 1] = RNNT_NEG_INF;
        if (tid == 0) {
            xch[0][0] = xch[1][0] = RNNT_NEG_INF;
            xch[0][blockDim.x + 1] = xch[1][blockDim.x + 1] = RNNT_NEG_INF;
        }
        __syncthreads();
    }
    const float c = shift_sh;
    const int u = tid;
    const bool col = (u <= U);
    const int nsteps = T + U;   // anti-diagonals 0 .. T+U-1
    float own = RNNT_NEG_INF;
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
                    const float left = xch[par][u];          // column u-1, previous step
                    float val = own;
                    if (act) {
                        if (k == 0) {
                            val = 0.0f;
                        } else {
                            const float a = (t > 0) ? own + (pb[i] + c) : RNNT_NEG_INF;
                            const float b = (u > 0) ? left + (py[i] + c) : RNNT_NEG_INF;
                            val = log_add_exp(a, b);
                        }
                        alpha[t * W1 + u] = val;
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
            const float lnP_off = own + (lpb[(T - 1) * W1 + U] + c);
            ls.lnP[s] = lnP_off;
            ls.shift[s] = c;
            loss[s] = -(lnP_off - c * (float)(T + U));
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
                    const float right = xch[par][u + 2];     // column u+1, previous step
                    float val = own;
                    if (act) {
                        if (k == 0) {
                            val = pb[i] + c;                 // beta[T-1,U] = final blank
                        } else {
                            const float a = (t < T - 1) ? own + (pb[i] + c) : RNNT_NEG_INF;
                            const float b = (u < U) ? right + (py[i] + c) : RNNT_NEG_INF;
                            val = log_add_exp(a, b);
                        }
                        beta[t * W1 + u] = val;
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
// (sample, direction), no LDS and no barrier; the neighbouring column arrives by a lane shift.
__global__ __launch_bounds__(64) void k_lattice_wave(SampleTable st, LatticeState ls, int s0,
                                                     float* __restrict__ loss) {
    const int s = s0 + blockIdx.x;
    const bool is_beta = (blockIdx.y != 0);
    const int u = threadIdx.x;
    const int T = st.T[s], U = st.U[s], W1 = U + 1;
    const long long base = st.row_off[s] - ls.row_base;
    const float* __restrict__ lpb = ls.lpb + base;
    const float* __restrict__ lpy = ls.lpy + base;
    const int n = T * W1;
    const float c = -wave_sum(emission_max_partial(lpb, lpy, n, W1, U, u, 64)) / (float)n;
    const bool col = (u <= U);
    const int nsteps = T + U;
    float own = RNNT_NEG_INF;
    float pb[LAT_PF], py[LAT_PF];
    if (!is_beta) {
        float* __restrict__ alpha = ls.alpha + base;
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
                    const float left = __shfl_up(own, 1, 64);       // column u-1, previous step
                    if (act) {
                        float val = 0.0f;
                        if (k != 0) {
                            const float a = (t > 0) ? own + (pb[i] + c) : RNNT_NEG_INF;
                            const float b = (u > 0) ? left + (py[i] + c) : RNNT_NEG_INF;
                            val = log_add_exp(a, b);
                        }
                        alpha[t * W1 + u] = val;
                        own = val;
                    }
                    fetch(k + LAT_PF, pb[i], py[i]);
                }
            }
        }
        if (u == U) {
            const float lnP_off = own + (lpb[(T - 1) * W1 + U] + c);
            ls.lnP[s] = lnP_off;
            ls.shift[s] = c;
            loss[s] = -(lnP_off - c * (float)(T + U));
        }
    } else {
        float* __restrict__ beta = ls.beta + base;
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
                    const float right = __shfl_down(own, 1, 64);    // column u+1, previous step
                    if (act) {
                        float val = pb[i] + c;                      // k == 0: beta[T-1,U] = final blank
                        if (k != 0) {
                            const float a = (t < T - 1) ? own + (pb[i] + c) : RNNT_NEG_INF;
                            const float b = (u < U) ? right + (py[i] + c) : RNNT_NEG_INF;
                            val = log_add_exp(a, b);
                        }
                        beta[t * W1 + u] = val;
                        own = val;
                    }
                    fetch(k + LAT_PF, pb[i], py[i]);
                }
            }
        }
    }
}

hipError_t launch_lattice(const SampleTable& st, const LatticeState& ls, int s0, int s1, int u_max, float* loss,
                          hipStream_t stream) {
    if (s1 <= s0) return hipSuccess;
    if (u_max + 1 <= 64) {
        k_lattice_wave<<<dim3((unsigned)(s1 - s0), 2), dim3(64), 0, stream>>>(st, ls, s0, loss);
        return hipGetLastError();
    }
    int threads = ((u_max + 1) + 63) / 64 * 64;
    if (threads > LAT_MAX_T) return hipErrorInvalidValue;
    k_lattice<<<dim3((unsigned)(s1 - s0), 2), dim3(threads), 0, stream>>>(st, ls, s0, loss);
    return hipGetLastError();
}

}  // namespace rnnt
