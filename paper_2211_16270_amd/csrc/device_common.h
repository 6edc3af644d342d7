// Device helpers shared by the HIP kernels of this library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace rnnt {

constexpr float LOG2E_F = 1.4426950408889634f;
constexpr float LN2_F = 0.6931471805599453f;
#define RNNT_NEG_INF (-__builtin_huge_valf())
// s_waitcnt operand (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14]) that waits for
// every outstanding LDS / scalar-memory operation of the wave and for nothing else.
constexpr int WAIT_LGKM0 = 0xC07F;

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Largest s in [lo, hi) with off[s] <= x  (off is non-decreasing, off[lo] <= x < off[hi]).
template <typename T>
__device__ __forceinline__ int find_segment(const T* __restrict__ off, int lo, int hi, T x) {
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (off[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// Position of a lattice tile: sample, first frame, first label position, and the sample's tile shape
// (uw = 8 or 4 label positions, us = log2 uw; row r of the tile is frame t0 + (r >> us), label u0 + (r & (uw-1))).
struct TilePos {
    int s, T, U, t0, u0, uw, us;
};

__device__ __forceinline__ TilePos locate_tile(const SampleTable& st, int s0, int s1, int tile) {
    TilePos p;
    (void)s0;
    (void)s1;
    p.s = st.tile_sample[tile];
    p.T = st.T[p.s];
    p.U = st.U[p.s];
    p.uw = tile_label_width(p.T, p.U);
    p.us = p.uw == 8 ? 3 : 2;
    const int tiles_u = (p.U + p.uw) >> p.us;     // ceil((U+1)/uw)
    const int lt = tile - st.tile_off[p.s];
    const int tb = lt / tiles_u;
    p.t0 = tb * (64 >> p.us);
    p.u0 = (lt - tb * tiles_u) << p.us;
    return p;
}

// tanh through one exp and one reciprocal; absolute error ~1e-7, saturates cleanly at +-1.
__device__ __forceinline__ float fast_tanh(float x) {
    float e = __builtin_amdgcn_exp2f(x * (2.0f * LOG2E_F));
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + e);
}

// Eight joint activations z = tanh(e + q), rounded to bf16; keep = 0 gives zeros, keep = ~0u the values
// (branch-free: a branch per element would cost more than the arithmetic).
__device__ __forceinline__ bf16x8 joint_tanh8(bf16x8 e, bf16x8 q, unsigned keep) {
    typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
    bf16x8 z;
#pragma unroll
    for (int j = 0; j < 8; ++j) z[j] = (bf16_t)fast_tanh((float)e[j] + (float)q[j]);
    u32x4_t w = __builtin_bit_cast(u32x4_t, z);
    w &= keep;
    return __builtin_bit_cast(bf16x8, w);
}

// The joint tile of a lattice tile (Eq. 4): zs[uw tl + ul][h] = tanh(enc[t0 + tl][h] + pred[u0 + ul][h]), bf16, row
// pitch ZP, rows outside the sample zero (they read row 0 of their input).  enc / prd point at the sample's rows.
// tanh(x) = 1 - 2 / (e^{2x} + 1) and e^{2(e+q)} = e^{2e} e^{2q}: a thread takes one 8-column piece of TG frames
// and 4 label positions, forms the TG + 4 exponentials per column once and pays one reciprocal per element, half
// the transcendental instructions of a tanh per element (at 1024 vocabulary entries building this tile costs a
// third of the cycles of the tile's score MFMAs).  The product can neither overflow nor lose the small factor
// while both exponents stay inside +-115 (|input| <= 40); a thread that sees a larger input computes its
// elements from the sums instead.
template <int NT, int TG>
__device__ __forceinline__ void build_joint_tile(bf16_t* __restrict__ zs, int ZP, const bf16_t* __restrict__ enc,
                                                 const bf16_t* __restrict__ prd, int H, const TilePos& tp, int tid) {
    typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
    constexpr int UG = 4, NG = 16 / TG;          // 16 / TG groups of TG frames x 4 label positions for either shape
    constexpr float K2 = 2.0f * LOG2E_F;
    const int cpr = H >> 3;
    const int nug = tp.uw >> 2;                  // groups side by side along the labels: 2 or 1
    for (int item = tid; item < cpr * NG; item += NT) {
        const int g = item / cpr, c = item - g * cpr;
        const int tl0 = (nug == 2 ? g >> 1 : g) * TG, ul0 = (nug == 2 ? g & 1 : 0) * UG;
        bf16x8 e[TG], q[UG];
#pragma unroll
        for (int i = 0; i < TG; ++i) {
            const int t = tp.t0 + tl0 + i;
            e[i] = *reinterpret_cast<const bf16x8*>(enc + (size_t)(t < tp.T ? t : 0) * H + c * 8);
        }
#pragma unroll
        for (int j = 0; j < UG; ++j) {
            const int u = tp.u0 + ul0 + j;
            q[j] = *reinterpret_cast<const bf16x8*>(prd + (size_t)(u <= tp.U ? u : 0) * H + c * 8);
        }
        float E[TG][8], Q[UG][8], big = 0.0f;
#pragma unroll
        for (int i = 0; i < TG; ++i)
#pragma unroll
            for (int k = 0; k < 8; k += 2) {
                const float a0 = (float)e[i][k] * K2, a1 = (float)e[i][k + 1] * K2;
                big = fmaxf(big, fmaxf(fabsf(a0), fabsf(a1)));
                E[i][k] = __builtin_amdgcn_exp2f(a0);
                E[i][k + 1] = __builtin_amdgcn_exp2f(a1);
            }
#pragma unroll
        for (int j = 0; j < UG; ++j)
#pragma unroll
            for (int k = 0; k < 8; k += 2) {
                const float a0 = (float)q[j][k] * K2, a1 = (float)q[j][k + 1] * K2;
                big = fmaxf(big, fmaxf(fabsf(a0), fabsf(a1)));
                Q[j][k] = __builtin_amdgcn_exp2f(a0);
                Q[j][k + 1] = __builtin_amdgcn_exp2f(a1);
            }
        const bool by_product = (big <= 115.0f);
#pragma unroll
        for (int i = 0; i < TG; ++i)
#pragma unroll
            for (int j = 0; j < UG; ++j) {
                const bool valid = (tp.t0 + tl0 + i < tp.T) && (tp.u0 + ul0 + j <= tp.U);
                bf16x8 z;
                if (by_product) {
#pragma unroll
                    for (int k = 0; k < 8; ++k)
                        z[k] = (bf16_t)(1.0f - 2.0f * __builtin_amdgcn_rcpf(fmaf(E[i][k], Q[j][k], 1.0f)));
                } else {
#pragma unroll
                    for (int k = 0; k < 8; ++k) z[k] = (bf16_t)fast_tanh((float)e[i][k] + (float)q[j][k]);
                }
                u32x4_t w = __builtin_bit_cast(u32x4_t, z);
                w &= valid ? ~0u : 0u;
                *reinterpret_cast<u32x4_t*>(zs + (((tl0 + i) << tp.us) + ul0 + j) * ZP + c * 8) = w;
            }
    }
}

// ln(e^a + e^b); either may be -inf.
__device__ __forceinline__ float log_add_exp(float a, float b) {
    float m = fmaxf(a, b);
    if (m == RNNT_NEG_INF) return m;
    float d = -fabsf(a - b);                      // -inf when exactly one is -inf
    return m + __logf(1.0f + __expf(d));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Posterior weights of one lattice node (f^W_4): ln gamma, and the occupation of its blank and
// label transitions.  alpha/beta/lnP carry the per-sample emission offset `shift`, which cancels.
// With per-sample loss weights all three are those of w_s * loss_s.
struct RowPost {
    float log_gamma, Bk, Yk;
};
__device__ __forceinline__ RowPost row_posteriors(const LatticeState& ls, long long idx, int t, int u,
                                                   int T, int U, int s) {
    const float a = ls.alpha[idx], lnP = ls.lnP[s], c = ls.shift[s];
    RowPost r;
    r.log_gamma = a + ls.beta[idx] - lnP;
    const float ab = a + ls.lpb[idx] + c - lnP;
    if (t < T - 1) r.Bk = __expf(ab + ls.beta[idx + (U + 1)]);
    else r.Bk = (u == U) ? __expf(ab) : 0.0f;
    r.Yk = (u < U) ? __expf(a + ls.lpy[idx] + c - lnP + ls.beta[idx + 1]) : 0.0f;
    if (ls.weight) {
        // gradients of sum_b w_b loss_b: every posterior weight of sample s is scaled by w_s >= 0
        const float w = ls.weight[s];
        r.log_gamma += __logf(w);          // -inf for w = 0: the sample contributes nothing
        r.Bk *= w;
        r.Yk *= w;
    }
    return r;
}

// Asynchronous global -> LDS copy of 16 bytes per lane (global_load_lds_dwordx4): lane l's 16 bytes land
// at LDS byte address lds_base + 16*l (lds_base wave-uniform, passed in M0).  Completion is tracked by
// the wave's vmcnt counter; the compiler does not see these loads, so the waits are explicit below.
__device__ __forceinline__ void lds_dma16(const void* gptr, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_base) : "memory", "m0");
}
// The same with a wave-uniform 64-bit base (scalar registers) plus a 32-bit byte offset per lane.
__device__ __forceinline__ void lds_dma16_s(const void* sbase, unsigned voff, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base)
                 : "memory", "m0");
}

}  // namespace rnnt
