// Fused backward kernel of the bf16 MFMA path (gfx950): for one lattice tile (64 rows: 8 frames x 8 label positions, or 16 x 4)
//   joint tile z = tanh(enc_t + pred_u) in LDS                                  (Eq. 4)
//   scores recomputed on MFMA, dh = gamma * softmax - posteriors               (Eq. 6, f^W_4)
//   dz = dh W_out^T accumulated over the whole vocabulary in registers           (Alg. 1 lines 10, 11)
//   dx = dz (1 - z^2), summed over the tile's label positions / frames, added to d_enc / d_pred
// and dh (bf16) plus z (bf16) written out row-major, straight from their LDS tiles, for the dW_out
// GEMM.  The score gradient is not re-read for dz.
//
// 512 threads = 8 waves, one workgroup per CU, two waves per SIMD with different jobs:
//  waves 0..3 ("score waves"): per step of 256 vocabulary entries, wave w owns entries [64w, 64w+64) for
//   all 64 rows (2 x 2 accumulator tiles, A = packed W_out^T fragments from L2, B = joint tile from LDS),
//   turns the scores into dh (exp, bf16) and lays its 64 x 64 piece down in one of two LDS buffers
//   [64][256], then copies that piece to the dH chunk buffer;
//  waves 4..7 ("dz waves"): one step behind, multiply the finished buffer into their own hidden columns
//   (hidden 32-tiles w-4, w, w+4, ...: A = dh from LDS (rows), B = packed W_out fragments from L2
//   (hidden x vocabulary)), and run the epilogue.
// The vector-ALU work of a wave never overlaps with that wave's own MFMAs, but it does overlap with the
// MFMAs of the other wave on its SIMD: while a score wave computes exponentials, the dz wave next to it
// keeps the matrix pipe busy.  One workgroup barrier per step separates writers and readers of a buffer.
// MFMA operand layouts: see kernels_bf16.hip.
#include <type_traits>

#include "device_common.h"

namespace rnnt {

constexpr int FB_ROWS = 64;
constexpr int FB_VSTEP = 256;         // vocabulary entries per step
constexpr int FB_DP = FB_VSTEP + 8;   // pitch (bf16 elements) of a dh LDS buffer [64 rows][256 entries]

struct FusedArgs {
    Problem pr;
    SampleTable st;
    LatticeState ls;
    const bf16_t* Wp;   // fragment-major W_out^T (score waves)
    const bf16_t* Wq;   // fragment-major W_out   (dz waves)
    int s0, s1, tile0, tile1;
    bf16_t* dH;         // [chunk rows, V]
    bf16_t* Z;          // [chunk rows, H]
    float* d_enc;
    float* d_pred;
    const float* kept_max;   // KEPT: running maxima of the kept scores, [chunk tiles][V/64][64 rows]
    ActiveTiles at;          // which tiles this launch works on (see kernels.h)
};

// HT = hidden 32-tiles per dz wave = ceil(H / 128); FB_PF = fragment prefetch distance of the score loop in
// k16-steps (H/16 must be a multiple of 2*FB_PF); PB = the same for the dz loop.
// KEPT: the forward pass has kept the scores (dH holds them as fp16 differences t to the running maxima
// kept_max, Z the joint tile): the score waves then only read their 64 x 64 piece of t, turn it into dh
// (one exponential per element), lay it into the LDS buffer and write it back over t for the dW_out GEMM;
// no score MFMAs, no copy-out of Z.
template <int HT, int FB_PF, int PB, bool KEPT>
__global__ __launch_bounds__(512) void k_joint_bwd_fused(FusedArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int H = a.pr.H, V = a.pr.V;
    const int ZP = H + 8;
    bf16_t* zs = reinterpret_cast<bf16_t*>(smem);                        // [64][ZP]
    bf16_t* dhs = zs + (size_t)FB_ROWS * ZP;                             // [2][64][FB_DP]
    int* row_lab = reinterpret_cast<int*>(dhs + 2 * FB_ROWS * FB_DP);    // [64]
    float* row_g = reinterpret_cast<float*>(row_lab + 64);               // [64] exponent offset (log2 units)
    float* row_B = row_g + 64;                                           // [64] dh at the blank entry
    float* row_Y = row_B + 64;                                           // [64] dh at the label entry

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hb = lane >> 5;
    int tile = a.tile0 + blockIdx.x;
    if (a.at.active) {
        // listed tiles only: entry cbase + blockIdx.x of the group's list, if there is one (uniform per workgroup)
        const int ci = a.at.cbase + (int)blockIdx.x;
        if (ci >= *a.at.n_active) return;
        tile = a.at.active[a.at.group_tile0 + ci];
    }
    const TilePos tp = locate_tile(a.st, a.s0, a.s1, tile);
    const int b = tp.s;
    // the tile's 64 rows in the chunk buffers: dense, or by tile position where the forward pass has filled them
    const int slot = (a.at.active && a.at.slot_tile0 >= 0) ? tile - a.at.slot_tile0 : (int)blockIdx.x;
    const long long chunk_row0 = (long long)slot * FB_ROWS;

    // ---- joint tile (Eq. 4)
    build_joint_tile<512, 2>(zs, ZP, reinterpret_cast<const bf16_t*>(a.pr.enc) + (size_t)b * a.pr.T_max * H,
                             reinterpret_cast<const bf16_t*>(a.pr.pred) + (size_t)b * (a.pr.U_max + 1) * H, H, tp, tid);
    if (tid < 64) {
        const int r = tid;
        const int t = tp.t0 + (r >> tp.us), u = tp.u0 + (r & (tp.uw - 1));
        const bool valid = (t < tp.T && u <= tp.U);
        row_lab[r] = (valid && u < tp.U) ? a.pr.labels[(size_t)b * a.pr.U_max + u] : -1;
        if (valid) {
            const long long idx = (a.st.row_off[b] - a.ls.row_base) + (long long)t * (tp.U + 1) + u;
            // dh = gamma * softmax - posteriors differs from gamma * softmax at two entries of the row
            // only; their final values follow from the stored log-probabilities, so the per-element
            // path below needs no indicator logic: the owning lane overwrites those two entries.
            const RowPost rp = row_posteriors(a.ls, idx, t, u, tp.T, tp.U, b);
            row_g[r] = (rp.log_gamma - a.ls.lse[idx]) * LOG2E_F;
            const int y = row_lab[r];
            const float both = (y == a.pr.blank) ? 1.0f : 0.0f;
            row_B[r] = __expf(rp.log_gamma + a.ls.lpb[idx]) - rp.Bk - both * rp.Yk;
            row_Y[r] = (y >= 0) ? __expf(rp.log_gamma + a.ls.lpy[idx]) - rp.Yk - both * rp.Bk : 0.0f;
        } else {
            row_g[r] = RNNT_NEG_INF;
            row_B[r] = 0.0f;
            row_Y[r] = 0.0f;
        }
    }
    __syncthreads();

    const int KK = H >> 4;             // k16-steps of the score GEMM
    const int VK = V >> 4;             // k16-steps of the dz GEMM (whole vocabulary)
    const int nht = H >> 5;            // hidden 32-tiles
    const int nvs = V / FB_VSTEP;
    const int w4 = __builtin_amdgcn_readfirstlane(wave & 3);
    const unsigned lane_b = (unsigned)lane * 16u;

    if (KEPT && wave < 4) {
        // =========================== score waves, scores kept ===========================
        typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
        const int seg = lane & 7, r0 = lane >> 3;          // rows r0 + 8 i, eight entries at 64 w4 + 8 seg
        const size_t DL = chunk_pitch(V);
        bf16_t* piece = a.dH + (size_t)chunk_row0 * DL + w4 * 64 + seg * 8;
        const float* mx = a.kept_max + ((size_t)slot * (V / 64) + w4) * 64;
        float g[8], vB[8], vY[8];
        int lb[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = r0 + 8 * i;
            g[i] = row_g[row];
            vB[i] = row_B[row];
            vY[i] = row_Y[row];
            lb[i] = row_lab[row];
        }
        f16x8 tn[8];
        float mn[8];
        auto fetch = [&](int step) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = r0 + 8 * i;
                tn[i] = __builtin_nontemporal_load(reinterpret_cast<const f16x8*>(piece + (size_t)row * DL + step * FB_VSTEP));
                mn[i] = mx[(size_t)step * 4 * 64 + row];
            }
        };
        fetch(0);
        for (int vs = 0; vs < nvs; ++vs) {
            bf16_t* buf = dhs + (vs & 1) * (FB_ROWS * FB_DP);
            f16x8 t[8];
            float e[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                t[i] = tn[i];
                e[i] = fmaf(mn[i], LOG2E_F, g[i]);
            }
            fetch(vs + 1 < nvs ? vs + 1 : vs);             // one step ahead (the last step reads its own again)
            const int cbase = vs * FB_VSTEP + w4 * 64 + seg * 8;
            const int relb = a.pr.blank - cbase;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = r0 + 8 * i;
                float d[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) d[k] = __builtin_amdgcn_exp2f(fmaf((float)t[i][k], LOG2E_F, e[i]));
                // the blank / label entry of the row takes its final value from the stored log-probabilities
                const int rely = lb[i] - cbase;
                if ((unsigned)relb < 8u || (unsigned)rely < 8u) {
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        if (k == relb) d[k] = vB[i];
                        if (k == rely) d[k] = vY[i];
                    }
                }
                bf16x8 o;
#pragma unroll
                for (int k = 0; k < 8; ++k) o[k] = (bf16_t)d[k];
                *reinterpret_cast<bf16x8*>(buf + row * FB_DP + w4 * 64 + seg * 8) = o;
                __builtin_nontemporal_store(o, reinterpret_cast<bf16x8*>(piece + (size_t)row * DL + vs * FB_VSTEP));
            }
            __syncthreads();    // barrier vs: this step's buffer is complete
        }
        return;
    }
    if (!KEPT && wave < 4) {
        // =========================== score waves ===========================
        const int nkb = KK / FB_PF;
        const int lab[2] = {row_lab[l32], row_lab[32 + l32]};
        const float gexp[2] = {row_g[l32], row_g[32 + l32]};
        const float Bk[2] = {row_B[l32], row_B[32 + l32]};
        const float Yk[2] = {row_Y[l32], row_Y[32 + l32]};
        const bf16_t* zrow0 = zs + l32 * ZP + hb * 8;
        const bf16_t* zrow1 = zs + (32 + l32) * ZP + hb * 8;
        const char* wpb = reinterpret_cast<const char*>(a.Wp);
        // A operand (W_out^T, vocabulary x hidden): fragment (vt, kk) at ((vt*KK + kk)*1024) bytes
        auto wp_off = [&](int vs_, int vt_, int kb_) -> size_t {
            return ((size_t)(vs_ * (FB_VSTEP / 32) + w4 * 2 + vt_) * KK + (size_t)kb_ * FB_PF) * 1024;
        };
        auto wp_load = [&](size_t off, int j) { return *reinterpret_cast<const bf16x8*>(wpb + off + j * 1024 + lane_b); };

        // The first fragment block and the bias of a step are fetched while the step before is still busy with
        // its exponentials and its copy-out (at the start of a step nothing else would hide their way from the L2).
        bf16x8 ringA[2][2][FB_PF];
        f32x4 bias_next[2][4];
        auto load_bias = [&](int vs_) {
#pragma unroll
            for (int vt = 0; vt < 2; ++vt) {
                const float* bp = a.pr.b_out + vs_ * FB_VSTEP + w4 * 64 + vt * 32 + 4 * hb;
#pragma unroll
                for (int j = 0; j < 4; ++j) bias_next[vt][j] = *reinterpret_cast<const f32x4*>(bp + 8 * j);
            }
        };
#pragma unroll
        for (int vt = 0; vt < 2; ++vt)
#pragma unroll
            for (int j = 0; j < FB_PF; ++j) ringA[0][vt][j] = wp_load(wp_off(0, vt, 0), j);
        load_bias(0);
        for (int vs = 0; vs < nvs; ++vs) {
            bf16_t* buf = dhs + (vs & 1) * (FB_ROWS * FB_DP);
            // -------- scores of 64 entries x 64 rows; accumulators start from the bias
            f32x16 acc[2][2];
#pragma unroll
            for (int vt = 0; vt < 2; ++vt)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        acc[vt][0][4 * j + i] = bias_next[vt][j][i];
                        acc[vt][1][4 * j + i] = bias_next[vt][j][i];
                    }
            bf16x8 bc[2] = {*reinterpret_cast<const bf16x8*>(zrow0), *reinterpret_cast<const bf16x8*>(zrow1)};
            const bf16_t* zc0 = zrow0;
            const bf16_t* zc1 = zrow1;
            __builtin_amdgcn_s_setprio(2);
            for (int kb2 = 0; kb2 < nkb; kb2 += 2) {
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int kb = kb2 + half;
                    const int cs = half, ns = half ^ 1;
                    // next block of this step, else the first block of the next step (of this one again at the end)
                    int nvs_ = vs, nkb_ = kb + 1;
                    if (nkb_ == nkb) { nkb_ = 0; nvs_ = (vs + 1 < nvs) ? vs + 1 : vs; }
                    const size_t noff0 = wp_off(nvs_, 0, nkb_), noff1 = wp_off(nvs_, 1, nkb_);
                    const int knext = (kb + 1 == nkb) ? 0 : (kb + 1) * FB_PF * 16;
                    const bf16_t* zn0 = zrow0 + knext;
                    const bf16_t* zn1 = zrow1 + knext;
#pragma unroll
                    for (int j = 0; j < FB_PF; ++j) {
                        bf16x8 bn[2];
                        if (j + 1 < FB_PF) {
                            bn[0] = *reinterpret_cast<const bf16x8*>(zc0 + (j + 1) * 16);
                            bn[1] = *reinterpret_cast<const bf16x8*>(zc1 + (j + 1) * 16);
                        } else {
                            bn[0] = *reinterpret_cast<const bf16x8*>(zn0);
                            bn[1] = *reinterpret_cast<const bf16x8*>(zn1);
                        }
                        ringA[ns][0][j] = wp_load(noff0, j);
                        ringA[ns][1][j] = wp_load(noff1, j);
                        __builtin_amdgcn_sched_barrier(0);
                        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ringA[cs][0][j], bc[0], acc[0][0], 0, 0, 0);
                        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ringA[cs][0][j], bc[1], acc[0][1], 0, 0, 0);
                        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ringA[cs][1][j], bc[0], acc[1][0], 0, 0, 0);
                        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ringA[cs][1][j], bc[1], acc[1][1], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        bc[0] = bn[0];
                        bc[1] = bn[1];
                    }
                    zc0 = zn0;
                    zc1 = zn1;
                }
            }
            __builtin_amdgcn_s_setprio(0);
            load_bias(vs + 1 < nvs ? vs + 1 : vs);
            // -------- f^W_4: dh = gamma * softmax - posteriors, to bf16, into this step's LDS buffer (row-major).
            //          The dz waves read the other buffer meanwhile; they left this one before the last barrier.
#pragma unroll
            for (int vt = 0; vt < 2; ++vt) {
                const int vbase = vs * FB_VSTEP + w4 * 64 + vt * 32;
                const int relb = a.pr.blank - vbase;
#pragma unroll
                for (int rt = 0; rt < 2; ++rt) {
                    const int rely = lab[rt] - vbase;
                    float d[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        d[i] = __builtin_amdgcn_exp2f(fmaf(acc[vt][rt][i], LOG2E_F, gexp[rt]));
                    bf16_t* sd = buf + (rt * 32 + l32) * FB_DP + w4 * 64 + vt * 32 + 4 * hb;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        bf16x4 q4 = {(bf16_t)d[4 * j], (bf16_t)d[4 * j + 1], (bf16_t)d[4 * j + 2], (bf16_t)d[4 * j + 3]};
                        *reinterpret_cast<bf16x4*>(sd + 8 * j) = q4;
                    }
                    // the lane that holds the blank / label entry of its row overwrites it (same lane,
                    // same address, program order): entry rel lives in lane half (rel/4)%2
                    const bool own_b = ((unsigned)relb < 32u) && (((relb >> 2) & 1) == hb);
                    const bool own_y = ((unsigned)rely < 32u) && (((rely >> 2) & 1) == hb);
                    if (own_b) {
                        const bf16_t v = (bf16_t)Bk[rt];
                        buf[(rt * 32 + l32) * FB_DP + w4 * 64 + vt * 32 + relb] = v;
                    }
                    if (own_y) {
                        const bf16_t v = (bf16_t)Yk[rt];
                        buf[(rt * 32 + l32) * FB_DP + w4 * 64 + vt * 32 + rely] = v;
                    }
                }
            }
            // this wave's 64 x 64 piece -> dH chunk buffer (row-major; 8 lanes store the 128 bytes of a row).
            // LDS operations of one wave execute in order, so the piece is complete for its own wave.
            {
                const int seg = lane & 7, r0 = lane >> 3;
                const size_t DL = chunk_pitch(V);
                bf16_t* o = a.dH + (size_t)chunk_row0 * DL + vs * FB_VSTEP + w4 * 64 + seg * 8;
                const bf16_t* src = buf + w4 * 64 + seg * 8;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int row = r0 + 8 * i;
                    __builtin_nontemporal_store(*reinterpret_cast<const bf16x8*>(src + row * FB_DP),
                                                reinterpret_cast<bf16x8*>(o + (size_t)row * DL));
                }
            }
            __syncthreads();    // barrier vs: this step's buffer is complete
        }
        return;
    }

    // =========================== dz waves ===========================
    // joint tile -> Z chunk buffer (row-major, coalesced 16-byte stores) for the dW GEMM, while the score
    // waves work on the first step
    if (!KEPT) {
        const int t4 = tid - 256;
        const int cpr = H >> 3;                              // 16-byte chunks per row
        const int drow = 256 / cpr, dch = 256 - drow * cpr;
        int row = t4 / cpr, ch = t4 - row * cpr;
        const size_t ZL = chunk_pitch(H);
        bf16_t* zo = a.Z + (size_t)chunk_row0 * ZL;
        while (row < FB_ROWS) {
            __builtin_nontemporal_store(*reinterpret_cast<const bf16x8*>(zs + row * ZP + ch * 8),
                                        reinterpret_cast<bf16x8*>(zo + (size_t)row * ZL + ch * 8));
            row += drow;
            ch += dch;
            if (ch >= cpr) { ch -= cpr; ++row; }
        }
    }
    // dz accumulators: hidden tiles w4, w4+4, ... (HT of them at most), two row tiles
    f32x16 dz[HT][2];
#pragma unroll
    for (int i = 0; i < HT; ++i)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) dz[i][rt] = f32x16{0};
    const char* wqb = reinterpret_cast<const char*>(a.Wq);
    // B operand (W_out, hidden x vocabulary): fragment (ht, vk) at ((ht*VK + vk)*1024) bytes
    auto wq_off = [&](int i, int vk) -> size_t {
        int ht = w4 + 4 * i;
        if (ht >= nht) ht = w4;        // unused slot: any valid fragment
        return ((size_t)ht * VK + vk) * 1024;
    };
    auto wq_load = [&](size_t off, int j) { return *reinterpret_cast<const bf16x8*>(wqb + off + j * 1024 + lane_b); };
    constexpr int NB2 = (FB_VSTEP / 16) / PB;  // fragment blocks per step (even)
    bf16x8 ringB[2][HT][PB];
#pragma unroll
    for (int i = 0; i < HT; ++i)
#pragma unroll
        for (int kk = 0; kk < PB; ++kk) ringB[0][i][kk] = wq_load(wq_off(i, 0), kk);
    __syncthreads();    // barrier 0: the first buffer is complete

    for (int s = 0; s < nvs; ++s) {
        // -------- dz += dh W^T over the 256 vocabulary entries of step s
        const bf16_t* buf = dhs + (s & 1) * (FB_ROWS * FB_DP);
        const bf16_t* drow0 = buf + l32 * FB_DP + hb * 8;
        const bf16_t* drow1 = buf + (32 + l32) * FB_DP + hb * 8;
        const int vk0 = s * (FB_VSTEP / 16);
        bf16x8 ac[2] = {*reinterpret_cast<const bf16x8*>(drow0), *reinterpret_cast<const bf16x8*>(drow1)};
        const bf16_t* dc0 = drow0;
        const bf16_t* dc1 = drow1;
        __builtin_amdgcn_s_setprio(1);
        for (int kb2 = 0; kb2 < NB2; kb2 += 2) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int kb = kb2 + half;
                const int cs = half, ns = half ^ 1;
                // next block of B fragments: next block of this step, else first block of the next step
                int vkn = vk0 + (kb + 1) * PB;
                if (vkn >= VK) vkn = vk0 + kb * PB;
                size_t noff[HT];
#pragma unroll
                for (int i = 0; i < HT; ++i) noff[i] = wq_off(i, vkn);
                const int knext = (kb + 1 == NB2) ? 0 : (kb + 1) * PB * 16;
                const bf16_t* dn0 = drow0 + knext;
                const bf16_t* dn1 = drow1 + knext;
#pragma unroll
                for (int j = 0; j < PB; ++j) {
                    bf16x8 an[2];
                    if (j + 1 < PB) {
                        an[0] = *reinterpret_cast<const bf16x8*>(dc0 + (j + 1) * 16);
                        an[1] = *reinterpret_cast<const bf16x8*>(dc1 + (j + 1) * 16);
                    } else {
                        an[0] = *reinterpret_cast<const bf16x8*>(dn0);
                        an[1] = *reinterpret_cast<const bf16x8*>(dn1);
                    }
#pragma unroll
                    for (int i = 0; i < HT; ++i) ringB[ns][i][j] = wq_load(noff[i], j);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < HT; ++i) {
                        dz[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ac[0], ringB[cs][i][j], dz[i][0], 0, 0, 0);
                        dz[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ac[1], ringB[cs][i][j], dz[i][1], 0, 0, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    ac[0] = an[0];
                    ac[1] = an[1];
                }
                dc0 = dn0;
                dc1 = dn1;
            }
        }
        __builtin_amdgcn_s_setprio(0);
        if (s + 1 < nvs) __syncthreads();   // barrier s+1: the next buffer is complete, this one may be rewritten
    }

    // ---- Alg. 1 lines 10, 11: dx = dz (1 - z^2); sum over label positions -> d_enc, over frames -> d_pred.
    // Accumulator register 4j+i of row tile rt is tile row r = 32 rt + 8j + 4 hb + i: in an 8 x 8 tile frame
    // 4 rt + j, label 4 hb + i (a frame's eight labels are spread over the two lane halves); in a 16 x 4 tile frame
    // 8 rt + 2j + hb, label i (a label's sixteen frames are).
    {
        float* d_enc = a.d_enc + (size_t)b * a.pr.T_max * H;
        float* d_prd = a.d_pred + (size_t)b * (a.pr.U_max + 1) * H;
        // one copy of the loop nest per tile shape (the shape is the same for the whole workgroup)
        auto reduce = [&](auto wide_tag) {
            constexpr bool WIDE = decltype(wide_tag)::value;
#pragma unroll
            for (int i = 0; i < HT; ++i) {
                const int ht = w4 + 4 * i;
                if (ht >= nht) continue;
                const int h = ht * 32 + l32;
                float pu[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        float se = 0.0f;
#pragma unroll
                        for (int ii = 0; ii < 4; ++ii) {
                            const int r = rt * 32 + 8 * j + 4 * hb + ii;
                            const float z = (float)zs[r * ZP + h];
                            const float dx = dz[i][rt][4 * j + ii] * (1.0f - z * z);
                            se += dx;
                            pu[ii] += dx;
                        }
                        if (WIDE) {
                            const int tl = 4 * rt + j;
                            se += __shfl_xor(se, 32, 64);
                            if (hb == (j & 1) && tp.t0 + tl < tp.T) atomicAdd(&d_enc[(size_t)(tp.t0 + tl) * H + h], se);
                        } else {
                            const int t16 = tp.t0 + 8 * rt + 2 * j + hb;
                            if (t16 < tp.T) atomicAdd(&d_enc[(size_t)t16 * H + h], se);
                        }
                    }
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) {
                    if (WIDE) {
                        if (tp.u0 + 4 * hb + ii <= tp.U) atomicAdd(&d_prd[(size_t)(tp.u0 + 4 * hb + ii) * H + h], pu[ii]);
                    } else {
                        const float both = pu[ii] + __shfl_xor(pu[ii], 32, 64);
                        if (hb == (ii & 1) && tp.u0 + ii <= tp.U) atomicAdd(&d_prd[(size_t)(tp.u0 + ii) * H + h], both);
                    }
                }
            }
        };
        if (tp.uw == 8) reduce(std::true_type{});
        else reduce(std::false_type{});
    }
}

static size_t fused_smem_bytes(int H) {
    return (size_t)FB_ROWS * (H + 8) * 2 + (size_t)2 * FB_ROWS * FB_DP * 2 + 64 * 4 * 4;
}

template <int HT, int FB_PF, int PB, bool KEPT>
static hipError_t launch_fused_t(const FusedArgs& a, hipStream_t stream) {
    const int n = a.tile1 - a.tile0;
    const size_t smem = fused_smem_bytes(a.pr.H);
    static size_t configured = 0;
    if (smem > configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_joint_bwd_fused<HT, FB_PF, PB, KEPT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        configured = smem;
    }
    k_joint_bwd_fused<HT, FB_PF, PB, KEPT><<<dim3((unsigned)n), dim3(512), smem, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_bwd_fused_bf16(const Problem& pr, const void* Wpack, const void* Wq, const SampleTable& st,
                                 const LatticeState& ls, int s0, int s1, int tile0, int tile1, void* dH, void* Z,
                                 float* d_enc, float* d_pred, const ActiveTiles& at, hipStream_t stream) {
    if (tile1 <= tile0) return hipSuccess;
    FusedArgs a{pr, st, ls, (const bf16_t*)Wpack, (const bf16_t*)Wq, s0, s1, tile0, tile1,
                (bf16_t*)dH, (bf16_t*)Z, d_enc, d_pred, nullptr, at};
    const int ht = (pr.H / 32 + 3) / 4;
    // H = 128 ... 640 in steps of 128: H/16 = 8, 16, 24, 32, 40 k16-steps
    if (ht <= 1) return launch_fused_t<1, 4, 4, false>(a, stream);
    if (ht == 2) return launch_fused_t<2, 8, 4, false>(a, stream);
    if (ht == 3) return launch_fused_t<3, 4, 2, false>(a, stream);
    if (ht == 4) return launch_fused_t<4, 4, 2, false>(a, stream);    // (4, 4, 2) measured 1 % ahead of (4, 8, 2)
    if (ht == 5) return launch_fused_t<5, 4, 1, false>(a, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_bwd_fused_kept_bf16(const Problem& pr, const void* Wq, const SampleTable& st, const LatticeState& ls,
                                      int s0, int s1, int tile0, int tile1, void* kept, const float* kept_max,
                                      float* d_enc, float* d_pred, const ActiveTiles& at, hipStream_t stream) {
    if (tile1 <= tile0) return hipSuccess;
    FusedArgs a{pr, st, ls, nullptr, (const bf16_t*)Wq, s0, s1, tile0, tile1,
                (bf16_t*)kept, nullptr, d_enc, d_pred, kept_max, at};
    const int ht = (pr.H / 32 + 3) / 4;
    if (ht <= 1) return launch_fused_t<1, 4, 4, true>(a, stream);
    if (ht == 2) return launch_fused_t<2, 8, 4, true>(a, stream);
    if (ht == 3) return launch_fused_t<3, 4, 2, true>(a, stream);
    if (ht == 4) return launch_fused_t<4, 8, 2, true>(a, stream);
    if (ht == 5) return launch_fused_t<5, 4, 1, true>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace rnnt
