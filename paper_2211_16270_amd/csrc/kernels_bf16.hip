// bf16 MFMA path (gfx950): joint tile in LDS -> score GEMM -> softmax statistics / score gradients,
// and the two backward GEMMs.  fp32 accumulation everywhere; tanh, exp, softmax in fp32.
//
// Work unit: a lattice tile of one sample: 8 frames x 8 label positions = 64 rows, row r = 8*tl + ul, or
// 16 x 4 (r = 4*tl + ul) where that covers the sample with fewer tiles.  Such a tile needs only 8 + 8
// (16 + 4) input vectors, and its contribution to d_enc / d_pred can be summed over ul resp. tl before
// it leaves the registers.
//
// MFMA operand layouts used below (v_mfma_f32_32x32x16_bf16, D = A B + C, wave64):
//   A (32 x 16): lane l holds row l%32, k = 8*(l/32) .. +7        (8 bf16)
//   B (16 x 32): lane l holds column l%32, k = 8*(l/32) .. +7     (8 bf16)
//   C/D (32x32): lane l holds column l%32; register 4*j+i is row 8*j + 4*(l/32) + i
// The score GEMM is run "transposed" (A = W_out^T tile, B = joint tile), so a lane owns one
// lattice row and its 16 registers are 16 vocabulary entries: the softmax reductions over the
// vocabulary are then register-local.
#include "device_common.h"

namespace rnnt {

// ------------------------------------------------------------------------------------------------
// Joint tile + score GEMM.  MODE 0: softmax statistics (forward).  MODE 1: score gradients (backward).
// MODE 2: forward that also keeps what the backward pass would otherwise compute again: the joint tile
// (Z chunk buffer) and the scores, as fp16 differences t = h - m to a running maximum m (dH chunk buffer).
// m is the largest score the wave has seen so far in the row (its 64 of every 256 vocabulary entries), one
// float per row, wave and vocabulary step; t <= 0, so an entry's error exp(t) |t| 2^-11 in the softmax is
// at most 2^-11 / e whatever the size of the scores.
// NW waves; per step of 256 vocabulary entries wave w owns NVT tiles of 32 entries for all 64 rows
// (NVT x 2 accumulator tiles of 32x32).
// ------------------------------------------------------------------------------------------------
constexpr int JT_ROWS = 64;
constexpr int JT_VSTEP = 256;
constexpr int STG_PITCH = 40;   // bf16 elements per row of a wave's 32x32 transposition buffer
constexpr int STG2_PITCH = 72;  // the same for the 32x64 buffer of MODE 2 (whole 128-byte lines per row)

struct JointArgs {
    Problem pr;
    SampleTable st;
    LatticeState ls;
    const bf16_t* Wp;
    int s0, s1, tile0, tile1;
    // MODE 1, 2 outputs
    bf16_t* dH;     // [chunk rows, V]   (MODE 2: fp16 score differences)
    bf16_t* Z;      // [chunk rows, H]
    float* kept_max;  // MODE 2: [chunk tiles][V/64][64 rows] running maxima
    ActiveTiles at;   // MODE 1: which tiles the launch works on (see kernels.h); unused (null) otherwise
};


// JT_PF: A-fragment prefetch distance in k16-steps; H/16 must be an even multiple of it.
template <int MODE, int NW, int NVT, int JT_PF>
__global__ __launch_bounds__(64 * NW, 2) void k_joint_scores(JointArgs a) {
    static_assert(NW * NVT * 32 == JT_VSTEP, "waves x tiles must cover one vocabulary step");
    constexpr int NT = 64 * NW;
    extern __shared__ __align__(16) unsigned char smem[];
    const int H = a.pr.H, V = a.pr.V;
    const int ZP = H + 8;                                   // padded row pitch of the joint tile
    bf16_t* zs = reinterpret_cast<bf16_t*>(smem);           // [64][ZP]
    unsigned char* p_after = smem + (size_t)JT_ROWS * ZP * 2;
    int* row_lat = reinterpret_cast<int*>(p_after);         // [64] lattice index, -1 = outside the sample
    int* row_lab = row_lat + 64;                            // [64] label, -1 = none
    float* row_f0 = reinterpret_cast<float*>(row_lab + 64); // MODE 0: cap_b   MODE 1: exponent offset
    float* row_f1 = row_f0 + 64;                            // MODE 0: cap_y   MODE 1: Bk
    float* row_f2 = row_f1 + 64;                            // MODE 1: Yk
    float* red_m = row_f2 + 64;                             // MODE 0: [2 NW][64] partial maxima
    float* red_s = red_m + 2 * NW * 64;                     // MODE 0: [2 NW][64] partial sums
    // [NW][32][STG_PITCH] transposition buffers: MODE 1 aliases red_*, MODE 2 lies behind them
    bf16_t* stg = reinterpret_cast<bf16_t*>(MODE == 2 ? red_s + 2 * NW * 64 : row_f2 + 64);

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hb = lane >> 5;
    int tile = a.tile0 + blockIdx.x;
    if (MODE == 1 && a.at.active) {
        // listed tiles only: entry cbase + blockIdx.x of the group's list, if there is one (uniform per workgroup)
        const int ci = a.at.cbase + (int)blockIdx.x;
        if (ci >= *a.at.n_active) return;
        tile = a.at.active[a.at.group_tile0 + ci];
    }
    const TilePos tp = locate_tile(a.st, a.s0, a.s1, tile);
    const int b = tp.s;
    const long long chunk_row0 = (long long)blockIdx.x * JT_ROWS;

    // ---- joint tile: z = tanh(enc_t + pred_u), bf16, rows outside the sample are zero (Eq. 4)
    build_joint_tile<NT, (NT == 256 ? 4 : 2)>(zs, ZP, reinterpret_cast<const bf16_t*>(a.pr.enc) + (size_t)b * a.pr.T_max * H,
                                            reinterpret_cast<const bf16_t*>(a.pr.pred) + (size_t)b * (a.pr.U_max + 1) * H,
                                            H, tp, tid);
    if (tid < 64) {
        const int r = tid;
        const int t = tp.t0 + (r >> tp.us), u = tp.u0 + (r & (tp.uw - 1));
        const bool valid = (t < tp.T && u <= tp.U);
        const long long idx = (a.st.row_off[b] - a.ls.row_base) + (long long)t * (tp.U + 1) + u;
        row_lat[r] = valid ? (int)idx : -1;
        row_lab[r] = (valid && u < tp.U) ? a.pr.labels[(size_t)b * a.pr.U_max + u] : -1;
        if (MODE != 1) {
            row_f0[r] = RNNT_NEG_INF;
            row_f1[r] = RNNT_NEG_INF;
        } else {
            if (valid) {
                const RowPost rp = row_posteriors(a.ls, idx, t, u, tp.T, tp.U, b);
                row_f0[r] = (rp.log_gamma - a.ls.lse[idx]) * LOG2E_F;
                row_f1[r] = rp.Bk;
                row_f2[r] = rp.Yk;
            } else {
                row_f0[r] = RNNT_NEG_INF;
                row_f1[r] = 0.0f;
                row_f2[r] = 0.0f;
            }
        }
    }
    __syncthreads();
    if (MODE != 0) {
        // joint tile -> Z chunk buffer (row-major, coalesced 16-byte stores) for the dW GEMM
        const int cpr = H >> 3;
        for (int idx = tid; idx < JT_ROWS * cpr; idx += NT) {
            const int row = idx / cpr, ch = idx - row * cpr;
            *reinterpret_cast<bf16x8*>(a.Z + (size_t)(chunk_row0 + row) * chunk_pitch(H) + ch * 8) =
                *reinterpret_cast<const bf16x8*>(zs + row * ZP + ch * 8);
        }
    }

    const int KK = H >> 4;
    int lab[2] = {row_lab[l32], row_lab[32 + l32]};
    float m_run[2] = {RNNT_NEG_INF, RNNT_NEG_INF}, s_run[2] = {0.0f, 0.0f};
    float gexp[2], Bk[2], Yk[2];
    if (MODE == 1) {
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            gexp[rt] = row_f0[rt * 32 + l32];
            Bk[rt] = row_f1[rt * 32 + l32];
            Yk[rt] = row_f2[rt * 32 + l32];
        }
    }
    const bf16_t* zrow0 = zs + l32 * ZP + hb * 8;
    const bf16_t* zrow1 = zs + (32 + l32) * ZP + hb * 8;

    // Main loop.  Per step of 256 vocabulary entries wave w owns NVT tiles of 32 entries for all 64
    // rows (NVT x 2 accumulator tiles).  VALU instructions of a wave do not overlap with its own MFMAs on this
    // hardware, so the loop is written to contain almost none: A fragments (W_out^T) stream from L2
    // with scalar base + lane offset + immediate addressing into the register set that is not being
    // consumed (two sets, blocks of JT_PF k16-steps, one block ahead, possibly into the next
    // vocabulary step); B fragments (joint tile, LDS) are read one k16-step ahead with immediate
    // offsets from a per-block pointer.  Scheduling barriers keep the reads ahead of the MFMAs.
    const int nvs = V / JT_VSTEP;
    const int nkb = KK / JT_PF;                       // even: H is a multiple of 32*JT_PF
    const int wv = __builtin_amdgcn_readfirstlane(wave);
    const char* wpb = reinterpret_cast<const char*>(a.Wp);
    const unsigned lane_b = (unsigned)lane * 16u;
    auto block_off = [&](int vs_, int vt_, int kb_) -> size_t {
        return ((size_t)(vs_ * (JT_VSTEP / 32) + wv * NVT + vt_) * KK + (size_t)kb_ * JT_PF) * 1024;
    };
    auto load_frag = [&](size_t boff, int j) {
        return *reinterpret_cast<const bf16x8*>(wpb + boff + j * 1024 + lane_b);
    };
    bf16x8 ring[2][NVT][JT_PF];
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
        for (int j = 0; j < JT_PF; ++j) ring[0][vt][j] = load_frag(block_off(0, vt, 0), j);
    bf16x8 bc[2] = {*reinterpret_cast<const bf16x8*>(zrow0), *reinterpret_cast<const bf16x8*>(zrow1)};
    const bf16_t* zc0 = zrow0;                        // joint-tile pointers of the current block
    const bf16_t* zc1 = zrow1;

    for (int vs = 0; vs < nvs; ++vs) {
        // accumulators start from the bias of their 16 vocabulary entries: v = vbase + 8j + 4hb + i
        f32x16 acc[NVT][2];
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) {
            const float* bp = a.pr.b_out + vs * JT_VSTEP + wave * (32 * NVT) + vt * 32 + 4 * hb;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const f32x4 t4 = *reinterpret_cast<const f32x4*>(bp + 8 * j);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc[vt][0][4 * j + i] = t4[i];
                    acc[vt][1][4 * j + i] = t4[i];
                }
            }
        }
        for (int kb2 = 0; kb2 < nkb; kb2 += 2) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int kb = kb2 + half;
                const int cs = half, ns = half ^ 1;   // register sets: consumed / being filled
                int nvs_ = vs, nkb_ = kb + 1;
                if (nkb_ == nkb) { nkb_ = 0; nvs_ = vs + 1; }
                if (nvs_ == nvs) { nvs_ = vs; nkb_ = kb; }
                size_t noff[NVT];
#pragma unroll
                for (int vt = 0; vt < NVT; ++vt) noff[vt] = block_off(nvs_, vt, nkb_);
                const int knext = (kb + 1 == nkb) ? 0 : (kb + 1) * JT_PF * 16;
                const bf16_t* zn0 = zrow0 + knext;
                const bf16_t* zn1 = zrow1 + knext;
#pragma unroll
                for (int j = 0; j < JT_PF; ++j) {
                    bf16x8 bn[2];
                    if (j + 1 < JT_PF) {
                        bn[0] = *reinterpret_cast<const bf16x8*>(zc0 + (j + 1) * 16);
                        bn[1] = *reinterpret_cast<const bf16x8*>(zc1 + (j + 1) * 16);
                    } else {
                        bn[0] = *reinterpret_cast<const bf16x8*>(zn0);
                        bn[1] = *reinterpret_cast<const bf16x8*>(zn1);
                    }
#pragma unroll
                    for (int vt = 0; vt < NVT; ++vt) ring[ns][vt][j] = load_frag(noff[vt], j);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int vt = 0; vt < NVT; ++vt) {
                        acc[vt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[cs][vt][j], bc[0], acc[vt][0], 0, 0, 0);
                        acc[vt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[cs][vt][j], bc[1], acc[vt][1], 0, 0, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    bc[0] = bn[0];
                    bc[1] = bn[1];
                }
                zc0 = zn0;
                zc1 = zn1;
            }
        }
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) {
        const int vbase = vs * JT_VSTEP + wave * (32 * NVT) + vt * 32;
        const int relb = a.pr.blank - vbase;
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            const f32x16 accv = acc[vt][rt];
            const int rely = lab[rt] - vbase;
            const bool hit_y = ((unsigned)rely < 32u);
            const bool slow = __any(hit_y) || ((unsigned)relb < 32u);
            if (MODE != 1) {
                // f^W_1: running maximum and sum of exponentials of this lane's share of the row
                float x[16];
                float tmax = RNNT_NEG_INF;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    x[i] = accv[i];
                    tmax = fmaxf(tmax, x[i]);
                }
                const float mn = fmaxf(m_run[rt], tmax);
                const float mn2 = mn * LOG2E_F;
                float ssum = 0.0f;
#pragma unroll
                for (int i = 0; i < 16; ++i) ssum += __builtin_amdgcn_exp2f(fmaf(x[i], LOG2E_F, -mn2));
                s_run[rt] = s_run[rt] * __builtin_amdgcn_exp2f((m_run[rt] - mn) * LOG2E_F) + ssum;
                m_run[rt] = mn;
                if (slow) {
                    asm volatile("" ::: "memory");   // keep this rare path a real branch (no if-conversion)
                    float cb = RNNT_NEG_INF, cy = RNNT_NEG_INF;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int vloc = 8 * (i >> 2) + 4 * hb + (i & 3);
                        if (vloc == relb) cb = x[i];
                        if (vloc == rely) cy = x[i];
                    }
                    const int row = rt * 32 + l32;
                    if (cb != RNNT_NEG_INF) row_f0[row] = cb;
                    if (cy != RNNT_NEG_INF) row_f1[row] = cy;
                }
            } else {
                // f^W_4: dh = gamma * softmax - posteriors, rounded to bf16 for the backward GEMMs
                float d[16];
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    d[i] = __builtin_amdgcn_exp2f(fmaf(accv[i], LOG2E_F, gexp[rt]));
                if (slow) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int vloc = 8 * (i >> 2) + 4 * hb + (i & 3);
                        if (vloc == relb) d[i] -= Bk[rt];
                        if (vloc == rely) d[i] -= Yk[rt];
                    }
                }
                bf16_t dbf[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) dbf[i] = (bf16_t)d[i];
                // row-major copy dH[row][v] through this wave's 32x32 transposition buffer
                {
                    bf16_t* sw = stg + wave * (32 * STG_PITCH);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        bf16x4 q4 = {dbf[4 * j], dbf[4 * j + 1], dbf[4 * j + 2], dbf[4 * j + 3]};
                        *reinterpret_cast<bf16x4*>(sw + l32 * STG_PITCH + 8 * j + 4 * hb) = q4;
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                    for (int it = 0; it < 2; ++it) {
                        const int row = (lane >> 2) + 16 * it, seg = lane & 3;
                        const bf16x8 v8 = *reinterpret_cast<const bf16x8*>(sw + row * STG_PITCH + seg * 8);
                        *reinterpret_cast<bf16x8*>(a.dH + (size_t)(chunk_row0 + rt * 32 + row) * chunk_pitch(V) + vbase + seg * 8) = v8;
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                }
            }
        }
        }
        if (MODE == 2) {
            // keep the scores of this step: t = h - m (fp16), m = the wave's running maximum of the row
            typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
            static_assert(MODE != 2 || NVT == 2, "a wave keeps 64 vocabulary entries (one 128-byte line) per row");
            _Float16* sw = reinterpret_cast<_Float16*>(stg) + wave * (32 * STG2_PITCH);
            _Float16* kept = reinterpret_cast<_Float16*>(a.dH);
            const int vbase = vs * JT_VSTEP + wave * (32 * NVT);
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
                const float mw = fmaxf(m_run[rt], __shfl_xor(m_run[rt], 32, 64));
                if (hb == 0)
                    a.kept_max[((size_t)blockIdx.x * (V / 64) + vs * NW + wave) * 64 + rt * 32 + l32] = mw;
#pragma unroll
                for (int vt = 0; vt < NVT; ++vt) {
                    const f32x16 accv = acc[vt][rt];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        f16x4 q4 = {(_Float16)(accv[4 * j] - mw), (_Float16)(accv[4 * j + 1] - mw),
                                    (_Float16)(accv[4 * j + 2] - mw), (_Float16)(accv[4 * j + 3] - mw)};
                        *reinterpret_cast<f16x4*>(sw + l32 * STG2_PITCH + vt * 32 + 8 * j + 4 * hb) = q4;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                // eight lanes store one row's 128 bytes: whole lines only
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int row = (lane >> 3) + 8 * it, seg = lane & 7;
                    const bf16x8 v8 = *reinterpret_cast<const bf16x8*>(sw + row * STG2_PITCH + seg * 8);
                    __builtin_nontemporal_store(
                        v8, reinterpret_cast<bf16x8*>(kept + (size_t)(chunk_row0 + rt * 32 + row) * chunk_pitch(V) +
                                                      vbase + seg * 8));
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        }
    }

    if (MODE != 1) {
        // combine the 2 NW partial (max, sum) pairs of every row, then lse, lpb, lpy
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            red_m[(wave * 2 + hb) * 64 + rt * 32 + l32] = m_run[rt];
            red_s[(wave * 2 + hb) * 64 + rt * 32 + l32] = s_run[rt];
        }
        __syncthreads();
        if (tid < 64) {
            const int r = tid;
            const int idx = row_lat[r];
            float esum = 0.0f;
            if (idx >= 0) {
                float M = RNNT_NEG_INF;
#pragma unroll
                for (int p = 0; p < 2 * NW; ++p) M = fmaxf(M, red_m[p * 64 + r]);
                float S = 0.0f;
#pragma unroll
                for (int p = 0; p < 2 * NW; ++p) S += red_s[p * 64 + r] * __expf(red_m[p * 64 + r] - M);
                const float lse = M + __logf(S);
                a.ls.lse[idx] = lse;
                a.ls.lpb[idx] = row_f0[r] - lse;
                a.ls.lpy[idx] = (row_lab[r] >= 0) ? row_f1[r] - lse : 0.0f;
                // this node's share of the sum the lattice kernels take their per-sample offset from
                const bool has_label = tp.u0 + (r & (tp.uw - 1)) < tp.U;
                esum = has_label ? fmaxf(row_f0[r], row_f1[r]) - lse : row_f0[r] - lse;
            }
            esum = wave_sum(esum);
            if (r == 0) a.ls.tile_esum[tile] = esum;
        }
    }
}

static size_t joint_smem_bytes(int H, int mode, int nw) {
    size_t z = (size_t)JT_ROWS * (H + 8) * 2;
    size_t meta = 64 * 4 * 5;
    const size_t red = (size_t)2 * (2 * nw * 64) * 4, stg = (size_t)nw * 32 * STG_PITCH * 2;
    const size_t stg2 = (size_t)nw * 32 * STG2_PITCH * 2;
    return z + meta + (mode == 0 ? red : mode == 1 ? stg : red + stg2);
}

// Forward and unfused backward: 4 waves x two 32-entry tiles each.
template <int MODE, int NW, int NVT, int PF>
static hipError_t launch_joint(const JointArgs& a, hipStream_t stream) {
    const int n = a.tile1 - a.tile0;
    if (n <= 0) return hipSuccess;
    const size_t smem = joint_smem_bytes(a.pr.H, MODE, NW);
    static size_t configured = 0;
    if (smem > configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_joint_scores<MODE, NW, NVT, PF>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        configured = smem;
    }
    k_joint_scores<MODE, NW, NVT, PF><<<dim3((unsigned)n), dim3(64 * NW), smem, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_fwd_bf16(const Problem& pr, const void* Wpack, const SampleTable& st, const LatticeState& ls,
                           int s0, int s1, int tile0, int tile1, hipStream_t stream) {
    JointArgs a{pr, st, ls, (const bf16_t*)Wpack, s0, s1, tile0, tile1, nullptr, nullptr, nullptr,
                EVERY_TILE};
    // a longer prefetch distance where the hidden size allows it (the forward kernel has the registers)
    if (pr.H % 256 == 0) return launch_joint<0, 4, 2, 8>(a, stream);
    return launch_joint<0, 4, 2, 4>(a, stream);
}

hipError_t launch_bwd_scores_bf16(const Problem& pr, const void* Wpack, const SampleTable& st,
                                  const LatticeState& ls, int s0, int s1, int tile0, int tile1, void* dH,
                                  void* Z, const ActiveTiles& at, hipStream_t stream) {
    JointArgs a{pr, st, ls, (const bf16_t*)Wpack, s0, s1, tile0, tile1, (bf16_t*)dH, (bf16_t*)Z, nullptr, at};
    return launch_joint<1, 4, 2, 4>(a, stream);
}

hipError_t launch_fwd_keep_bf16(const Problem& pr, const void* Wpack, const SampleTable& st,
                                const LatticeState& ls, int s0, int s1, int tile0, int tile1, void* kept,
                                void* Z, float* kept_max, hipStream_t stream) {
    JointArgs a{pr, st, ls, (const bf16_t*)Wpack, s0, s1, tile0, tile1, (bf16_t*)kept, (bf16_t*)Z, kept_max,
                EVERY_TILE};
    if (pr.H % 256 == 0) return launch_joint<2, 4, 2, 8>(a, stream);
    return launch_joint<2, 4, 2, 4>(a, stream);
}

// ------------------------------------------------------------------------------------------------
// Kept scores -> score gradients, in place (f^W_4 without the second score GEMM):
//   dh[r,v] = exp(t[r,v] + m[r, v/64] - lse[r] + ln gamma[r]) - [v = blank] B[r] - [v = y_u] Y[r],
// rounded to bf16 over the fp16 t.  One workgroup per lattice tile (64 rows); wave w takes rows w, w+4, ...
// and its lanes consecutive 16-byte pieces of the row.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_kept_to_dh(JointArgs a) {
    __shared__ int row_lab[64];
    __shared__ float row_g[64], row_b[64], row_y[64];
    typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
    const int V = a.pr.V;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    int tile = a.tile0 + blockIdx.x;
    if (a.at.active) {
        // listed tiles only (uniform per workgroup); the kept scores of a tile lie at its position in the launch
        const int ci = a.at.cbase + (int)blockIdx.x;
        if (ci >= *a.at.n_active) return;
        tile = a.at.active[a.at.group_tile0 + ci];
    }
    const int slot = tile - a.tile0;
    const TilePos tp = locate_tile(a.st, a.s0, a.s1, tile);
    const int b = tp.s;
    if (tid < 64) {
        const int r = tid;
        const int t = tp.t0 + (r >> tp.us), u = tp.u0 + (r & (tp.uw - 1));
        const bool valid = (t < tp.T && u <= tp.U);
        row_lab[r] = (valid && u < tp.U) ? a.pr.labels[(size_t)b * a.pr.U_max + u] : -1;
        float g = RNNT_NEG_INF, bk = 0.0f, yk = 0.0f;
        if (valid) {
            const long long idx = (a.st.row_off[b] - a.ls.row_base) + (long long)t * (tp.U + 1) + u;
            const RowPost rp = row_posteriors(a.ls, idx, t, u, tp.T, tp.U, b);
            g = (rp.log_gamma - a.ls.lse[idx]) * LOG2E_F;
            bk = rp.Bk;
            yk = rp.Yk;
        }
        row_g[r] = g;
        row_b[r] = bk;
        row_y[r] = yk;
    }
    __syncthreads();
    const int cpr = V >> 3;                      // 16-byte pieces per row
    const float* mx = a.kept_max + (size_t)slot * (V / 64) * 64;
    for (int row = wave; row < 64; row += 4) {
        bf16_t* rowp = a.dH + (size_t)((long long)slot * JT_ROWS + row) * chunk_pitch(V);
        const float g = row_g[row], bk = row_b[row], yk = row_y[row];
        const int lab = row_lab[row];
        for (int c0 = lane; c0 < cpr; c0 += 256) {
            f16x8 t[4];
            float e[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = c0 + 64 * i < cpr ? c0 + 64 * i : c0;
                t[i] = __builtin_nontemporal_load(reinterpret_cast<const f16x8*>(rowp + c * 8));
                e[i] = fmaf(mx[(c >> 3) * 64 + row], LOG2E_F, g);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = c0 + 64 * i;
                if (c < cpr) {
                    float d[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) d[k] = __builtin_amdgcn_exp2f(fmaf((float)t[i][k], LOG2E_F, e[i]));
                    const int relb = a.pr.blank - c * 8, rely = lab - c * 8;
                    if ((unsigned)relb < 8u || (unsigned)rely < 8u) {
#pragma unroll
                        for (int k = 0; k < 8; ++k) {
                            if (k == relb) d[k] -= bk;
                            if (k == rely) d[k] -= yk;
                        }
                    }
                    bf16x8 o;
#pragma unroll
                    for (int k = 0; k < 8; ++k) o[k] = (bf16_t)d[k];
                    __builtin_nontemporal_store(o, reinterpret_cast<bf16x8*>(rowp + c * 8));
                }
            }
        }
    }
}

hipError_t launch_kept_to_dh_bf16(const Problem& pr, const SampleTable& st, const LatticeState& ls, int s0,
                                  int s1, int tile0, int tile1, void* kept, const float* kept_max,
                                  const ActiveTiles& at, hipStream_t stream) {
    const int n = tile1 - tile0;
    if (n <= 0) return hipSuccess;
    JointArgs a{pr, st, ls, nullptr, s0, s1, tile0, tile1, (bf16_t*)kept, nullptr, const_cast<float*>(kept_max),
                at};
    k_kept_to_dh<<<dim3((unsigned)n), dim3(256), 0, stream>>>(a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// dW += Z^T dH and db += column sums of dH (Alg. 1 line 8) as one split-K GEMM with 256x256 tiles.
// 256 threads = 4 waves in 2 (hidden) x 2 (vocabulary), one per SIMD; each wave owns 128 x 128 = 4 x 4
// accumulator tiles (256 accumulator registers), so that a k16-step reads 8 fragments from LDS for 16
// MFMAs and every byte of a stage feeds 128 flops.  Both operands are row-major with the contraction index (the
// chunk's rows) as the slow one:
// Z [rows,H], dH [rows,V].  Stages of 32 rows travel global -> LDS asynchronously (global_load_lds, no
// registers), four stages deep, and lie in LDS as in memory ([row][column], 16-byte chunks
// XOR-swizzled by 4*(row%4), which spreads the four rows a transposing read touches per 32 lanes over all 64 banks); MFMA fragments, which need 8 consecutive rows of one column per lane,
// come from the transposing LDS read (ds_read_b64_tr_b16): within 16 lanes, lane 4j+c supplies 4
// columns of row j and lane i receives rows 0..3 of column i.
// The workgroups of the first hidden-tile row also sum their B fragments over the rows (the bias
// gradient) with packed bf16 dot products against ones.
// ------------------------------------------------------------------------------------------------
constexpr int WT = 256;       // tile edge
constexpr int WK = 32;        // rows per pipeline stage
constexpr int WST = 4;        // pipeline stages (LDS buffers)

struct DwArgs {
    const bf16_t* Z;
    const bf16_t* dH;
    long long K, k_per_split;
    float* slots;    // [splits][tiles][4 waves][4][4][4][64 lanes] float4: partial sums, accumulator layout
    float* db;
    int first;       // overwrite the slot instead of adding to it
    int H, V;
    int mt, nt;      // output tiles along H and V
    int splits;
    ActiveTiles at;  // at.active set: the chunk holds 64 * (*at.n_active - at.cbase) rows if that is less than K
};
// BY_TILE (at.slot_tile0 >= 0): the 64 rows of the list's entry i lie in slot (tile - at.slot_tile0) of both chunk
// buffers instead of slot i.  A stage of 32 rows lies inside one slot, so only the first row of a stage changes;
// the list entry of a stage is read (a scalar load) one loop iteration before the stage's copies are issued.

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ bf16x8 lds_read_tr_frag(const bf16_t* p) {
    // rows +0..3 and +4..7 of this lane's column: two transposing reads, 4 rows (= 4*256 elements) apart
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + 4 * WT));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

template <bool BY_TILE>
__global__ __launch_bounds__(256) void k_gemm_dw256(DwArgs g) {
    extern __shared__ __align__(16) unsigned char dw_smem[];   // [WST] x { A [WK][256], B [WK][256] } bf16
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hb = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  All output tiles of
    // one K split read the same rows of Z and dH, so they are mapped to the same XCD (ids that
    // agree modulo 8) and adjacent in its dispatch order: the rows then come from HBM once.
    const int ntile = g.mt * g.nt;
    const int L = blockIdx.x, xcd = L & 7, q = L >> 3;
    const int tile = q % ntile, split = xcd + 8 * (q / ntile);
    const int bm = tile % g.mt, bn = tile / g.mt;
    const long long m0 = (long long)bm * WT, n0 = (long long)bn * WT;
    long long K = g.K, k_per_split = g.k_per_split;
    if (g.at.active) {
        long long act = (long long)*g.at.n_active - g.at.cbase;
        act = act < 0 ? 0 : act * JT_ROWS;
        if (act < K) {
            K = act;
            const long long per = (K + g.splits - 1) / g.splits;
            k_per_split = (per + WK - 1) / WK * WK;
        }
    }
    const long long ks = (long long)split * k_per_split;
    const long long ke = ks + k_per_split < K ? ks + k_per_split : K;
    const bool do_db = (bm == 0) && (wm == 0);
    constexpr unsigned STAGE_BYTES = 2u * WK * WT * 2u;
    constexpr unsigned OPER_BYTES = (unsigned)WK * WT * 2u;
    const unsigned smem_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)dw_smem;

    // global -> LDS: one DMA instruction moves two tile rows (2 x 512 B).  Wave w moves row pairs w,
    // w+4, w+8 and w+12 of both operands.  LDS slot (row, position p) receives global chunk p ^ 4*(row%4) of
    // that row.  A lane's byte offset within a row pair is the same for all four pairs (8 rows apart, so the
    // swizzle agrees); everything that changes from pair to pair and stage to stage is wave-uniform and
    // lives in scalar registers, so issuing a DMA costs no vector instruction.
    const int wv = __builtin_amdgcn_readfirstlane(wave);
    const long long ZL = chunk_pitch(g.H), DL = chunk_pitch(g.V);   // row pitches of the chunk buffers
    unsigned offA, offB;
    {
        const int ch = (lane & 31) ^ (((2 * wave + (lane >> 5)) & 3) << 2);
        long long acol = m0 + ch * 8;
        if (acol > g.H - 8) acol = g.H - 8;      // columns beyond H (H not a multiple of 256): never stored
        offA = (unsigned)(((long long)(lane >> 5) * ZL + acol) * 2);
        offB = (unsigned)(((long long)(lane >> 5) * DL + n0 + ch * 8) * 2);
    }
    const char* Zs = reinterpret_cast<const char*>(g.Z) + (ks + 2 * wv) * ZL * 2;
    const char* Ds = reinterpret_cast<const char*>(g.dH) + (ks + 2 * wv) * DL * 2;
    const unsigned dst0 = smem_base + (unsigned)(2 * wv) * (WT * 2u);
    // First buffer row of stage gstep (rows [gstep*WK, +WK) of the split), relative to row ks; `entry` is the list
    // entry of the stage's slot (BY_TILE only).
    // (read through the constant address space: the list was written before this launch, and only such a load
    // becomes a scalar load that stays clear of the vector-memory counter the copies below are tracked with)
    typedef const int __attribute__((address_space(4))) * list_ptr;
    const list_ptr lst = BY_TILE ? (list_ptr)(g.at.active + g.at.group_tile0 + g.at.cbase) : nullptr;
    auto stage_entry = [&](long long gstep) { return BY_TILE ? lst[(ks + gstep * WK) >> 6] : 0; };
    auto stage_row = [&](long long gstep, int entry) -> long long {
        if (!BY_TILE) return gstep * WK;
        return ((long long)(entry - g.at.slot_tile0) << 6) + ((ks + gstep * WK) & 63) - ks;
    };
    // DMA j (0..7) of the stage whose first row is row0 into LDS buffer buf
    auto issue_one = [&](long long row0, unsigned buf, int j) {
        const int i = j >> 1;
        const unsigned sb = dst0 + buf * STAGE_BYTES + (unsigned)(8 * i) * (WT * 2u);
        const long long krow = row0 + 8 * i;
        if (j & 1) lds_dma16_s(Ds + krow * DL * 2, offB, sb + OPER_BYTES);
        else lds_dma16_s(Zs + krow * ZL * 2, offA, sb);
    };
    // fragment addresses: lane = 16 g + 4 j + c supplies row 8*(g/2) + j, columns 16*(g%2) + 4c .. +3
    const int fg = lane >> 4, fj = (lane >> 2) & 3, fc = lane & 3;
    const int frow = 8 * (fg >> 1) + fj;
    int aoff[4], boff[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        const int col = wm * 128 + mt * 32 + 16 * (fg & 1) + 4 * fc;
        aoff[mt] = frow * WT + (((col >> 3) ^ (fj << 2)) << 3) + (col & 7);
    }
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        const int col = wn * 128 + nt * 32 + 16 * (fg & 1) + 4 * fc;
        boff[nt] = WK * WT + frow * WT + (((col >> 3) ^ (fj << 2)) << 3) + (col & 7);
    }

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x16{0};
    float dbs[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};

    const long long nsteps = ke > ks ? (ke - ks) / WK : 0;   // a split beyond the chunk still writes its slot
    if (nsteps == 0 && !g.first) return;                     // ... unless the slot already holds a sum: nothing to add
    static_assert(WK == 32, "the loop below is written for two k16-steps per stage");
    bf16x8 fa[2][4], fb[2][4];
    auto read_frags = [&](int set, long long stage, int kk) {
        const bf16_t* st = reinterpret_cast<const bf16_t*>(dw_smem + (size_t)(stage & (WST - 1)) * STAGE_BYTES) +
                           kk * 16 * WT;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) fa[set][mt] = lds_read_tr_frag(st + aoff[mt]);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) fb[set][nt] = lds_read_tr_frag(st + boff[nt]);
    };
    // The 16 MFMAs of one k16-step (register set `set`); behind each of the first eight, one fragment of the
    // following k16-step is read into the other set.  An MFMA keeps the matrix pipe busy for 32 clocks but
    // the issue port only briefly: the reads go out in its shadow, and the last of them is 8 MFMAs old when
    // the step ends.
    // Behind each of the last eight goes one DMA of a later stage (dma_g >= 0).
    auto multiply = [&](int set, long long next_stage, int next_kk, long long dma_row0, unsigned dma_buf) {
        const bf16_t* st = reinterpret_cast<const bf16_t*>(dw_smem + (size_t)(next_stage & (WST - 1)) * STAGE_BYTES) +
                           next_kk * 16 * WT;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][mt], fb[set][nt], acc[mt][nt], 0, 0, 0);
                const int idx = mt * 4 + nt;
                if (idx < 4) fa[set ^ 1][idx] = lds_read_tr_frag(st + aoff[idx]);
                else if (idx < 8) fb[set ^ 1][idx - 4] = lds_read_tr_frag(st + boff[idx - 4]);
                else if (set == 1) issue_one(dma_row0, dma_buf, idx - 8);
                __builtin_amdgcn_sched_barrier(0);
            }
        if (do_db) {
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int q2 = 0; q2 < 4; ++q2) {
                    const bf16x2 pr2 = {fb[set][nt][2 * q2], fb[set][nt][2 * q2 + 1]};
                    dbs[nt] = __builtin_amdgcn_fdot2_f32_bf16(pr2, ones, dbs[nt], false);
                }
        }
    };
    // Three stages in flight before the first one is consumed (8 DMA instructions per wave and stage).
    // One wave per SIMD: nothing else hides an LDS read or the issue of a DMA, so both are spread over the
    // MFMAs (see multiply).  The hand-over to the next stage (wait for this wave's copies, then for
    // everyone's) sits in the middle of a stage.  Beyond the last stage the pipeline keeps re-loading the
    // last one into buffers nobody reads any more, which keeps the loop free of branches and the number of
    // copies in flight constant.
    if (nsteps > 0) {
        const long long last = nsteps - 1;
#pragma unroll
        for (int st3 = 0; st3 < 3; ++st3) {
            const long long gs = st3 < last ? st3 : last;
            const long long row0 = stage_row(gs, stage_entry(gs));
#pragma unroll
            for (int j = 0; j < 8; ++j) issue_one(row0, (unsigned)st3, j);
        }
        int entry_ahead = stage_entry(3 < last ? 3 : last);
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        __syncthreads();
        read_frags(0, 0, 0);
        for (long long it = 0; it < nsteps; ++it) {
            __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);     // set 0 landed (read behind the first MFMAs of the step before)
            __builtin_amdgcn_sched_barrier(0);
            const long long dma_row0 = stage_row(it + 3 < last ? it + 3 : last, entry_ahead);
            entry_ahead = stage_entry(it + 4 < last ? it + 4 : last);      // arrives during this iteration
            multiply(0, it, 1, 0, 0);
            __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);     // set 1 landed
            // stage it+1 landed (stage it+2 stays in flight); every wave is past stage it-1, whose buffer
            // takes stage it+3
            asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
            multiply(1, it + 1, 0, dma_row0, (unsigned)((it + 3) & (WST - 1)));
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // no copy may land after the workgroup has ended
    }
    // Partial sums go to this workgroup's own slot, in accumulator order (one 16-byte store per lane
    // and four accumulator rows): no atomics, and the same workgroup adds the next chunk's product.
    {
        f32x4* slot = reinterpret_cast<f32x4*>(g.slots) +
                      (((size_t)split * ntile + tile) * 4 + wave) * (size_t)(4 * 4 * 4 * 64) + lane;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    f32x4 v = {acc[mt][nt][4 * j], acc[mt][nt][4 * j + 1], acc[mt][nt][4 * j + 2],
                               acc[mt][nt][4 * j + 3]};
                    f32x4* q = slot + ((mt * 4 + nt) * 4 + j) * 64;
                    if (!g.first) v += *q;
                    *q = v;
                }
    }
    if (do_db) {
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            float v = dbs[nt] + __shfl_xor(dbs[nt], 32, 64);
            if (hb == 0) atomicAdd(&g.db[n0 + wn * 128 + nt * 32 + l32], v);
        }
    }
}

hipError_t launch_gemm_dw_bf16(int H, int V, long long rows, int splits, int first, const void* Z, const void* dH,
                               float* slots, float* db, const ActiveTiles& at, hipStream_t stream) {
    if (rows <= 0 || splits <= 0 || (splits & 7) != 0 || rows % WK != 0) return hipErrorInvalidValue;
    const long long mt = (H + WT - 1) / WT, nt = V / WT;
    DwArgs g{(const bf16_t*)Z, (const bf16_t*)dH, rows, 0, slots, db, first, H, V, (int)mt, (int)nt, splits, at};
    // split s runs on XCD s % 8; a split past the end of a short chunk only touches its slot
    long long per = (rows + splits - 1) / splits;
    g.k_per_split = (per + WK - 1) / WK * WK;
    const size_t smem = (size_t)WST * 2 * WK * WT * 2;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_dw256<false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_dw256<true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const dim3 grid((unsigned)(mt * nt * splits));
    if (at.active && at.slot_tile0 >= 0) k_gemm_dw256<true><<<grid, dim3(256), smem, stream>>>(g);
    else k_gemm_dw256<false><<<grid, dim3(256), smem, stream>>>(g);
    return hipGetLastError();
}

// dW (+)= sum over the splits of the slots.  One thread per float4 of a tile's slot (four consecutive
// hidden rows of one vocabulary column), decoded back from the accumulator order of k_gemm_dw256.
__global__ __launch_bounds__(256) void k_dw_reduce(const f32x4* __restrict__ slots, float* __restrict__ dW, int H, int V,
                                                   int mt_tiles, int ntile, int splits, int accumulate) {
    const int tile = blockIdx.y;
    const int e = blockIdx.x * 256 + threadIdx.x;          // 0 .. 16383
    f32x4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int s = 0; s < splits; ++s) sum += slots[((size_t)s * ntile + tile) * 16384 + e];
    const int wave = e >> 12, mt = (e >> 10) & 3, nt = (e >> 8) & 3, j = (e >> 6) & 3, lane = e & 63;
    const int bm = tile % mt_tiles, bn = tile / mt_tiles;
    const int m = bm * WT + (wave >> 1) * 128 + mt * 32 + 8 * j + 4 * (lane >> 5);
    const int n = bn * WT + (wave & 1) * 128 + nt * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (m + i < H) {
            float* q = dW + (size_t)(m + i) * V + n;
            *q = accumulate ? *q + sum[i] : sum[i];
        }
    }
}

hipError_t launch_dw_reduce(int H, int V, int splits, const float* slots, float* dW, int accumulate,
                            hipStream_t stream) {
    const int mt = (H + WT - 1) / WT, nt = V / WT;
    k_dw_reduce<<<dim3(64, (unsigned)(mt * nt)), dim3(256), 0, stream>>>((const f32x4*)slots, dW, H, V, mt, mt * nt, splits,
                                                                      accumulate);
    return hipGetLastError();
}

}  // namespace rnnt
