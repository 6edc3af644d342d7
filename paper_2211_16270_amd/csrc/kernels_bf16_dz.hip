// Unfused backward, second half (Alg. 1 lines 10, 11) for hidden sizes the fused kernel does not cover:
//   dz = dH W_out^T   (dH [rows,V] from the chunk buffer, W_out [H,V]: both with the contraction index,
//                      the vocabulary, contiguous),
//   dx = dz (1 - z^2),  d_enc[t] += sum_u dx,  d_pred[u] += sum_t dx  per lattice tile (64 rows: 8 frames x 8 labels or 16 x 4).
//
// 256x256 output tile (4 lattice tiles x 256 hidden) per workgroup; 256 threads = 4 waves in 2 x 2, one per
// SIMD, each 128 x 128 = 4 x 4 accumulator tiles (256 accumulator registers), so that one k16-step is 8
// LDS fragment reads for 16 MFMAs.  Stages of 64 vocabulary entries (whole 128-byte lines of the operand
// rows) travel global -> LDS asynchronously (global_load_lds) into two stage buffers.  A stage holds the
// operand rows as 128-byte LDS rows; the 16-byte segment s of row r lies at position s ^ ((r/2)%8), which
// makes the 16-byte fragment reads of 16 consecutive rows hit all 64 banks.  Fragments are read one
// k16-step ahead of their MFMAs, also across the stage hand-over.  The epilogue recomputes
// z = tanh(enc + pred) in fp32 from input rows staged in LDS.
#include <type_traits>

#include "device_common.h"

namespace rnnt {

namespace {

constexpr int ZT = 256;       // tile edge
constexpr int ZK = 64;        // vocabulary entries per stage: one 128-byte line of every operand row
constexpr int ZST = 2;        // stages
constexpr unsigned Z_OPER = (unsigned)ZT * ZK * 2u;     // bytes of one operand of a stage
constexpr unsigned Z_STAGE = 2u * Z_OPER;
constexpr int Z_EP = 264;     // pitch (bf16 elements) of the epilogue's enc / pred rows in LDS

struct DzArgs {
    const bf16_t* dH;
    const bf16_t* W;
    Problem pr;
    SampleTable st;
    int s0, s1, tile0, tile1;
    float* d_enc;
    float* d_pred;
    int m_tiles, n_tiles;
    long long rows;           // rows of the dH chunk buffer that were written (a multiple of 64)
    ActiveTiles at;           // which tiles the chunk's 64-row slots hold (see kernels.h)
};

__global__ __launch_bounds__(256) void k_gemm_dz256(DzArgs g) {
    extern __shared__ __align__(16) unsigned char dz_smem[];   // [ZST] x { A [256][64], B [256][64] } bf16
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hb = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    // XCD-aware order (ids that agree modulo 8 share an L2): the hidden tiles of one row tile are
    // neighbours on one XCD, so the rows of dH are fetched from HBM once.
    const int L = blockIdx.x, xcd = L & 7, q = L >> 3;
    const int by = q % g.n_tiles, bx = xcd + 8 * (q / g.n_tiles);
    // slots of the chunk that hold a tile: all of the launch's, or what is left of the group's list
    int n_slots = g.tile1 - g.tile0;
    if (g.at.active) {
        const int left = *g.at.n_active - g.at.cbase;
        n_slots = left < n_slots ? left : n_slots;
    }
    if (bx * 4 >= n_slots) return;          // also covers bx >= m_tiles (uniform per workgroup)
    const int H = g.pr.H, V = g.pr.V;
    const long long m0 = (long long)bx * ZT;
    const int n0 = by * ZT;
    const unsigned smem_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)dz_smem;

    // global -> LDS: one DMA instruction moves 8 operand rows of 128 bytes (whole cache lines: with
    // 64-byte pieces every line would be fetched into L1 twice, by two stages).  Wave w moves row groups
    // w, w+4, ..., w+28 of both operands.  Lane l serves row l/8 of the group and LDS segment l%8, which
    // holds global segment (l%8) ^ ((row/2)%8); row groups are 32 rows apart, so a lane's byte offset
    // within its group is the same for all of them, and
    // everything else is wave-uniform: issuing a DMA costs no vector instruction.  Rows of dH past the
    // written ones lie inside the chunk buffer (its size is a multiple of the tile edge) and hidden rows
    // past H (H is a multiple of 128: the upper half of the last tile) re-read the lower half; their
    // products are never stored.
    const int wv = __builtin_amdgcn_readfirstlane(wave);
    const long long DL = chunk_pitch(V);      // row pitch of the dH chunk buffer
    const int lseg = ((lane & 7) ^ ((4 * wave + (lane >> 4)) & 7)) * 8;
    const unsigned lane_offA = (unsigned)(((long long)(lane >> 3) * DL + lseg) * 2);
    const unsigned lane_offB = (unsigned)(((long long)(lane >> 3) * V + lseg) * 2);
    // the workgroup's four 64-row slots of the dH buffer: consecutive, or (kept scores) wherever the forward pass
    // has put the listed tiles; entries past the list's end read the last listed tile again
    const char* As[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        long long row = m0 + 64 * k;
        if (g.at.active && g.at.slot_tile0 >= 0) {
            const int e = bx * 4 + k < n_slots ? bx * 4 + k : n_slots - 1;
            row = (long long)(g.at.active[g.at.group_tile0 + g.at.cbase + e] - g.at.slot_tile0) * 64;
        }
        As[k] = reinterpret_cast<const char*>(g.dH) + (row + 8 * wv) * DL * 2;
    }
    const char* Bs = reinterpret_cast<const char*>(g.W) + (long long)(n0 + 8 * wv) * V * 2;
    const bool half_tile = (n0 + 128 >= H);
    const unsigned dst0 = smem_base + (unsigned)(8 * wv) * 128u;
    // DMA j (0..15) of the stage that takes vocabulary entries [gstep*ZK, +ZK) into LDS buffer buf
    auto issue_one = [&](int gstep, unsigned buf, int j) {
        const int i = j >> 1;
        const unsigned sb = dst0 + buf * Z_STAGE + (unsigned)(32 * i) * 128u;
        if (j & 1) {
            const int ib = (half_tile && i >= 4) ? i - 4 : i;
            lds_dma16_s(Bs + ((long long)(32 * ib) * V + (long long)gstep * ZK) * 2, lane_offB, sb + Z_OPER);
        } else {
            lds_dma16_s(As[i >> 1] + ((long long)(32 * (i & 1)) * DL + (long long)gstep * ZK) * 2, lane_offA, sb);
        }
    };
    // fragment of 32 rows, k16-step kk of a stage: lane holds row l32, segment 2*kk + hb at position
    // (2*kk + hb) ^ ((row/2)%8): sixteen consecutive rows then cover all 64 banks
    const int xr = (l32 >> 1) & 7;
    unsigned frag_off[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) frag_off[kk] = (unsigned)l32 * 128u + (unsigned)(((2 * kk + hb) ^ xr) << 4);

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x16{0};

    const int nsteps = V / ZK;
    bf16x8 fa[2][4], fb[2][4];
    auto read_frags = [&](int set, int stage, int kk) {
        const unsigned char* st = dz_smem + (size_t)(stage & (ZST - 1)) * Z_STAGE + frag_off[kk];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
            fa[set][mt] = *reinterpret_cast<const bf16x8*>(st + (wm * 128 + mt * 32) * 128);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
            fb[set][nt] = *reinterpret_cast<const bf16x8*>(st + Z_OPER + (wn * 128 + nt * 32) * 128);
    };
    // The 16 MFMAs of one k16-step (register set `set`).  Behind each of the first eight, one fragment of the
    // following k16-step is read into the other set; behind each of the last eight go two DMAs of a later
    // stage (DMA = true).  An MFMA keeps the matrix pipe busy for 32 clocks but the issue port only briefly:
    // with one wave per SIMD nothing else would hide these instructions.
    auto multiply = [&](int set, int next_stage, int next_kk, bool DMA, int dma_g, unsigned dma_buf) {
        const unsigned char* st = dz_smem + (size_t)(next_stage & (ZST - 1)) * Z_STAGE + frag_off[next_kk];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][mt], fb[set][nt], acc[mt][nt], 0, 0, 0);
                const int idx = mt * 4 + nt;
                if (idx < 4) {
                    fa[set ^ 1][idx] = *reinterpret_cast<const bf16x8*>(st + (wm * 128 + idx * 32) * 128);
                } else if (idx < 8) {
                    fb[set ^ 1][idx - 4] = *reinterpret_cast<const bf16x8*>(st + Z_OPER + (wn * 128 + (idx - 4) * 32) * 128);
                } else if (DMA) {
                    issue_one(dma_g, dma_buf, 2 * (idx - 8));
                    issue_one(dma_g, dma_buf, 2 * (idx - 8) + 1);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
    };
    // Two stage buffers.  Fragments are read one k16-step ahead of their MFMAs.  Before the last k16-step of
    // a stage every wave has issued and completed all its reads of that stage: there the next stage is
    // waited for (own copies, then everyone's) and the stage after it is sent into the buffer just left.
    // Beyond the last stage the pipeline re-loads the last one into a buffer nobody reads any more, which
    // keeps the loop free of branches.  The waits for LDS reads are placed by hand (as the builtin the
    // compiler's own counter tracking understands) before the reads of the following step are issued: the
    // counter completes in order, so a wait placed after them would wait for them too.
    const int last = nsteps - 1;
#pragma unroll
    for (int j = 0; j < 16; ++j) issue_one(0, 0u, j);
#pragma unroll
    for (int j = 0; j < 16; ++j) issue_one(last < 1 ? last : 1, 1u, j);
    asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    __syncthreads();
    read_frags(0, 0, 0);
    for (int it = 0; it < nsteps; ++it) {
        __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);
        __builtin_amdgcn_sched_barrier(0);
        multiply(0, it, 1, false, 0, 0u);
        __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);
        __builtin_amdgcn_sched_barrier(0);
        multiply(1, it, 2, false, 0, 0u);
        __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);
        __builtin_amdgcn_sched_barrier(0);
        multiply(0, it, 3, false, 0, 0u);
        // all reads of stage `it` are complete, stage it+1 has landed: its buffer takes stage it+2
        __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        multiply(1, it + 1, 0, true, it + 2 < last ? it + 2 : last, (unsigned)(it & (ZST - 1)));
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // no copy may land after the workgroup has ended

    // ---- epilogue: dx = dz (1 - z^2) with z = tanh(enc + pred) recomputed in fp32, summed over the label
    // positions / frames of each lattice tile.  The input rows of the workgroup's four lattice tiles (8 + 8 or
    // 16 + 4 of them; this tile's 256 hidden columns) go through LDS, which the main loop no longer needs:
    // per tile 20 row slots, the tile's frames first, its label positions behind them.
    __shared__ TilePos tpos[4];      // where the workgroup's four lattice tiles lie (s < 0: past the last tile)
    if (tid < 4) {
        const int slot = bx * 4 + tid;
        TilePos t{};
        t.s = -1;
        if (slot < n_slots)
            t = locate_tile(g.st, g.s0, g.s1,
                            g.at.active ? g.at.active[g.at.group_tile0 + g.at.cbase + slot] : g.tile0 + slot);
        tpos[tid] = t;
    }
    __syncthreads();
    bf16_t* eq = reinterpret_cast<bf16_t*>(dz_smem);              // [4 tiles][20 rows][Z_EP]
    {
        // 4 tiles x 20 rows x 32 chunks of 8 columns = 2560 chunks, 10 per thread
#pragma unroll
        for (int i = 0; i < 10; ++i) {
            const int e = tid + 256 * i;
            const int c = e & 31, r = (e >> 5) % 20, t4 = e / (32 * 20);
            const TilePos tp = tpos[t4];
            bf16x8 v;
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = (bf16_t)0.0f;
            if (tp.s >= 0 && n0 + c * 8 < H) {
                const int th = 64 >> tp.us;
                if (r < th) {
                    if (tp.t0 + r < tp.T)
                        v = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const bf16_t*>(g.pr.enc) +
                                                             ((size_t)tp.s * g.pr.T_max + tp.t0 + r) * H + n0 + c * 8);
                } else if (r - th < tp.uw && tp.u0 + r - th <= tp.U) {
                    v = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const bf16_t*>(g.pr.pred) +
                                                         ((size_t)tp.s * (g.pr.U_max + 1) + tp.u0 + r - th) * H + n0 + c * 8);
                }
            }
            *reinterpret_cast<bf16x8*>(eq + (t4 * 20 + r) * Z_EP + c * 8) = v;
        }
    }
    __syncthreads();
    // Rows wm*128 + 64*lt .. +63 are one lattice tile; accumulator register 4j+i of row block mt = 2*lt + m2 is
    // tile row r = 32 m2 + 8j + 4 hb + i, hidden column l32: in an 8 x 8 tile frame 4 m2 + j, label 4 hb + i; in a
    // 16 x 4 tile frame 8 m2 + 2j + hb, label i.  One copy of the loop nest per shape.
    // (the two lattice tiles of a wave as two instantiations: every accumulator index is a constant)
    auto tile_epilogue = [&](auto lt_tag) {
        constexpr int lt = decltype(lt_tag)::value;
        const int t4 = wm * 2 + lt;
        const TilePos tp = tpos[t4];
        if (tp.s < 0) return;
        const int b = tp.s;
        float* d_enc = g.d_enc + (size_t)b * g.pr.T_max * H;
        float* d_prd = g.d_pred + (size_t)b * (g.pr.U_max + 1) * H;
        const bf16_t* er = eq + (t4 * 20) * Z_EP;
        auto reduce = [&](auto wide_tag) {
            constexpr bool WIDE = decltype(wide_tag)::value;
            constexpr int TH = WIDE ? 8 : 16;
            const int ulb = WIDE ? 4 * hb : 0;              // first of this lane's four label positions
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                const int hc = wn * 128 + nt * 32 + l32;        // column inside the tile
                const int h = n0 + hc;
                if (h >= H) continue;
                float qv[4], pu[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int i = 0; i < 4; ++i) qv[i] = (float)er[(TH + ulb + i) * Z_EP + hc];
#pragma unroll
                for (int m2 = 0; m2 < 2; ++m2)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int tl = WIDE ? 4 * m2 + j : 8 * m2 + 2 * j + hb;
                        const bool tv = (tp.t0 + tl < tp.T);
                        const float ev = (float)er[tl * Z_EP + hc];
                        float se = 0.0f;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const bool ok = tv && (tp.u0 + ulb + i <= tp.U);
                            const float z = fast_tanh(ev + qv[i]);
                            const float dx = ok ? acc[2 * lt + m2][nt][4 * j + i] * (1.0f - z * z) : 0.0f;
                            se += dx;
                            pu[i] += dx;
                        }
                        if (WIDE) {
                            se += __shfl_xor(se, 32, 64);       // a frame's eight labels lie in both lane halves
                            if (tv && hb == (j & 1)) atomicAdd(&d_enc[(size_t)(tp.t0 + tl) * H + h], se);
                        } else if (tv) {
                            atomicAdd(&d_enc[(size_t)(tp.t0 + tl) * H + h], se);
                        }
                    }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (WIDE) {
                        if (tp.u0 + 4 * hb + i <= tp.U) atomicAdd(&d_prd[(size_t)(tp.u0 + 4 * hb + i) * H + h], pu[i]);
                    } else {
                        const float both = pu[i] + __shfl_xor(pu[i], 32, 64);   // a label's sixteen frames do
                        if (hb == (i & 1) && tp.u0 + i <= tp.U) atomicAdd(&d_prd[(size_t)(tp.u0 + i) * H + h], both);
                    }
                }
            }
        };
        if (tp.uw == 8) reduce(std::true_type{});
        else reduce(std::false_type{});
    };
    tile_epilogue(std::integral_constant<int, 0>{});
    tile_epilogue(std::integral_constant<int, 1>{});
}

}  // namespace

hipError_t launch_gemm_dz_bf16(const Problem& pr, const SampleTable& st, int s0, int s1, int tile0, int tile1,
                               const void* dH, float* d_enc, float* d_pred, const ActiveTiles& at,
                               hipStream_t stream) {
    const int n = tile1 - tile0;
    if (n <= 0) return hipSuccess;
    if (pr.V % ZK != 0) return hipErrorInvalidValue;
    DzArgs g{(const bf16_t*)dH, (const bf16_t*)pr.W, pr, st, s0, s1, tile0, tile1, d_enc, d_pred,
             (n + 3) / 4, (pr.H + ZT - 1) / ZT, (long long)n * 64, at};
    const size_t smem = (size_t)ZST * Z_STAGE;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_dz256),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int m8 = (g.m_tiles + 7) / 8 * 8;
    k_gemm_dz256<<<dim3((unsigned)(m8 * g.n_tiles)), dim3(256), smem, stream>>>(g);
    return hipGetLastError();
}

}  // namespace rnnt
