// Internal launch interface between the C-ABI layer (api.cpp) and the HIP kernels.
// Every function enqueues on `stream` and returns the launch status; none synchronises.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace rnnt {

// Device-resident description of the scheduled samples (one table per call).
struct SampleTable {
    const int* T;              // [B] T_len
    const int* U;              // [B] U_len
    const int* tile_off;       // [B+1] cumulative lattice-tile counts (64 nodes per tile)
    const int* tile_sample;    // [tiles] sample that owns each tile (filled by launch_prepare)
    const long long* row_off;  // [B+1] cumulative lattice-node counts
};

// Per-group lattice state; arrays are indexed by (row_off[s] - row_base) + t*(U_s+1) + u.
struct LatticeState {
    float* lse;    // ln of the softmax denominator (f^W_1)
    float* lpb;    // blank log-probability
    float* lpy;    // log-probability of label y_u (unused at u = U_s)
    float* alpha;  // forward variable, offset by shift*(t+u)
    float* beta;   // backward variable, offset by shift*((T-t)+(U-u))
    float* lnP;    // [B] ln P(y|x) + shift*(T+U), per sample
    float* shift;  // [B] per-sample offset added to every emission log-probability
    const float* weight;  // [B] weight of loss[b] in the differentiated sum, or null (all ones)
    float* tile_esum;     // [tiles of the call] sum over a tile's nodes of max(lpb, lpy) (lpb where there is no
                          // label), written by the bf16 forward kernels for the lattice kernels' offset; or null
    long long row_base;
};

struct Problem {
    int B, T_max, U_max, H, V, blank;
    const void* enc;
    const void* pred;
    const void* W;         // [H,V] as given by the caller
    const float* b_out;
    const int* labels;
};

struct GradOut {
    float* d_enc;
    float* d_pred;
    float* dW;
    float* db;
};

// Set-up of one call in a single launch: clears up to four float regions (null or empty ones are
// skipped), writes tile_sample[tile] = s for every tile of every sample (one lookup instead of a
// search per workgroup; skipped if tile_sample is null) and the fragment-major copies of W_out [H,V]
// (bf16): Wp for the A operand of the score GEMM, Wq for the dz GEMM (each skipped if null).
struct PrepArgs {
    float* zero_ptr[4];
    size_t zero_n[4];
    const int* tile_off;     // [B+1], device
    int* tile_sample;        // [tiles], device
    int B;
    const void* W;
    void* Wp;
    void* Wq;
    int H, V;
};
hipError_t launch_prepare(const PrepArgs& a, hipStream_t stream);
// dst[i] = bf16(src[i]), n a multiple of 8 (the gradients of a group, accumulated in fp32, on their way out)
hipError_t launch_f32_to_bf16(const float* src, void* dst, size_t n, hipStream_t stream);
// plain copy of n floats (n a multiple of 4): the known-size kernel the HBM counters are calibrated with
hipError_t launch_copy_f32(const float* src, float* dst, size_t n, hipStream_t stream);

// loop of workgroups x 4 waves x iters x 16 MFMAs (32x32x16 bf16) on the 32 x 1 KiB fragments at `frags`;
// writes workgroups x 256 floats to `out` (measurement support)
// every workgroup (256 threads) reads the same `bytes` (a multiple of 32 KiB) `iters` times; out: 4096 bytes per workgroup
hipError_t launch_stream_read(const void* src, size_t bytes, void* out, int workgroups, int iters, hipStream_t stream);
hipError_t launch_mfma_loop(const void* frags, float* out, int workgroups, int iters, hipStream_t stream);
// the same with the fp8 (e4m3) MFMA 32x32x64, unit scales: fragments of 64 lanes x 32 bytes (64 KiB in all)
hipError_t launch_mfma_loop_fp8(const void* frags, float* out, int workgroups, int iters, hipStream_t stream);

// ---- fp32 path (plain FMA kernels, any H, V) ------------------------------------------------
hipError_t launch_fwd_f32(const Problem& pr, const SampleTable& st, const LatticeState& ls,
                          int s0, int s1, long long rows, hipStream_t stream);
hipError_t launch_bwd_f32(const Problem& pr, const SampleTable& st, const LatticeState& ls,
                          const GradOut& go, int s0, int s1, long long rows, hipStream_t stream);

// fp32 MFMA GEMM form of the same two steps for H, V multiples of 4, over lattice nodes [r0, r0 + n) of the
// group (node index relative to the group's first).  S [rows, V], Z and dZ [rows, H] are chunk buffers of
// n rounded up to a multiple of 128 rows.
hipError_t launch_fwd_f32_gemm(const Problem& pr, const SampleTable& st, const LatticeState& ls, int s0, int s1,
                               long long r0, long long n, float* S, float* Z, hipStream_t stream);
hipError_t launch_bwd_f32_gemm(const Problem& pr, const SampleTable& st, const LatticeState& ls, const GradOut& go,
                               int s0, int s1, long long r0, long long n, float* S, float* Z, float* dZ,
                               hipStream_t stream);

// ---- lattice (alpha, beta, loss) ------------------------------------------------------------
// wide != 0: the sweep accumulates in fp64 (alpha, beta, ln P still stored as fp32); used by the fp32 path
hipError_t launch_lattice(const SampleTable& st, const LatticeState& ls, int s0, int s1, int u_max, int wide,
                          float* loss, hipStream_t stream);

// After the lattice pass of a group: flags[tile] = 1 for tiles [tile0, tile1) with a node whose posterior
// ln gamma = alpha + beta - ln P is at least log_floor, their ids in ascending order in active[tile0 ...] and their
// number in *n_active.
hipError_t launch_select_tiles(const SampleTable& st, const LatticeState& ls, int s0, int s1, int tile0, int tile1,
                               float log_floor, int* flags, int* active, int* n_active, hipStream_t stream);
// The tiles a backward launch works on: null active = tiles [tile0, tile1) one by one; else entry cbase + i of the
// group's list active[group_tile0 ...], for i below *n_active - cbase (workgroups beyond that return at once).
// Where a listed tile's 64 rows lie in the chunk buffers: in slot i (slot_tile0 < 0: the backward pass fills the
// buffers itself, densely), or in slot tile - slot_tile0 (kept scores: the forward pass has filled the buffers
// tile by tile before the list existed).
struct ActiveTiles {
    const int* active;
    const int* n_active;
    int group_tile0;
    int cbase;
    int slot_tile0;
};
constexpr ActiveTiles EVERY_TILE{nullptr, nullptr, 0, 0, -1};

// ---- bf16 MFMA path -------------------------------------------------------------------------
// joint tile in LDS -> scores on MFMA -> online log-softmax -> lse, lpb, lpy   (tiles [tile0,tile1))
hipError_t launch_fwd_bf16(const Problem& pr, const void* Wpack, const SampleTable& st,
                           const LatticeState& ls, int s0, int s1, int tile0, int tile1,
                           hipStream_t stream);
// joint tile -> scores recomputed -> dh (bf16) into the chunk buffers dH [rows,V], Z [rows,H]
hipError_t launch_bwd_scores_bf16(const Problem& pr, const void* Wpack, const SampleTable& st,
                                  const LatticeState& ls, int s0, int s1, int tile0, int tile1,
                                  void* dH, void* Z, const ActiveTiles& at, hipStream_t stream);
// The forward launch that also keeps the joint tiles (Z [rows,H]) and the scores (kept [rows,V]: fp16
// differences to the running maxima kept_max [tiles][V/64][64]) of tiles [tile0,tile1), and the launch that
// turns the kept scores into dh (bf16, in place) once alpha and beta are known.
hipError_t launch_fwd_keep_bf16(const Problem& pr, const void* Wpack, const SampleTable& st,
                                const LatticeState& ls, int s0, int s1, int tile0, int tile1, void* kept,
                                void* Z, float* kept_max, hipStream_t stream);
hipError_t launch_kept_to_dh_bf16(const Problem& pr, const SampleTable& st, const LatticeState& ls, int s0,
                                  int s1, int tile0, int tile1, void* kept, const float* kept_max,
                                  const ActiveTiles& at, hipStream_t stream);
// dz = dH W^T, times the tanh derivative, reduced over the tile's u resp. t, added to d_enc, d_pred
hipError_t launch_gemm_dz_bf16(const Problem& pr, const SampleTable& st, int s0, int s1, int tile0,
                               int tile1, const void* dH, float* d_enc, float* d_pred, const ActiveTiles& at,
                               hipStream_t stream);
// Shape of a sample's lattice tiles (64 rows each): 8 frames x 8 label positions, or 16 x 4 where that covers the
// sample's T x (U + 1) lattice with at least 3 % fewer tiles (the padding rows of partly filled tiles cost as
// much as real ones; a 16 x 4 tile adds to 20 rows of d_enc / d_pred instead of 16, which costs about 2 %).
// Returns the label positions per tile, 8 or 4; a tile then has 64 / that many frames, and row r of a tile is
// frame r / uw, label position r % uw.
__host__ __device__ inline int tile_label_width(int T, int U) {
    const long long a = (long long)((T + 7) / 8) * ((U + 8) / 8), b = (long long)((T + 15) / 16) * ((U + 4) / 4);
    return b * 33 < a * 32 ? 4 : 8;
}
__host__ __device__ inline long long sample_tiles(int T, int U) {
    const int uw = tile_label_width(T, U), th = 64 / uw;
    return (long long)((T + th - 1) / th) * ((U + uw) / uw);
}
// Row pitch (elements) of the two bf16 chunk buffers Z [rows, H] and dH [rows, V]: one 128-byte line more
// than the row, so that rows whose length is a power of two do not all start in the same memory channel.
__host__ __device__ inline int chunk_pitch(int n) { return n + 64; }

// fused backward: scores recomputed, dh, dz = dh W^T, tanh derivative, reductions into d_enc / d_pred;
// writes dH [rows,V] and Z [rows,H] (bf16, row-major) for the dW GEMM.  Wq is the second
// fragment-major copy of W_out.
hipError_t launch_bwd_fused_bf16(const Problem& pr, const void* Wpack, const void* Wq, const SampleTable& st,
                                 const LatticeState& ls, int s0, int s1, int tile0, int tile1, void* dH,
                                 void* Z, float* d_enc, float* d_pred, const ActiveTiles& at, hipStream_t stream);
// The same for scores the forward pass has kept (launch_fwd_keep_bf16): `kept` holds them and leaves as dH; Z is
// not touched.
hipError_t launch_bwd_fused_kept_bf16(const Problem& pr, const void* Wq, const SampleTable& st, const LatticeState& ls,
                                      int s0, int s1, int tile0, int tile1, void* kept, const float* kept_max,
                                      float* d_enc, float* d_pred, const ActiveTiles& at, hipStream_t stream);
// Split-K GEMM Z^T dH over one chunk's rows: every (split, tile) workgroup adds its 256x256 partial
// product to its own slot (`first` != 0: overwrites it), db += column sums of dH.  `splits` and the
// slot buffer size follow dw_split_count / dw_slot_bytes (plan.h).
// With at.active set the chunk holds only min(rows, 64 * (*at.n_active - at.cbase)) rows (read on the device).
hipError_t launch_gemm_dw_bf16(int H, int V, long long rows, int splits, int first, const void* Z,
                               const void* dH, float* slots, float* db, const ActiveTiles& at, hipStream_t stream);
// dW = (accumulate ? dW : 0) + sum of the slots over the splits
hipError_t launch_dw_reduce(int H, int V, int splits, const float* slots, float* dW, int accumulate,
                            hipStream_t stream);

// ---- input projections of the joint network (Eq. 4) and their backward -----------------------
// Row r of a [B*period, D] array is real data iff there is no mask (len == nullptr) or
// (r % period) < len[r / period] + extra; other rows are read as zero.
struct RowMask {
    const int* len;   // device, [B]
    int period;       // T_max, or U_max + 1
    int extra;        // 0 for frames (t < T_len), 1 for label positions (u <= U_len)
};
// out[r,:] = h[r,:] W + bias  (out in the input dtype; bias may be null)   h [rows,D], W [D,H]
hipError_t launch_proj_forward(int bf16, const void* h, long long rows, int D, const RowMask& mask, const void* W,
                               const float* bias, int H, void* out, hipStream_t stream);
// d_in[r,:] = d_out[r,:] W^T   (d_out fp32 [rows,H], zero in padded rows; d_in fp32 [rows,D])
hipError_t launch_proj_backward_input(int bf16, const float* d_out, long long rows, int H, const void* W, int D,
                                      float* d_in, hipStream_t stream);
// dW += h^T d_out over the real rows   (dW fp32 [D,H])
hipError_t launch_proj_backward_weight(int bf16, const void* h, long long rows, int D, const RowMask& mask,
                                       const float* d_out, int H, float* dW, hipStream_t stream);
// C[m,n] (+)= sum_k A(m,k) B(k,n) (+ bias[n]) in fp32 on the fp32 MFMA instruction, any M, N, K.  An operand
// is k-slow (element (i,k) at p[k*ld + i]) or k-contiguous (at p[i*ld + k]); combinations: A contiguous with
// either B, or both slow.  Rows of an operand's source array outside its mask read as zero.  atomic: C is
// added to with float atomics (required for splits > 1).  gemm_f32_edge_fits: the 16-byte alignment the
// kernel's loads need (extents along the contiguous index: K resp. M for A, K resp. N for B).
bool gemm_f32_edge_fits(const void* A, long long lda, const void* B, long long ldb, long long a_contig_extent,
                        long long b_contig_extent);
hipError_t launch_gemm_f32_masked(int a_kslow, int b_kslow, const float* A, long long lda, const RowMask& ma,
                                  const float* B, long long ldb, const RowMask& mb, float* C, long long ldc,
                                  const float* bias, int atomic, long long M, long long N, long long K, int splits,
                                  hipStream_t stream);
// out[c] += sum_r x[r,c]   (x fp32 [rows,cols])
hipError_t launch_col_sum(const float* x, long long rows, int cols, float* out, hipStream_t stream);

}  // namespace rnnt
