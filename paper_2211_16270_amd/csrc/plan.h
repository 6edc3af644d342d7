// Host-side scheduler: packs the samples of a call into groups and backward chunks and lays
// out the workspace.  Pure C++ (no HIP), so it is unit-testable without a GPU.
//
// The paper recovers parallelism lost by sample-wise processing by running several loop
// iterations of Algorithm 1 at once, as many as a memory limit allows (Section 4.1.2, Eq. 11).
// Here the same idea is a packing problem: samples are cut into lattice tiles of 64 nodes (8 frames x 8 label positions, or 16 x 4), the tiles of
// all samples of a *group* are processed by one launch, and a group holds as many samples as
// its per-node state (5 floats per lattice node) fits the workspace.  The backward pass walks a
// group in *chunks* of tiles whose bf16 score-gradient buffers fit the rest of the workspace.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/rnnt_joint_loss.h"

namespace rnnt {

constexpr int TILE_ROWS = 64;    // lattice tile: 8 frames x 8 label positions or 16 x 4 (kernels.h: tile_label_width)
constexpr int GEMM_TILE = 128;   // row granularity of the backward GEMMs (two lattice tiles)
constexpr size_t WS_ALIGN = 256;

struct Group {
    int s0, s1;          // samples [s0, s1)
    int tile0, tile1;    // global tile range
    long long rows;      // lattice nodes of the group
    int u_max;           // largest U_len in the group
};

struct Chunk {
    int group;
    int tile0, tile1;    // global tile range, inside the group's range
    long long row0 = 0, rows = 0;   // fp32 GEMM form: lattice nodes [row0, row0 + rows) of the group instead
};

struct Plan {
    int B = 0;
    bool bf16 = false;
    bool fused = false;                 // bf16 only: backward runs in the fused kernel
    bool f32_gemm = false;              // fp32 only: H, V multiples of 4 from 64 on, the steps run as fp32 MFMA GEMMs over chunks
    bool keep = false;                  // bf16 only: forward keeps the scores, one backward chunk per group
    bool stage = false;                 // bf16 only: d_enc, d_pred leave as bf16; fp32 sums of one group in the workspace
    long long stage_samples = 0;        // samples a group may hold then
    std::vector<int> tile_off;          // [B+1] cumulative tile counts
    std::vector<long long> row_off;     // [B+1] cumulative lattice nodes
    std::vector<Group> groups;
    std::vector<Chunk> chunks;
    long long rows_total = 0, tiles_total = 0;
    long long group_rows_cap = 0;       // lattice nodes a group may hold
    int lat_buffers = 1;                // 2: the lattice arrays hold two groups (group g uses half g % 2)
    long long chunk_rows = 0;           // rows (multiple of GEMM_TILE) of the chunk buffers (fp32 GEMM form: lattice nodes)
    // workspace layout (byte offsets)
    size_t off_T = 0, off_U = 0, off_weight = 0, off_tile_off = 0, off_row_off = 0, off_lnP = 0, off_shift = 0, off_tile_sample = 0;
    size_t off_tile_esum = 0;          // bf16: per-tile emission sums (float per tile)
    int skip_log2 = 0;                 // > 0: tiles whose posteriors all lie below 2^-skip_log2 stay out of the backward pass
    size_t off_n_active = 0;           // skip_log2 > 0: per group the number of tiles that stay (their list lies in the
                                       // tile_esum array, over the entries of the same tiles)
    size_t off_wpack = 0, off_wq = 0;
    size_t off_lse = 0, off_lpb = 0, off_lpy = 0, off_alpha = 0, off_beta = 0;
    size_t off_dh = 0, off_z = 0, off_kept_max = 0;
    size_t off_dz32 = 0;                // fp32 GEMM form: dZ [chunk_rows, H]; off_dh, off_z hold S and Z as fp32
    size_t off_stage_enc = 0, off_stage_pred = 0;   // fp32 [stage_samples, T_max, H], [stage_samples, U_max+1, H]
    size_t off_dwslots = 0;             // bf16: per-workgroup partial sums of the dW GEMM
    int dw_splits = 0;                  // bf16: K splits of the dW GEMM (a multiple of 8)
    size_t lattice_bytes = 0, chunk_bytes = 0, total_bytes = 0;
    size_t min_bytes = 0;               // smallest workable workspace
};

// A score gradient dh = gamma * softmax - posteriors is at most the node's posterior gamma in magnitude, and a
// magnitude below 2^-134 (half the smallest bfloat16 denormal) rounds to zero as bf16: with gamma < 2^-135 at every
// node of a tile, every operand the tile would feed into the backward GEMMs is exactly zero.
constexpr int ZERO_IN_BF16_LOG2 = 135;

// Shapes the fused backward kernel covers (its dz accumulators must fit the register file).
inline bool fused_backward_shape(int H, int V) { return H % 128 == 0 && H <= 640 && V % 256 == 0; }

// Shapes the fp32 GEMM form covers: rows of 16-byte pieces, and wide enough for 128 x 128 tiles to pay.
inline bool f32_gemm_shape(int H, int V) { return H % 4 == 0 && V % 4 == 0 && H >= 64 && V >= 64; }

// dW GEMM geometry: 256x256 output tiles, and as many K splits (a multiple of 8, one set per XCD) as
// give about one workgroup per compute unit.  Every (split, tile) workgroup owns a 256 KiB slot of
// partial sums in the workspace.
constexpr int DW_TILE = 256;
inline int dw_tiles(int H, int V) { return ((H + DW_TILE - 1) / DW_TILE) * (V / DW_TILE); }
inline int dw_split_count(int H, int V) {
    const int t = dw_tiles(H, V);
    return ((256 + t - 1) / t + 7) / 8 * 8;
}
inline size_t dw_slot_bytes(int H, int V) {
    return (size_t)dw_tiles(H, V) * dw_split_count(H, V) * DW_TILE * DW_TILE * 4;
}

// Argument checks shared by every entry point (no pointers to data arrays here).
rnnt_status check_desc(const rnnt_desc* d);
rnnt_status check_lengths(const rnnt_desc* d, const int32_t* T_len, const int32_t* U_len);

// Builds the plan for a workspace of `workspace_bytes` (0 = default trade-off).  If the size
// is below the smallest workable one, plan.total_bytes = plan.min_bytes > workspace_bytes and
// the group/chunk lists are those of the smallest plan.
// two_lattice_buffers: room for the lattice state of two groups at a time (for calls that run a group's lattice
// sweep on a second stream while the previous group's backward pass is still reading its own state).
void build_plan(const rnnt_desc& d, const int32_t* T_len, const int32_t* U_len,
                size_t workspace_bytes, Plan& plan, bool two_lattice_buffers = false);

}  // namespace rnnt
