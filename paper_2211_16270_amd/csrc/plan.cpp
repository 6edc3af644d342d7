// Host scheduler and workspace layout (see plan.h).  No HIP in this file.
#include "plan.h"

#include "kernels.h"

#include <algorithm>
#include <cmath>

namespace rnnt {

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

rnnt_status check_desc(const rnnt_desc* d) {
    if (!d) return RNNT_ERR_NULL;
    if (d->B < 1 || d->T_max < 1 || d->U_max < 0 || d->H < 1 || d->V < 2) return RNNT_ERR_SHAPE;
    if (d->blank < 0 || d->blank >= d->V) return RNNT_ERR_SHAPE;
    if (d->accumulate_params != 0 && d->accumulate_params != 1) return RNNT_ERR_SHAPE;
    if (d->keep_scores != 0 && d->keep_scores != 1) return RNNT_ERR_SHAPE;
    if (d->keep_scores && d->dtype != RNNT_BF16) return RNNT_ERR_UNSUPPORTED;
    if (d->input_grads_bf16 != 0 && d->input_grads_bf16 != 1) return RNNT_ERR_SHAPE;
    if (d->input_grads_bf16 && d->dtype != RNNT_BF16) return RNNT_ERR_UNSUPPORTED;
    if (d->dtype != RNNT_F32 && d->dtype != RNNT_BF16) return RNNT_ERR_UNSUPPORTED;
    if (d->skip_below_log2 < -1 || d->skip_below_log2 > 126) return RNNT_ERR_SHAPE;
    if (d->skip_below_log2 > 0 && d->dtype != RNNT_BF16)
        return RNNT_ERR_UNSUPPORTED;                            // the bf16 backward kernels take a tile list
    if (d->U_max > 1023) return RNNT_ERR_UNSUPPORTED;           // one lattice thread per label position
    if ((long long)d->T_max * (d->U_max + 1) > (1LL << 30)) return RNNT_ERR_UNSUPPORTED;
    if (d->dtype == RNNT_BF16) {
        if (d->H % 128 != 0 || d->H > 1024) return RNNT_ERR_UNSUPPORTED;
        if (d->V % 256 != 0) return RNNT_ERR_UNSUPPORTED;
    } else {
        if (d->H > 4096 || d->V > 16384) return RNNT_ERR_UNSUPPORTED;
    }
    return RNNT_OK;
}

rnnt_status check_lengths(const rnnt_desc* d, const int32_t* T_len, const int32_t* U_len) {
    if (!T_len || !U_len) return RNNT_ERR_NULL;
    for (int b = 0; b < d->B; ++b) {
        if (T_len[b] < 1 || T_len[b] > d->T_max) return RNNT_ERR_LENGTH;
        if (U_len[b] < 0 || U_len[b] > d->U_max) return RNNT_ERR_LENGTH;
    }
    return RNNT_OK;
}

namespace {

struct Sizes {
    size_t fixed;          // tables + packed W
    size_t chunk_row_bytes;
};

// Fills every offset for the given capacities and returns the total size.
size_t lay_out(const rnnt_desc& d, Plan& p, long long lat_cap, long long chunk_rows, long long stage_samples) {
    const size_t B = (size_t)d.B;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, WS_ALIGN); return at; };
    p.off_T = take(B * 4);
    p.off_U = take(B * 4);
    p.off_weight = take(B * 4);
    p.off_tile_off = take((B + 1) * 4);
    p.off_row_off = take((B + 1) * 8);
    p.off_lnP = take(B * 4);
    p.off_shift = take(B * 4);
    p.off_tile_sample = take((size_t)p.tiles_total * 4);
    p.off_tile_esum = take(p.bf16 ? (size_t)p.tiles_total * 4 : 0);
    // the list of tiles that take part in the backward pass is written over the emission sums of the same tiles
    // (the lattice pass has consumed them by then): only the per-group counts need room of their own
    p.off_n_active = take(p.skip_log2 ? B * 4 : 0);
    p.off_wpack = take(p.bf16 ? (size_t)d.H * d.V * 2 : 0);
    p.off_wq = take(p.fused ? (size_t)d.H * d.V * 2 : 0);
    p.dw_splits = p.bf16 ? dw_split_count(d.H, d.V) : 0;
    p.off_dwslots = take(p.bf16 ? dw_slot_bytes(d.H, d.V) : 0);
    size_t lat0 = o;
    // lat_buffers = 2: consecutive groups alternate between two halves of each array, so that one group's
    // lattice sweep can run while its neighbour's state is still in use
    const size_t lat_elems = (size_t)lat_cap * (size_t)p.lat_buffers;
    p.off_lse = take(lat_elems * 4);
    p.off_lpb = take(lat_elems * 4);
    p.off_lpy = take(lat_elems * 4);
    p.off_alpha = take(lat_elems * 4);
    p.off_beta = take(lat_elems * 4);
    p.lattice_bytes = o - lat0;
    size_t ch0 = o;
    if (p.bf16) {
        // the dz GEMM reads dH in tiles of 256 rows: the buffer ends on such a boundary
        p.off_dh = take(align_up((size_t)chunk_rows, 256) * chunk_pitch(d.V) * 2);
        p.off_z = take((size_t)chunk_rows * chunk_pitch(d.H) * 2);
        p.off_kept_max = take(p.keep ? (size_t)chunk_rows * (d.V / 64) * 4 : 0);
    } else if (p.f32_gemm) {
        p.off_dh = take((size_t)chunk_rows * d.V * 4);
        p.off_z = take((size_t)chunk_rows * d.H * 4);
        p.off_dz32 = take((size_t)chunk_rows * d.H * 4);
        p.off_kept_max = o;
    } else {
        p.off_dh = p.off_z = p.off_kept_max = o;
    }
    p.chunk_bytes = o - ch0;
    p.off_stage_enc = take((size_t)stage_samples * d.T_max * d.H * 4);
    p.off_stage_pred = take((size_t)stage_samples * (d.U_max + 1) * d.H * 4);
    p.stage_samples = stage_samples;
    p.group_rows_cap = lat_cap;
    p.chunk_rows = (p.bf16 || p.f32_gemm) ? chunk_rows : 0;
    p.total_bytes = o;
    return o;
}

}  // namespace

void build_plan(const rnnt_desc& d, const int32_t* T_len, const int32_t* U_len,
                size_t workspace_bytes, Plan& p, bool two_lattice_buffers) {
    const int B = d.B;
    p.B = B;
    p.lat_buffers = two_lattice_buffers ? 2 : 1;
    const long long lat_row_bytes = 20LL * p.lat_buffers;    // workspace bytes per lattice node a group may hold
    p.bf16 = (d.dtype == RNNT_BF16);
    p.keep = p.bf16 && d.keep_scores;
    p.fused = p.bf16 && fused_backward_shape(d.H, d.V);
    p.stage = p.bf16 && d.input_grads_bf16;
    // 0: on the bf16 paths, tiles whose score gradients are all zero as bf16 values are left out
    // (ZERO_IN_BF16_LOG2); -1: no tile is ever left out
    p.skip_log2 = d.skip_below_log2 > 0 ? d.skip_below_log2
                  : (d.skip_below_log2 == 0 && p.bf16) ? ZERO_IN_BF16_LOG2 : 0;
    p.f32_gemm = !p.bf16 && f32_gemm_shape(d.H, d.V);
    const bool chunked = p.bf16 || p.f32_gemm;
    const size_t stage_per_sample = ((size_t)d.T_max + d.U_max + 1) * d.H * 4;
    p.tile_off.assign(B + 1, 0);
    p.row_off.assign(B + 1, 0);
    long long max_rows = 0, max_tile_rows = 0;
    for (int b = 0; b < B; ++b) {
        long long rows = (long long)T_len[b] * (U_len[b] + 1);
        long long tiles = sample_tiles(T_len[b], U_len[b]);
        p.row_off[b + 1] = p.row_off[b] + rows;
        p.tile_off[b + 1] = (int)(p.tile_off[b] + tiles);
        max_rows = std::max(max_rows, rows);
        max_tile_rows = std::max(max_tile_rows, (long long)align_up((size_t)tiles * TILE_ROWS, GEMM_TILE));
    }
    p.rows_total = p.row_off[B];
    p.tiles_total = p.tile_off[B];
    // the most rows a chunk can hold: tile rows (bf16), lattice nodes (fp32 GEMM form)
    const long long all_tile_rows =
        (long long)align_up((size_t)(p.bf16 ? p.tiles_total * TILE_ROWS : p.rows_total), GEMM_TILE);
    const size_t crb = p.f32_gemm ? (size_t)4 * d.V + (size_t)8 * d.H
                       : !p.bf16  ? 0
                                  : (size_t)2 * chunk_pitch(d.V) + (size_t)2 * chunk_pitch(d.H) +
                                        (p.keep ? (size_t)(d.V / 64) * 4 : 0);
    // With kept scores a group's backward pass is one chunk: the chunk buffers hold whole samples.
    const long long chunk_floor = p.keep ? max_tile_rows : GEMM_TILE;

    // smallest workable plan: one (largest) sample per group, one GEMM tile of rows per chunk
    Plan tmp = p;
    p.min_bytes = lay_out(d, tmp, max_rows, chunked ? chunk_floor : 0, p.stage ? 1 : 0);

    // the default plan; a caller that passes exactly the size it was told gets exactly this plan back
    const long long lat_default = std::min(p.rows_total, std::max(max_rows, (256LL << 20) / lat_row_bytes));
    long long chunk_default = 0;
    if (chunked) {
        // 832 MiB: 768 MiB of rows at H = 512, V = 1024 plus the padding of their row pitch
        // kept scores: 8 GiB, so that a group still fills the GPU when a row takes 10 KB
        const unsigned long long budget = p.keep ? (8ULL << 30) : (832ULL << 20);
        long long by_bytes = (long long)(budget / crb) / GEMM_TILE * GEMM_TILE;
        chunk_default = std::min(all_tile_rows, std::max<long long>(chunk_floor, by_bytes));
    }
    // fp32 sums of d_enc, d_pred for the samples of a group: 256 MiB by default
    const long long stage_default =
        !p.stage ? 0 : std::min<long long>(B, std::max<long long>(1, (long long)((256ULL << 20) / stage_per_sample)));
    Plan dflt = p;
    const size_t default_bytes = lay_out(d, dflt, lat_default, chunk_default, stage_default);

    long long lat_cap, chunk_rows, stage_samples;
    if (workspace_bytes == 0 || workspace_bytes == default_bytes) {
        lat_cap = lat_default;
        chunk_rows = chunk_default;
        stage_samples = stage_default;
    } else if (workspace_bytes < p.min_bytes) {
        lat_cap = max_rows;
        chunk_rows = chunked ? chunk_floor : 0;
        stage_samples = p.stage ? 1 : 0;
    } else {
        // the fixed part and the alignment slack come off first
        Plan probe = p;
        size_t fixed = lay_out(d, probe, 0, 0, 0) + 10 * WS_ALIGN;
        size_t avail = workspace_bytes > fixed ? workspace_bytes - fixed : 0;
        // an eighth of the rest (at most the default) for the fp32 sums of a group
        stage_samples = !p.stage ? 0
                                 : std::min<long long>(stage_default,
                                                       std::max<long long>(1, (long long)(avail / 8 / stage_per_sample)));
        const size_t stage_bytes = (size_t)stage_samples * stage_per_sample;
        avail = avail > stage_bytes ? avail - stage_bytes : 0;
        if (!chunked) {
            lat_cap = std::min<long long>(p.rows_total, std::max<long long>(max_rows, (long long)(avail / lat_row_bytes)));
            chunk_rows = 0;
        } else {
            long long lat_quarter = (long long)(avail / 4 / lat_row_bytes);
            lat_cap = std::min(p.rows_total, std::max(max_rows, lat_quarter));
            size_t lat_bytes = (size_t)lat_cap * lat_row_bytes;
            size_t rest = avail > lat_bytes ? avail - lat_bytes : 0;
            chunk_rows = (long long)(rest / crb) / GEMM_TILE * GEMM_TILE;
            chunk_rows = std::min(all_tile_rows, std::max<long long>(chunk_floor, chunk_rows));
            // what the chunk buffers do not need goes to the lattice
            size_t chunk_bytes = (size_t)chunk_rows * crb;
            if (avail > chunk_bytes) {
                long long more = (long long)((avail - chunk_bytes) / lat_row_bytes);
                lat_cap = std::min(p.rows_total, std::max(lat_cap, more));
            }
        }
        // never below the minimum, never above the given size
        Plan t2 = p;
        while (lay_out(d, t2, lat_cap, chunk_rows, stage_samples) > workspace_bytes) {
            if (chunk_rows > chunk_floor) chunk_rows -= GEMM_TILE;
            else if (lat_cap > max_rows) lat_cap = std::max(max_rows, lat_cap - 4096);
            else if (stage_samples > 1) --stage_samples;
            else break;
        }
    }
    // the kernels index a group's lattice state with 32-bit integers (a sample alone has at most 2^30 nodes)
    lat_cap = std::min<long long>(lat_cap, 2147483647LL);
    lay_out(d, p, lat_cap, chunk_rows, stage_samples);
    if (workspace_bytes != 0 && workspace_bytes < p.min_bytes) p.total_bytes = p.min_bytes;

    // groups: consecutive samples while the lattice state fits
    p.groups.clear();
    p.chunks.clear();
    int s = 0;
    while (s < B) {
        Group g{};
        g.s0 = s;
        g.rows = 0;
        g.u_max = 0;
        while (s < B) {
            long long rows = p.row_off[s + 1] - p.row_off[s];
            if (g.rows > 0 && g.rows + rows > lat_cap) break;
            if (p.stage && s - g.s0 >= stage_samples) break;
            if (p.keep && g.rows > 0 &&
                (long long)align_up((size_t)(p.tile_off[s + 1] - p.tile_off[g.s0]) * TILE_ROWS, GEMM_TILE) > chunk_rows)
                break;
            g.rows += rows;
            g.u_max = std::max(g.u_max, (int)U_len[s]);
            ++s;
        }
        g.s1 = s;
        g.tile0 = p.tile_off[g.s0];
        g.tile1 = p.tile_off[g.s1];
        p.groups.push_back(g);
    }
    // backward chunks of at most chunk_rows rows: a group that fits one chunk is one chunk; a larger one is cut
    // into chunks of whole rounds of 256 tiles where the chunk buffers hold at least four rounds (the last chunk
    // takes the rest), else into equal parts of an even number of tiles
    if (p.bf16 && !p.keep) {
        const long long cap_tiles = chunk_rows / TILE_ROWS;
        for (int gi = 0; gi < (int)p.groups.size(); ++gi) {
            const Group& g = p.groups[gi];
            long long n = g.tile1 - g.tile0;
            long long nch = (n + cap_tiles - 1) / cap_tiles;
            long long per = (n + nch - 1) / nch;
            per = std::min(cap_tiles, (per + 1) / 2 * 2);
            // the backward kernels run one workgroup per tile (fused kernel, dz GEMM: one per compute unit of the 256;
            // score kernel: one or two): chunks of whole rounds of 256 tiles leave no partly filled last round
            // (B=64, T<=500, U<=100, H=1024, V=4096: 5 rounds instead of 5.3 per chunk, both kernels -12 %)
            if (cap_tiles >= 1024 && n > cap_tiles) per = cap_tiles / 256 * 256;
            for (long long t = g.tile0; t < g.tile1; t += per) {
                Chunk c{gi, (int)t, (int)std::min<long long>(g.tile1, t + per)};
                p.chunks.push_back(c);
            }
        }
    } else if (p.f32_gemm) {
        // fp32 GEMM form: ranges of lattice nodes that fit the chunk buffers
        for (int gi = 0; gi < (int)p.groups.size(); ++gi) {
            const Group& g = p.groups[gi];
            for (long long r0 = 0; r0 < g.rows; r0 += chunk_rows) {
                Chunk c{gi, g.tile0, g.tile1};
                c.row0 = r0;
                c.rows = std::min(chunk_rows, g.rows - r0);
                p.chunks.push_back(c);
            }
        }
    } else {
        for (int gi = 0; gi < (int)p.groups.size(); ++gi)
            p.chunks.push_back(Chunk{gi, p.groups[gi].tile0, p.groups[gi].tile1});
    }
}

}  // namespace rnnt
