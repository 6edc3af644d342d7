// C-ABI entry points (include/rnnt_joint_loss.h): argument checks, the host schedule, and the
// launch sequence.  Compiled with hipcc as host code; the kernels live in the .hip files.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <initializer_list>
#include <vector>

#include "../../include/rnnt_joint_loss.h"
#include "../../include/rnnt_joint_loss_debug.h"
#include "kernels.h"
#include "plan.h"

using namespace rnnt;

extern "C" const char* rnnt_status_string(rnnt_status s) {
    switch (s) {
        case RNNT_OK: return "ok";
        case RNNT_ERR_NULL: return "null pointer argument";
        case RNNT_ERR_SHAPE: return "shape or blank index out of range";
        case RNNT_ERR_LENGTH: return "T_len or U_len out of range";
        case RNNT_ERR_LABEL: return "label out of range";
        case RNNT_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case RNNT_ERR_UNSUPPORTED: return "shape not supported for this dtype";
        case RNNT_ERR_HIP: return "HIP runtime error";
        case RNNT_ERR_WEIGHT: return "a sample weight is negative or not finite";
    }
    return "unknown status";
}

static void fill_info(const rnnt_desc& d, const Plan& p, rnnt_plan_info* info) {
    info->rows_total = p.rows_total;
    info->rows_padded = (int64_t)d.B * d.T_max * (d.U_max + 1);
    info->tiles_total = p.tiles_total;
    info->n_groups = (int32_t)p.groups.size();
    info->n_chunks = (int32_t)p.chunks.size();
    info->group_rows_cap = p.group_rows_cap;
    info->chunk_rows = p.chunk_rows;
    info->workspace_bytes = p.total_bytes;
    info->lattice_bytes = p.lattice_bytes;
    info->chunk_bytes = p.chunk_bytes;
}

extern "C" size_t rnnt_joint_loss_workspace_bytes(const rnnt_desc* desc, const int32_t* T_len,
                                                  const int32_t* U_len, size_t budget_bytes) {
    if (check_desc(desc) != RNNT_OK || check_lengths(desc, T_len, U_len) != RNNT_OK) return 0;
    Plan p;
    build_plan(*desc, T_len, U_len, budget_bytes, p);
    return p.total_bytes;
}

extern "C" rnnt_status rnnt_joint_loss_plan(const rnnt_desc* desc, const int32_t* T_len, const int32_t* U_len,
                                            size_t workspace_bytes, rnnt_plan_info* info, int32_t* sample_group) {
    rnnt_status st = check_desc(desc);
    if (st != RNNT_OK) return st;
    st = check_lengths(desc, T_len, U_len);
    if (st != RNNT_OK) return st;
    if (!info) return RNNT_ERR_NULL;
    Plan p;
    build_plan(*desc, T_len, U_len, workspace_bytes, p);
    if (workspace_bytes != 0 && p.total_bytes > workspace_bytes) return RNNT_ERR_WORKSPACE;
    fill_info(*desc, p, info);
    if (sample_group)
        for (int g = 0; g < (int)p.groups.size(); ++g)
            for (int s = p.groups[g].s0; s < p.groups[g].s1; ++s) sample_group[s] = g;
    return RNNT_OK;
}

extern "C" int32_t rnnt_parallel_iterations(int64_t T, int64_t U, int64_t V) {
    if (T <= 0 || U <= 0 || V <= 0) return 0;
    const double ratio = 1e9 / (4.0 * (double)T * (double)U * (double)V);
    int e = (int)std::floor(std::log(ratio) / std::log(2.0));
    if (e > 4) e = 4;
    if (e < 0) e = 0;
    return 1 << e;
}

extern "C" rnnt_status rnnt_validate_labels_host(const rnnt_desc* desc, const int32_t* labels,
                                                 const int32_t* U_len) {
    rnnt_status st = check_desc(desc);
    if (st != RNNT_OK) return st;
    if (!labels || !U_len) return RNNT_ERR_NULL;
    for (int b = 0; b < desc->B; ++b) {
        if (U_len[b] < 0 || U_len[b] > desc->U_max) return RNNT_ERR_LENGTH;
        for (int u = 0; u < U_len[b]; ++u) {
            const int32_t y = labels[(size_t)b * desc->U_max + u];
            if (y < 0 || y >= desc->V) return RNNT_ERR_LABEL;
        }
    }
    return RNNT_OK;
}

namespace {

// Optional per-kernel timing with HIP events on the caller's stream (off by default).
enum KernelClass { KC_PREPARE = 0, KC_FWD_SCORES, KC_LATTICE, KC_BWD_SCORES, KC_GEMM_DZ, KC_GEMM_DW,
                   KC_BWD_FUSED, KC_FWD_F32, KC_BWD_F32, KC_DW_REDUCE, KC_PROJ, KC_FWD_KEEP, KC_KEPT_TO_DH,
                   KC_GRADS_TO_BF16, KC_SELECT, KC_COUNT };
const char* const kKernelNames[KC_COUNT] = {"prepare", "joint_scores_fwd", "lattice",
                                            "joint_scores_bwd", "gemm_dz", "gemm_dw_db", "joint_bwd_fused",
                                            "fwd_f32", "bwd_f32", "dw_reduce", "projections",
                                            "joint_scores_fwd_keep", "kept_scores_to_dh", "input_grads_to_bf16",
                                            "select_tiles"};
struct Profiler {
    bool enabled = false;
    struct Rec { int cls; hipEvent_t e0, e1; };
    std::vector<Rec> recs;
    std::vector<hipEvent_t> pool;
    hipEvent_t get() {
        if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
    void clear() {
        for (auto& r : recs) { pool.push_back(r.e0); pool.push_back(r.e1); }
        recs.clear();
    }
};
Profiler g_prof;

template <typename F>
hipError_t timed(int cls, hipStream_t stream, F&& launch) {
    if (!g_prof.enabled) return launch();
    hipEvent_t e0 = g_prof.get(), e1 = g_prof.get();
    if (!e0 || !e1) return hipErrorOutOfMemory;
    hipError_t e = hipEventRecord(e0, stream);
    if (e != hipSuccess) return e;
    e = launch();
    if (e != hipSuccess) return e;
    e = hipEventRecord(e1, stream);
    g_prof.recs.push_back({cls, e0, e1});
    return e;
}

// What the last failed HIP call was (process-wide, for rnnt_last_hip_error).
hipError_t g_last_hip_error = hipSuccess;
int g_last_hip_line = 0;

#define RNNT_HIP(expr)                           \
    do {                                         \
        const hipError_t rnnt_e_ = (expr);       \
        if (rnnt_e_ != hipSuccess) {             \
            g_last_hip_error = rnnt_e_;          \
            g_last_hip_line = __LINE__;          \
            (void)hipGetLastError();             \
            return RNNT_ERR_HIP;                 \
        }                                        \
    } while (0)

// Host tables -> device without a copy engine and without touching host memory after the call returns: the
// values travel as kernel arguments (at most 960 ints per launch), which the runtime captures at launch.
struct TableChunk {
    int n;
    int v[960];
};
__global__ void k_put_table(TableChunk c, int* __restrict__ dst) {
    for (int i = threadIdx.x; i < c.n; i += blockDim.x) dst[i] = c.v[i];
}
hipError_t put_table(const unsigned char* src, size_t bytes, void* dst, hipStream_t stream) {
    // bytes is a multiple of 4 (all tables are int32 / int64 / float)
    const size_t n = bytes / 4;
    const int* s = reinterpret_cast<const int*>(src);
    for (size_t at = 0; at < n; at += 960) {
        TableChunk c;
        c.n = (int)std::min<size_t>(960, n - at);
        std::memcpy(c.v, s + at, (size_t)c.n * 4);
        k_put_table<<<dim3(1), dim3(256), 0, stream>>>(c, reinterpret_cast<int*>(dst) + at);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}
// tables of at most this many bytes always travel that way (a pageable host-to-device copy makes the host wait
// for the stream; a few small launches do not)
constexpr size_t TABLE_BY_KERNEL_MAX = 8 * 960 * 4;

struct WsView {
    SampleTable st;
    LatticeState ls;   // row_base filled per group
    void* wpack;
    void* wq;
    void* dH;
    void* Z;
    float* dZ32;
    float* kept_max;
    float* stage_enc;
    float* stage_pred;
    float* dw_slots;
};

WsView view_workspace(const Plan& p, void* ws) {
    unsigned char* w = (unsigned char*)ws;
    WsView v{};
    v.st.T = (const int*)(w + p.off_T);
    v.st.U = (const int*)(w + p.off_U);
    v.st.tile_off = (const int*)(w + p.off_tile_off);
    v.st.row_off = (const long long*)(w + p.off_row_off);
    v.st.tile_sample = (const int*)(w + p.off_tile_sample);
    v.ls.lse = (float*)(w + p.off_lse);
    v.ls.lpb = (float*)(w + p.off_lpb);
    v.ls.lpy = (float*)(w + p.off_lpy);
    v.ls.alpha = (float*)(w + p.off_alpha);
    v.ls.beta = (float*)(w + p.off_beta);
    v.ls.lnP = (float*)(w + p.off_lnP);
    v.ls.shift = (float*)(w + p.off_shift);
    v.ls.row_base = 0;
    v.ls.tile_esum = p.bf16 ? (float*)(w + p.off_tile_esum) : nullptr;
    v.wpack = w + p.off_wpack;
    v.wq = w + p.off_wq;
    v.dH = w + p.off_dh;
    v.Z = w + p.off_z;
    v.dZ32 = (float*)(w + p.off_dz32);
    v.kept_max = (float*)(w + p.off_kept_max);
    v.stage_enc = (float*)(w + p.off_stage_enc);
    v.stage_pred = (float*)(w + p.off_stage_pred);
    v.dw_slots = (float*)(w + p.off_dwslots);
    return v;
}

// How the host tables reach the workspace.
struct TableSource {
    const unsigned char* staged = nullptr;   // tables laid out as in the workspace (from plan.off_T on), or null
    bool staged_pinned = false;              // `staged` is pinned host memory that outlives the call
    bool no_copy_engine = false;             // kernel arguments only
};
// Second stream for the lattice sweeps, with the events that order it against the main stream.
struct Overlap {
    hipStream_t lattice_stream = nullptr;
    hipEvent_t* fwd_done = nullptr;          // [groups]
    hipEvent_t* lat_done = nullptr;          // [groups]
};

size_t table_bytes(const Plan& plan, size_t B) { return plan.off_row_off + (B + 1) * 8 - plan.off_T; }

void fill_tables(const Plan& plan, size_t B, const int32_t* T_len, const int32_t* U_len, unsigned char* tab) {
    std::memset(tab, 0, table_bytes(plan, B));
    std::memcpy(tab, T_len, B * 4);
    std::memcpy(tab + (plan.off_U - plan.off_T), U_len, B * 4);
    std::memcpy(tab + (plan.off_tile_off - plan.off_T), plan.tile_off.data(), (B + 1) * 4);
    std::memcpy(tab + (plan.off_row_off - plan.off_T), plan.row_off.data(), (B + 1) * 8);
}

rnnt_status check_call(const rnnt_desc* desc, const void* enc, const void* pred, const void* W_out,
                       const float* b_out, const int32_t* labels, float* loss, void* d_enc_out, void* d_pred_out,
                       float* dW_out, float* db_out, bool grads, const float* sample_weight) {
    if (!enc || !pred || !W_out || !b_out || !loss) return RNNT_ERR_NULL;
    if (desc->U_max > 0 && !labels) return RNNT_ERR_NULL;
    if (grads && (!d_enc_out || !d_pred_out || !dW_out || !db_out)) return RNNT_ERR_NULL;
    // the MFMA kernels read and write these arrays in 16-byte pieces
    if (desc->dtype == RNNT_BF16 || f32_gemm_shape(desc->H, desc->V))
        for (const void* q : {enc, pred, W_out, (const void*)b_out, (const void*)d_enc_out, (const void*)d_pred_out,
                              (const void*)dW_out, (const void*)db_out})
            if ((uintptr_t)q % 16 != 0) return RNNT_ERR_UNSUPPORTED;
    if (sample_weight)
        for (int b = 0; b < desc->B; ++b)
            if (!(sample_weight[b] >= 0.0f) || !std::isfinite(sample_weight[b])) return RNNT_ERR_WEIGHT;
    return RNNT_OK;
}

// The launch sequence of one call for a plan that fits the workspace.
rnnt_status execute(const rnnt_desc* desc, const Plan& plan, const int32_t* T_len, const int32_t* U_len,
                    const TableSource& ts, const Overlap& ov, const void* enc, const void* pred, const void* W_out,
                    const float* b_out, const int32_t* labels, float* loss, void* d_enc_out, void* d_pred_out,
                    float* dW_out, float* db_out, void* workspace, void* hip_stream, bool grads,
                    const float* sample_weight) {
    hipStream_t stream = (hipStream_t)hip_stream;
    const WsView wv = view_workspace(plan, workspace);
    unsigned char* w = (unsigned char*)workspace;
    const size_t B = (size_t)desc->B;
    {
        const size_t tab_bytes = table_bytes(plan, B);
        if (ts.staged && ts.staged_pinned && !ts.no_copy_engine) {
            // pinned source owned by the plan handle: a truly asynchronous copy
            RNNT_HIP(hipMemcpyAsync(w + plan.off_T, ts.staged, tab_bytes, hipMemcpyHostToDevice, stream));
        } else {
            std::vector<unsigned char> tab;
            const unsigned char* src = ts.staged;
            if (!src) {
                tab.resize(tab_bytes);
                fill_tables(plan, B, T_len, U_len, tab.data());
                src = tab.data();
            }
            // small tables travel as kernel arguments (a pageable host-to-device copy makes the host wait for
            // the stream; a few small launches do not); large ones by one copy, consumed before the call returns
            if (ts.no_copy_engine || tab_bytes <= TABLE_BY_KERNEL_MAX)
                RNNT_HIP(put_table(src, tab_bytes, w + plan.off_T, stream));
            else
                RNNT_HIP(hipMemcpyAsync(w + plan.off_T, src, tab_bytes, hipMemcpyHostToDevice, stream));
        }
        if (sample_weight)
            RNNT_HIP(put_table(reinterpret_cast<const unsigned char*>(sample_weight), B * 4, w + plan.off_weight, stream));
    }

    Problem pr{desc->B, desc->T_max, desc->U_max, desc->H, desc->V, desc->blank, enc, pred, W_out, b_out, labels};
    const bool bf16 = (desc->dtype == RNNT_BF16);
    // bf16 d_enc / d_pred: the kernels add into fp32 arrays of one group's samples in the workspace
    const bool stage = plan.stage && grads;
    float* d_enc = stage ? nullptr : (float*)d_enc_out;
    float* d_pred = stage ? nullptr : (float*)d_pred_out;
    const size_t enc_per_sample = (size_t)desc->T_max * desc->H, pred_per_sample = (size_t)(desc->U_max + 1) * desc->H;
    GradOut go{d_enc, d_pred, dW_out, db_out};
    {
        PrepArgs pa{};
        if (grads) {
            pa.zero_ptr[0] = d_enc;                   // null with bf16 outputs: cleared per group below
            pa.zero_n[0] = B * enc_per_sample;
            pa.zero_ptr[1] = d_pred;
            pa.zero_n[1] = B * pred_per_sample;
            if (!desc->accumulate_params) {
                if (!bf16) {          // the bf16 path writes dW from its partial sums at the end
                    pa.zero_ptr[2] = dW_out;
                    pa.zero_n[2] = (size_t)desc->H * desc->V;
                }
                pa.zero_ptr[3] = db_out;
                pa.zero_n[3] = (size_t)desc->V;
            }
        }
        pa.tile_off = wv.st.tile_off;
        pa.tile_sample = (int*)(w + plan.off_tile_sample);
        pa.B = desc->B;
        pa.W = W_out;
        pa.Wp = bf16 ? wv.wpack : nullptr;
        pa.Wq = (plan.fused && grads) ? wv.wq : nullptr;
        pa.H = desc->H;
        pa.V = desc->V;
        RNNT_HIP(timed(KC_PREPARE, stream, [&] { return launch_prepare(pa, stream); }));
    }

    // fp32 path: sweeps of 128 steps or more accumulate in fp64 (the rounding of a dependent chain of fp32
    // log-add-exps grows with its length; short lattices stay inside the fp32 tolerance without it)
    const int wide_lattice = (!bf16 && desc->T_max + desc->U_max >= 128) ? 1 : 0;
    size_t ci = 0;
    int dw_first = 1;
    const bool keep = plan.keep && grads;
    const bool skip = plan.skip_log2 > 0 && grads;
    const float skip_log_floor = -(float)plan.skip_log2 * 0.6931471805599453f;
    // lattice state of group gi: with two buffers consecutive groups alternate between the halves of each array
    auto group_state = [&](size_t gi) {
        const Group& g = plan.groups[gi];
        LatticeState ls = wv.ls;
        const size_t half = (plan.lat_buffers == 2 && (gi & 1)) ? (size_t)plan.group_rows_cap : 0;
        ls.lse += half; ls.lpb += half; ls.lpy += half; ls.alpha += half; ls.beta += half;
        ls.row_base = plan.row_off[g.s0];
        ls.weight = sample_weight ? (const float*)(w + plan.off_weight) : nullptr;
        return ls;
    };
    // Eq. 4, Eq. 6, f^W_1 for one group
    auto forward = [&](size_t gi) -> rnnt_status {
        const Group& g = plan.groups[gi];
        const LatticeState ls = group_state(gi);
        if (keep)
            RNNT_HIP(timed(KC_FWD_KEEP, stream, [&] {
                return launch_fwd_keep_bf16(pr, wv.wpack, wv.st, ls, g.s0, g.s1, g.tile0, g.tile1, wv.dH, wv.Z,
                                            wv.kept_max, stream);
            }));
        else if (bf16)
            RNNT_HIP(timed(KC_FWD_SCORES, stream, [&] {
                return launch_fwd_bf16(pr, wv.wpack, wv.st, ls, g.s0, g.s1, g.tile0, g.tile1, stream);
            }));
        else if (plan.f32_gemm)
            for (long long r0 = 0; r0 < g.rows; r0 += plan.chunk_rows)
                RNNT_HIP(timed(KC_FWD_F32, stream, [&] {
                    return launch_fwd_f32_gemm(pr, wv.st, ls, g.s0, g.s1, r0, std::min(plan.chunk_rows, g.rows - r0),
                                               (float*)wv.dH, (float*)wv.Z, stream);
                }));
        else
            RNNT_HIP(timed(KC_FWD_F32, stream,
                           [&] { return launch_fwd_f32(pr, wv.st, ls, g.s0, g.s1, g.rows, stream); }));
        return RNNT_OK;
    };
    // f^W_2, f^W_3 for one group, on the given stream
    auto lattice = [&](size_t gi, hipStream_t on) -> rnnt_status {
        const Group& g = plan.groups[gi];
        const LatticeState ls = group_state(gi);
        RNNT_HIP(timed(KC_LATTICE, on,
                       [&] { return launch_lattice(wv.st, ls, g.s0, g.s1, g.u_max, wide_lattice, loss, on); }));
        if (skip)
            // tiles whose posteriors all lie below the floor are left out of this group's backward pass
            RNNT_HIP(timed(KC_SELECT, on, [&] {
                return launch_select_tiles(wv.st, ls, g.s0, g.s1, g.tile0, g.tile1, skip_log_floor,
                                           (int*)(w + plan.off_tile_esum), (int*)(w + plan.off_tile_esum),
                                           (int*)(w + plan.off_n_active) + gi, on);
            }));
        return RNNT_OK;
    };
    // f^W_4 and Algorithm 1 lines 8, 10, 11 for one group
    auto backward = [&](size_t gi) -> rnnt_status {
        const Group& g = plan.groups[gi];
        const LatticeState ls = group_state(gi);
        if (stage) {
            // the kernels index d_enc, d_pred by the sample's number in the call: base pointers such that
            // sample g.s0 is the first one of the (cleared) workspace arrays
            PrepArgs pz{};
            pz.zero_ptr[0] = wv.stage_enc;
            pz.zero_n[0] = (size_t)(g.s1 - g.s0) * enc_per_sample;
            pz.zero_ptr[1] = wv.stage_pred;
            pz.zero_n[1] = (size_t)(g.s1 - g.s0) * pred_per_sample;
            RNNT_HIP(timed(KC_PREPARE, stream, [&] { return launch_prepare(pz, stream); }));
            d_enc = (float*)((uintptr_t)wv.stage_enc - (uintptr_t)g.s0 * enc_per_sample * 4);
            d_pred = (float*)((uintptr_t)wv.stage_pred - (uintptr_t)g.s0 * pred_per_sample * 4);
        }
        for (; ci < plan.chunks.size() && plan.chunks[ci].group == (int)gi; ++ci) {
            if (!grads) continue;
            const Chunk& c = plan.chunks[ci];
            if (bf16) {
                const long long rows = (long long)(c.tile1 - c.tile0) * TILE_ROWS;
                // with a tile list the chunk takes entries [c.tile0 - g.tile0, c.tile1 - g.tile0) of the group's list
                // (kept scores: one chunk per group, filled tile by tile by the forward pass)
                const ActiveTiles at{skip ? (const int*)(w + plan.off_tile_esum) : nullptr,
                                     skip ? (const int*)(w + plan.off_n_active) + gi : nullptr, g.tile0,
                                     c.tile0 - g.tile0, keep ? c.tile0 : -1};
                if (keep && plan.fused) {
                    // the group's scores are in the chunk buffers already: the fused kernel turns them into dh
                    // on their way into the dz GEMM and writes dh back for the dW GEMM
                    RNNT_HIP(timed(KC_BWD_FUSED, stream, [&] {
                        return launch_bwd_fused_kept_bf16(pr, wv.wq, wv.st, ls, g.s0, g.s1, c.tile0, c.tile1, wv.dH,
                                                          wv.kept_max, d_enc, d_pred, at, stream);
                    }));
                } else if (keep) {
                    // ... or, for joint sizes the fused kernel does not cover, one pass turns them into dh
                    RNNT_HIP(timed(KC_KEPT_TO_DH, stream, [&] {
                        return launch_kept_to_dh_bf16(pr, wv.st, ls, g.s0, g.s1, c.tile0, c.tile1, wv.dH,
                                                      wv.kept_max, at, stream);
                    }));
                    RNNT_HIP(timed(KC_GEMM_DZ, stream, [&] {
                        return launch_gemm_dz_bf16(pr, wv.st, g.s0, g.s1, c.tile0, c.tile1, wv.dH, d_enc, d_pred,
                                                   at, stream);
                    }));
                } else if (plan.fused) {
                    RNNT_HIP(timed(KC_BWD_FUSED, stream, [&] {
                        return launch_bwd_fused_bf16(pr, wv.wpack, wv.wq, wv.st, ls, g.s0, g.s1, c.tile0, c.tile1,
                                                     wv.dH, wv.Z, d_enc, d_pred, at, stream);
                    }));
                } else {
                    RNNT_HIP(timed(KC_BWD_SCORES, stream, [&] {
                        return launch_bwd_scores_bf16(pr, wv.wpack, wv.st, ls, g.s0, g.s1, c.tile0, c.tile1, wv.dH,
                                                      wv.Z, at, stream);
                    }));
                    RNNT_HIP(timed(KC_GEMM_DZ, stream, [&] {
                        return launch_gemm_dz_bf16(pr, wv.st, g.s0, g.s1, c.tile0, c.tile1, wv.dH, d_enc, d_pred,
                                                   at, stream);
                    }));
                }
                RNNT_HIP(timed(KC_GEMM_DW, stream, [&] {
                    return launch_gemm_dw_bf16(desc->H, desc->V, rows, plan.dw_splits, dw_first, wv.Z, wv.dH,
                                               wv.dw_slots, db_out, at, stream);
                }));
                dw_first = 0;
            } else if (plan.f32_gemm) {
                RNNT_HIP(timed(KC_BWD_F32, stream, [&] {
                    return launch_bwd_f32_gemm(pr, wv.st, ls, go, g.s0, g.s1, c.row0, c.rows, (float*)wv.dH,
                                               (float*)wv.Z, wv.dZ32, stream);
                }));
            } else {
                RNNT_HIP(timed(KC_BWD_F32, stream,
                               [&] { return launch_bwd_f32(pr, wv.st, ls, go, g.s0, g.s1, g.rows, stream); }));
            }
        }
        if (stage) {
            // the group's sums, padded rows included (zeros), rounded into the caller's bf16 arrays
            RNNT_HIP(timed(KC_GRADS_TO_BF16, stream, [&] {
                return launch_f32_to_bf16(wv.stage_enc, (unsigned char*)d_enc_out + (size_t)g.s0 * enc_per_sample * 2,
                                          (size_t)(g.s1 - g.s0) * enc_per_sample, stream);
            }));
            RNNT_HIP(timed(KC_GRADS_TO_BF16, stream, [&] {
                return launch_f32_to_bf16(wv.stage_pred, (unsigned char*)d_pred_out + (size_t)g.s0 * pred_per_sample * 2,
                                          (size_t)(g.s1 - g.s0) * pred_per_sample, stream);
            }));
        }
        return RNNT_OK;
    };
    const size_t ng = plan.groups.size();
    rnnt_status stt = RNNT_OK;
    // The second stream takes the lattice sweeps.  Order on the main stream: forward(0), forward(1), backward(0),
    // forward(2), backward(1), ...: the sweep of group g+1 (latency-bound, a few workgroups per sample) runs beside
    // the backward pass of group g, whose lattice state lies in the other half of the lattice arrays.  Kept scores
    // occupy the chunk buffers from a group's forward to its backward pass, so that mode stays on one stream.
    const bool overlap = ov.lattice_stream && plan.lat_buffers == 2 && !keep && ng > 1;
    if (!overlap) {
        for (size_t gi = 0; gi < ng; ++gi) {
            if ((stt = forward(gi)) != RNNT_OK) return stt;
            if ((stt = lattice(gi, stream)) != RNNT_OK) return stt;
            if ((stt = backward(gi)) != RNNT_OK) return stt;
        }
    } else {
        auto forward_then_sweep = [&](size_t gi) -> rnnt_status {
            rnnt_status s2 = forward(gi);
            if (s2 != RNNT_OK) return s2;
            RNNT_HIP(hipEventRecord(ov.fwd_done[gi], stream));
            RNNT_HIP(hipStreamWaitEvent(ov.lattice_stream, ov.fwd_done[gi], 0));
            if ((s2 = lattice(gi, ov.lattice_stream)) != RNNT_OK) return s2;
            RNNT_HIP(hipEventRecord(ov.lat_done[gi], ov.lattice_stream));
            return RNNT_OK;
        };
        if ((stt = forward_then_sweep(0)) != RNNT_OK) return stt;
        for (size_t gi = 0; gi < ng; ++gi) {
            if (gi + 1 < ng && (stt = forward_then_sweep(gi + 1)) != RNNT_OK) return stt;
            RNNT_HIP(hipStreamWaitEvent(stream, ov.lat_done[gi], 0));
            if ((stt = backward(gi)) != RNNT_OK) return stt;
        }
    }
    if (bf16 && grads && !dw_first)
        RNNT_HIP(timed(KC_DW_REDUCE, stream, [&] {
            return launch_dw_reduce(desc->H, desc->V, plan.dw_splits, wv.dw_slots, dW_out, desc->accumulate_params,
                                    stream);
        }));
    return RNNT_OK;
}

rnnt_status run(const rnnt_desc* desc, const void* enc, const void* pred, const void* W_out, const float* b_out,
                const int32_t* labels, const int32_t* T_len, const int32_t* U_len, float* loss, void* d_enc_out,
                void* d_pred_out, float* dW_out, float* db_out, void* workspace, size_t workspace_bytes,
                void* hip_stream, bool grads, const float* sample_weight = nullptr, bool no_copy_engine = false) {
    rnnt_status stt = check_desc(desc);
    if (stt != RNNT_OK) return stt;
    if (!T_len || !U_len) return RNNT_ERR_NULL;
    stt = check_call(desc, enc, pred, W_out, b_out, labels, loss, d_enc_out, d_pred_out, dW_out, db_out, grads, nullptr);
    if (stt != RNNT_OK) return stt;
    stt = check_lengths(desc, T_len, U_len);
    if (stt != RNNT_OK) return stt;
    stt = check_call(desc, enc, pred, W_out, b_out, labels, loss, d_enc_out, d_pred_out, dW_out, db_out, grads,
                     sample_weight);
    if (stt != RNNT_OK) return stt;
    if (!workspace || ((uintptr_t)workspace % WS_ALIGN) != 0 || workspace_bytes == 0) return RNNT_ERR_WORKSPACE;
    Plan plan;
    build_plan(*desc, T_len, U_len, workspace_bytes, plan);
    if (plan.total_bytes > workspace_bytes) return RNNT_ERR_WORKSPACE;
    TableSource ts;
    ts.no_copy_engine = no_copy_engine;
    return execute(desc, plan, T_len, U_len, ts, Overlap{}, enc, pred, W_out, b_out, labels, loss, d_enc_out,
                   d_pred_out, dW_out, db_out, workspace, hip_stream, grads, sample_weight);
}

}  // namespace

// ---- a plan kept between calls ----------------------------------------------------------------------------
struct rnnt_plan_handle {
    rnnt_desc desc;
    std::vector<int32_t> T_len, U_len;
    Plan plan;
    unsigned char* tables = nullptr;     // the host tables as they lie in the workspace
    bool tables_pinned = false;
    std::vector<hipEvent_t> events;      // 2 per group once a call has used a second stream
};

extern "C" rnnt_status rnnt_plan_create(const rnnt_desc* desc, const int32_t* T_len, const int32_t* U_len,
                                        size_t budget_bytes, int32_t overlap_lattice, rnnt_plan_handle** out) {
    if (!out) return RNNT_ERR_NULL;
    *out = nullptr;
    rnnt_status stt = check_desc(desc);
    if (stt != RNNT_OK) return stt;
    stt = check_lengths(desc, T_len, U_len);
    if (stt != RNNT_OK) return stt;
    if (overlap_lattice != 0 && overlap_lattice != 1) return RNNT_ERR_SHAPE;
    rnnt_plan_handle* h = new (std::nothrow) rnnt_plan_handle();
    if (!h) return RNNT_ERR_NULL;
    h->desc = *desc;
    h->T_len.assign(T_len, T_len + desc->B);
    h->U_len.assign(U_len, U_len + desc->B);
    build_plan(*desc, T_len, U_len, budget_bytes, h->plan, overlap_lattice != 0);
    const size_t tb = table_bytes(h->plan, (size_t)desc->B);
    // pinned, so that the copy of a call never makes the host wait; ordinary memory where no GPU is present
    // (the plan can then still be inspected) or pinning fails
    void* pinned = nullptr;
    if (hipHostMalloc(&pinned, tb, hipHostMallocDefault) == hipSuccess && pinned) {
        h->tables = (unsigned char*)pinned;
        h->tables_pinned = true;
    } else {
        (void)hipGetLastError();
        h->tables = (unsigned char*)std::malloc(tb);
        if (!h->tables) { delete h; return RNNT_ERR_NULL; }
    }
    fill_tables(h->plan, (size_t)desc->B, T_len, U_len, h->tables);
    *out = h;
    return RNNT_OK;
}

extern "C" void rnnt_plan_destroy(rnnt_plan_handle* h) {
    if (!h) return;
    for (hipEvent_t e : h->events) (void)hipEventDestroy(e);
    if (h->tables_pinned) (void)hipHostFree(h->tables);
    else std::free(h->tables);
    delete h;
}

extern "C" size_t rnnt_plan_workspace_bytes(const rnnt_plan_handle* h) { return h ? h->plan.total_bytes : 0; }

extern "C" rnnt_status rnnt_plan_describe(const rnnt_plan_handle* h, rnnt_plan_info* info) {
    if (!h || !info) return RNNT_ERR_NULL;
    fill_info(h->desc, h->plan, info);
    return RNNT_OK;
}

extern "C" rnnt_status rnnt_joint_loss_fwd_bwd_planned(rnnt_plan_handle* h, const void* enc, const void* pred,
                                                       const void* W_out, const float* b_out, const int32_t* labels,
                                                       const float* sample_weight, float* loss, void* d_enc,
                                                       void* d_pred, float* dW_out, float* db_out, void* workspace,
                                                       size_t workspace_bytes, void* hip_stream,
                                                       void* hip_stream_lattice) {
    if (!h) return RNNT_ERR_NULL;
    rnnt_status stt = check_call(&h->desc, enc, pred, W_out, b_out, labels, loss, d_enc, d_pred, dW_out, db_out, true,
                                 sample_weight);
    if (stt != RNNT_OK) return stt;
    if (!workspace || ((uintptr_t)workspace % WS_ALIGN) != 0 || workspace_bytes < h->plan.total_bytes)
        return RNNT_ERR_WORKSPACE;
    Overlap ov;
    const size_t ng = h->plan.groups.size();
    if (hip_stream_lattice && hip_stream_lattice != hip_stream && h->plan.lat_buffers == 2 && ng > 1) {
        while (h->events.size() < 2 * ng) {
            hipEvent_t e = nullptr;
            RNNT_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
            h->events.push_back(e);
        }
        ov.lattice_stream = (hipStream_t)hip_stream_lattice;
        ov.fwd_done = h->events.data();
        ov.lat_done = h->events.data() + ng;
    }
    TableSource ts;
    ts.staged = h->tables;
    ts.staged_pinned = h->tables_pinned;
    return execute(&h->desc, h->plan, h->T_len.data(), h->U_len.data(), ts, ov, enc, pred, W_out, b_out, labels, loss,
                   d_enc, d_pred, dW_out, db_out, workspace, hip_stream, true, sample_weight);
}

extern "C" rnnt_status rnnt_joint_loss_fwd_bwd(const rnnt_desc* desc, const void* enc, const void* pred,
                                               const void* W_out, const float* b_out, const int32_t* labels,
                                               const int32_t* T_len, const int32_t* U_len, float* loss,
                                               void* d_enc, void* d_pred, float* dW_out, float* db_out,
                                               void* workspace, size_t workspace_bytes, void* hip_stream) {
    return run(desc, enc, pred, W_out, b_out, labels, T_len, U_len, loss, d_enc, d_pred, dW_out, db_out,
               workspace, workspace_bytes, hip_stream, true);
}

extern "C" rnnt_status rnnt_joint_loss_fwd_bwd_weighted(const rnnt_desc* desc, const void* enc, const void* pred,
                                                        const void* W_out, const float* b_out,
                                                        const int32_t* labels, const int32_t* T_len,
                                                        const int32_t* U_len, const float* sample_weight,
                                                        float* loss, void* d_enc, void* d_pred, float* dW_out,
                                                        float* db_out, void* workspace, size_t workspace_bytes,
                                                        void* hip_stream) {
    return run(desc, enc, pred, W_out, b_out, labels, T_len, U_len, loss, d_enc, d_pred, dW_out, db_out,
               workspace, workspace_bytes, hip_stream, true, sample_weight);
}

// ---- the entry point that allocates nothing --------------------------------------------------------------
// Its workspace is this array: every GPU the library runs on holds one copy until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; the address a kernel can use is looked up
// once per device and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[RNNT_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {};
}  // namespace

extern "C" rnnt_status rnnt_joint_loss_fwd_bwd_static(const rnnt_desc* desc, const void* enc, const void* pred,
                                                      const void* W_out, const float* b_out, const int32_t* labels,
                                                      const int32_t* T_len, const int32_t* U_len, float* loss,
                                                      void* d_enc, void* d_pred, float* dW_out, float* db_out,
                                                      void* hip_stream) {
    rnnt_status stt = check_desc(desc);
    if (stt != RNNT_OK) return stt;
    stt = check_lengths(desc, T_len, U_len);
    if (stt != RNNT_OK) return stt;
    if (desc->B > RNNT_STATIC_MAX_B) return RNNT_ERR_WORKSPACE;
    {
        // the smallest plan of this call must fit the array (host arithmetic only)
        Plan p;
        build_plan(*desc, T_len, U_len, RNNT_STATIC_SCRATCH_BYTES, p);
        if (p.total_bytes > (size_t)RNNT_STATIC_SCRATCH_BYTES) return RNNT_ERR_WORKSPACE;
    }
    int dev = -1;
    RNNT_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return RNNT_ERR_UNSUPPORTED;
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        RNNT_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return RNNT_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    return run(desc, enc, pred, W_out, b_out, labels, T_len, U_len, loss, d_enc, d_pred, dW_out, db_out,
               g_scratch_ptr[dev], (size_t)RNNT_STATIC_SCRATCH_BYTES, hip_stream, true, nullptr, true);
}

namespace {

struct ProjLayout {
    size_t off_enc, off_pred, off_denc, off_dpred, bytes;
};
ProjLayout proj_layout(const rnnt_desc& d) {
    const size_t esz = d.dtype == RNNT_BF16 ? 2 : 4;
    const size_t ne = (size_t)d.B * d.T_max * d.H, np = (size_t)d.B * (d.U_max + 1) * d.H;
    ProjLayout l{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = (o + bytes + WS_ALIGN - 1) / WS_ALIGN * WS_ALIGN; return at; };
    l.off_enc = take(ne * esz);
    l.off_pred = take(np * esz);
    l.off_denc = take(ne * 4);
    l.off_dpred = take(np * 4);
    l.bytes = o;
    return l;
}
rnnt_status check_proj_dims(const rnnt_desc* d, int32_t H_A, int32_t H_L) {
    if (H_A < 1 || H_L < 1) return RNNT_ERR_SHAPE;
    if (d->input_grads_bf16) return RNNT_ERR_UNSUPPORTED;     // d_enc, d_pred are internal here and stay fp32
    if (H_A > 4096 || H_L > 4096) return RNNT_ERR_UNSUPPORTED;
    if (d->dtype == RNNT_BF16 && (H_A % 128 != 0 || H_L % 128 != 0)) return RNNT_ERR_UNSUPPORTED;
    return RNNT_OK;
}

}  // namespace

extern "C" size_t rnnt_joint_proj_workspace_bytes(const rnnt_desc* desc, int32_t H_A, int32_t H_L,
                                                  const int32_t* T_len, const int32_t* U_len, size_t budget_bytes) {
    if (check_desc(desc) != RNNT_OK || check_lengths(desc, T_len, U_len) != RNNT_OK) return 0;
    if (check_proj_dims(desc, H_A, H_L) != RNNT_OK) return 0;
    const ProjLayout l = proj_layout(*desc);
    Plan p;
    size_t inner_budget = 0;
    if (budget_bytes != 0) inner_budget = budget_bytes > l.bytes ? budget_bytes - l.bytes : 1;
    build_plan(*desc, T_len, U_len, inner_budget, p);
    return l.bytes + p.total_bytes;
}

extern "C" rnnt_status rnnt_joint_proj_loss_fwd_bwd(const rnnt_desc* desc, int32_t H_A, int32_t H_L, const void* hA,
                                                    const void* hL, const void* W_A, const float* b_Z,
                                                    const void* W_L, const void* W_out, const float* b_out,
                                                    const int32_t* labels, const int32_t* T_len,
                                                    const int32_t* U_len, float* loss, float* d_hA, float* d_hL,
                                                    float* dW_A, float* db_Z, float* dW_L, float* dW_out,
                                                    float* db_out, void* workspace, size_t workspace_bytes,
                                                    void* hip_stream) {
    rnnt_status stt = check_desc(desc);
    if (stt != RNNT_OK) return stt;
    stt = check_proj_dims(desc, H_A, H_L);
    if (stt != RNNT_OK) return stt;
    if (!hA || !hL || !W_A || !b_Z || !W_L || !d_hA || !d_hL || !dW_A || !db_Z || !dW_L) return RNNT_ERR_NULL;
    if (!W_out || !b_out || !loss || !dW_out || !db_out || !T_len || !U_len) return RNNT_ERR_NULL;
    stt = check_lengths(desc, T_len, U_len);
    if (stt != RNNT_OK) return stt;
    if (!workspace || ((uintptr_t)workspace % WS_ALIGN) != 0) return RNNT_ERR_WORKSPACE;
    const ProjLayout l = proj_layout(*desc);
    if (workspace_bytes <= l.bytes) return RNNT_ERR_WORKSPACE;
    {
        Plan p;
        build_plan(*desc, T_len, U_len, workspace_bytes - l.bytes, p);
        if (p.total_bytes > workspace_bytes - l.bytes) return RNNT_ERR_WORKSPACE;
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    unsigned char* w = (unsigned char*)workspace;
    void* enc = w + l.off_enc;
    void* pred = w + l.off_pred;
    float* d_enc = (float*)(w + l.off_denc);
    float* d_pred = (float*)(w + l.off_dpred);
    const int bf16 = desc->dtype == RNNT_BF16;
    const long long rows_a = (long long)desc->B * desc->T_max, rows_l = (long long)desc->B * (desc->U_max + 1);
    const int H = desc->H;

    // Eq. 4, the two linear maps.  The length tables of the inner call are not on the device yet:
    // the projections run over all rows and the padded ones, whose input may be anything, are
    // skipped by the inner path (never read), so no mask is needed here.
    const RowMask none{nullptr, 1, 0};
    RNNT_HIP(timed(KC_PROJ, stream, [&] { return launch_proj_forward(bf16, hA, rows_a, H_A, none, W_A, b_Z, H, enc, stream); }));
    RNNT_HIP(timed(KC_PROJ, stream, [&] { return launch_proj_forward(bf16, hL, rows_l, H_L, none, W_L, nullptr, H, pred, stream); }));

    stt = run(desc, enc, pred, W_out, b_out, labels, T_len, U_len, loss, d_enc, d_pred, dW_out, db_out,
              w + l.bytes, workspace_bytes - l.bytes, hip_stream, true);
    if (stt != RNNT_OK) return stt;

    // the inner call has put T_len, U_len at the start of its workspace (plan offsets off_T, off_U)
    Plan p;
    build_plan(*desc, T_len, U_len, workspace_bytes - l.bytes, p);
    const RowMask mask_a{(const int*)(w + l.bytes + p.off_T), desc->T_max, 0};
    const RowMask mask_l{(const int*)(w + l.bytes + p.off_U), desc->U_max + 1, 1};
    if (!desc->accumulate_params) {
        PrepArgs pa{};
        pa.zero_ptr[0] = dW_A;
        pa.zero_n[0] = (size_t)H_A * H;
        pa.zero_ptr[1] = dW_L;
        pa.zero_n[1] = (size_t)H_L * H;
        pa.zero_ptr[2] = db_Z;
        pa.zero_n[2] = (size_t)H;
        RNNT_HIP(timed(KC_PREPARE, stream, [&] { return launch_prepare(pa, stream); }));
    }
    RNNT_HIP(timed(KC_PROJ, stream, [&] { return launch_proj_backward_input(bf16, d_enc, rows_a, H, W_A, H_A, d_hA, stream); }));
    RNNT_HIP(timed(KC_PROJ, stream, [&] { return launch_proj_backward_input(bf16, d_pred, rows_l, H, W_L, H_L, d_hL, stream); }));
    RNNT_HIP(timed(KC_PROJ, stream, [&] { return launch_proj_backward_weight(bf16, hA, rows_a, H_A, mask_a, d_enc, H, dW_A, stream); }));
    RNNT_HIP(timed(KC_PROJ, stream, [&] { return launch_proj_backward_weight(bf16, hL, rows_l, H_L, mask_l, d_pred, H, dW_L, stream); }));
    RNNT_HIP(timed(KC_PROJ, stream, [&] { return launch_col_sum(d_enc, rows_a, H, db_Z, stream); }));
    return RNNT_OK;
}

extern "C" rnnt_status rnnt_joint_loss_fwd(const rnnt_desc* desc, const void* enc, const void* pred,
                                           const void* W_out, const float* b_out, const int32_t* labels,
                                           const int32_t* T_len, const int32_t* U_len, float* loss,
                                           void* workspace, size_t workspace_bytes, void* hip_stream) {
    return run(desc, enc, pred, W_out, b_out, labels, T_len, U_len, loss, nullptr, nullptr, nullptr, nullptr,
               workspace, workspace_bytes, hip_stream, false);
}

extern "C" rnnt_status rnnt_debug_read_lattice(const rnnt_desc* desc, const int32_t* T_len, const int32_t* U_len,
                                               const void* workspace, size_t workspace_bytes, int32_t b,
                                               float* alpha_host, float* beta_host) {
    rnnt_status stt = check_desc(desc);
    if (stt != RNNT_OK) return stt;
    stt = check_lengths(desc, T_len, U_len);
    if (stt != RNNT_OK) return stt;
    if (!workspace || !alpha_host || !beta_host) return RNNT_ERR_NULL;
    if (b < 0 || b >= desc->B) return RNNT_ERR_SHAPE;
    Plan plan;
    build_plan(*desc, T_len, U_len, workspace_bytes, plan);
    if (plan.total_bytes > workspace_bytes) return RNNT_ERR_WORKSPACE;
    if (plan.groups.size() != 1) return RNNT_ERR_UNSUPPORTED;
    const unsigned char* w = (const unsigned char*)workspace;
    const int T = T_len[b], U = U_len[b];
    const size_t n = (size_t)T * (U + 1);
    const size_t off = (size_t)plan.row_off[b] * 4;
    float shift = 0.0f;
    RNNT_HIP(hipDeviceSynchronize());
    RNNT_HIP(hipMemcpy(alpha_host, w + plan.off_alpha + off, n * 4, hipMemcpyDeviceToHost));
    RNNT_HIP(hipMemcpy(beta_host, w + plan.off_beta + off, n * 4, hipMemcpyDeviceToHost));
    RNNT_HIP(hipMemcpy(&shift, w + plan.off_shift + (size_t)b * 4, 4, hipMemcpyDeviceToHost));
    for (int t = 0; t < T; ++t)
        for (int u = 0; u <= U; ++u) {
            const size_t i = (size_t)t * (U + 1) + u;
            alpha_host[i] -= shift * (float)(t + u);
            beta_host[i] -= shift * (float)((T - t) + (U - u));
        }
    return RNNT_OK;
}

extern "C" rnnt_status rnnt_debug_read_active_tiles(const rnnt_desc* desc, const int32_t* T_len, const int32_t* U_len,
                                                    const void* workspace, size_t workspace_bytes,
                                                    int64_t* active_tiles, int64_t* all_tiles) {
    rnnt_status stt = check_desc(desc);
    if (stt != RNNT_OK) return stt;
    stt = check_lengths(desc, T_len, U_len);
    if (stt != RNNT_OK) return stt;
    if (!workspace || !active_tiles || !all_tiles) return RNNT_ERR_NULL;
    Plan plan;
    build_plan(*desc, T_len, U_len, workspace_bytes, plan);
    if (plan.total_bytes > workspace_bytes) return RNNT_ERR_WORKSPACE;
    *all_tiles = plan.tiles_total;
    *active_tiles = plan.tiles_total;
    if (plan.skip_log2 == 0) return RNNT_OK;
    std::vector<int> n(plan.groups.size());
    RNNT_HIP(hipDeviceSynchronize());
    RNNT_HIP(hipMemcpy(n.data(), (const unsigned char*)workspace + plan.off_n_active, n.size() * 4, hipMemcpyDeviceToHost));
    *active_tiles = 0;
    for (int v : n) *active_tiles += v;
    return RNNT_OK;
}

extern "C" rnnt_status rnnt_debug_copy_f32(const float* src, float* dst, size_t n, void* hip_stream) {
    if (!src || !dst) return RNNT_ERR_NULL;
    if (n % 4 != 0) return RNNT_ERR_SHAPE;
    RNNT_HIP(launch_copy_f32(src, dst, n, (hipStream_t)hip_stream));
    return RNNT_OK;
}

extern "C" rnnt_status rnnt_debug_mfma_loop(const void* frags, float* out, int32_t workgroups, int32_t iters,
                                            void* hip_stream) {
    if (!frags || !out) return RNNT_ERR_NULL;
    if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > 1000000) return RNNT_ERR_SHAPE;
    RNNT_HIP(launch_mfma_loop(frags, out, workgroups, iters, (hipStream_t)hip_stream));
    return RNNT_OK;
}

extern "C" rnnt_status rnnt_debug_stream_read(const void* src, size_t bytes, void* out, int32_t workgroups,
                                              int32_t iters, void* hip_stream) {
    if (!src || !out) return RNNT_ERR_NULL;
    if (bytes < 32768 || bytes % 32768 != 0 || bytes > ((size_t)1 << 32) || workgroups < 1 || workgroups > 65536 ||
        iters < 1 || iters > 1000000 || ((uintptr_t)src % 16) != 0 || ((uintptr_t)out % 16) != 0)
        return RNNT_ERR_SHAPE;
    RNNT_HIP(launch_stream_read(src, bytes, out, workgroups, iters, (hipStream_t)hip_stream));
    return RNNT_OK;
}

extern "C" rnnt_status rnnt_debug_mfma_loop_fp8(const void* frags, float* out, int32_t workgroups, int32_t iters,
                                                void* hip_stream) {
    if (!frags || !out) return RNNT_ERR_NULL;
    if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > 1000000) return RNNT_ERR_SHAPE;
    RNNT_HIP(launch_mfma_loop_fp8(frags, out, workgroups, iters, (hipStream_t)hip_stream));
    return RNNT_OK;
}

extern "C" const char* rnnt_last_hip_error(void) {
    static char text[160];
    if (g_last_hip_error == hipSuccess) return "";
    snprintf(text, sizeof text, "%s (%s) at api.cpp:%d", hipGetErrorName(g_last_hip_error),
             hipGetErrorString(g_last_hip_error), g_last_hip_line);
    return text;
}

extern "C" rnnt_status rnnt_profile_enable(int32_t enable) {
    g_prof.clear();
    g_prof.enabled = (enable != 0);
    return RNNT_OK;
}

extern "C" int32_t rnnt_profile_kernel_count(void) { return KC_COUNT; }

extern "C" const char* rnnt_profile_kernel_name(int32_t cls) {
    return (cls >= 0 && cls < KC_COUNT) ? kKernelNames[cls] : "";
}

extern "C" rnnt_status rnnt_profile_read(int32_t n, int64_t* launches, double* total_ms) {
    if (!launches || !total_ms) return RNNT_ERR_NULL;
    if (n < KC_COUNT) return RNNT_ERR_SHAPE;
    for (int i = 0; i < n; ++i) { launches[i] = 0; total_ms[i] = 0.0; }
    for (auto& r : g_prof.recs) {
        RNNT_HIP(hipEventSynchronize(r.e1));
        float ms = 0.0f;
        RNNT_HIP(hipEventElapsedTime(&ms, r.e0, r.e1));
        launches[r.cls] += 1;
        total_ms[r.cls] += ms;
    }
    g_prof.clear();
    return RNNT_OK;
}
