/*
 * rnnt_joint_loss.h - C ABI of the MI355X (gfx950) transducer joint -> loss -> gradient library.
 *
 * One call computes, for a batch of already projected acoustic and label encodings, what the
 * loop body of Algorithm 1 (arxiv 2211.16270, Section 4, lines 4-12) computes for every sample:
 * joint network (Eq. 4), output layer (Eq. 6), transducer loss f^W_1..f^W_4 (Eqs. 7-10) and the
 * gradients with respect to the output-layer parameters (line 8) and to both encodings
 * (lines 10, 11).  Padding is never touched (Section 4.1.1) and several samples share one launch
 * (Section 4.1.2); the [B,T,U+1,V] score tensor is never formed: scores live in MFMA
 * accumulators one tile at a time and are recomputed for the backward pass.
 *
 * Conventions
 *   - "dev" pointers are device memory of the current HIP device, "host" pointers are ordinary
 *     host memory.  All arrays are dense, row-major, last index contiguous.
 *   - The caller owns every buffer.  The library allocates no device memory, enqueues all work on the
 *     given stream and returns without waiting for it (host arrays are consumed before the call
 *     returns).  State it keeps between calls: none that changes a result; process-wide, the text of the
 *     last HIP error (rnnt_last_hip_error), the static workspace of rnnt_joint_loss_fwd_bwd_static, and,
 *     while the measurement hooks of rnnt_joint_loss_debug.h are switched on, their event records.
 *   - The length tables go to the GPU as kernel arguments while they are small (up to about 1200
 *     samples); beyond that by one host-to-device copy from pageable memory, which the runtime may
 *     complete only after earlier work on the stream has finished (the call then returns that much later).
 *   - Outputs must not alias inputs or each other.
 *   - Every entry point returns a status; nothing throws or aborts across this boundary.  All
 *     argument checks happen on the host before anything is launched.
 *   - Gradients are those of L = sum_b loss[b] (Section 2: L = -sum_b ln P(y_b|x_b)).
 */
#ifndef RNNT_JOINT_LOSS_H
#define RNNT_JOINT_LOSS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RNNT_OK = 0,
    RNNT_ERR_NULL = 1,        /* a required pointer is NULL                                   */
    RNNT_ERR_SHAPE = 2,       /* B, T_max, U_max, H, V or blank out of range                  */
    RNNT_ERR_LENGTH = 3,      /* some T_len[b] not in [1,T_max] or U_len[b] not in [0,U_max]  */
    RNNT_ERR_LABEL = 4,       /* a label outside [0,V) (only rnnt_validate_labels_host)       */
    RNNT_ERR_WORKSPACE = 5,   /* workspace NULL, misaligned (256 B) or too small              */
    RNNT_ERR_UNSUPPORTED = 6, /* shape not supported by the kernels of the requested dtype    */
    RNNT_ERR_HIP = 7,         /* a HIP call or launch failed                                  */
    RNNT_ERR_WEIGHT = 8       /* a sample weight is negative, NaN or infinite                 */
} rnnt_status;

typedef enum {
    RNNT_F32 = 0, /* enc, pred, W_out are float; everything is computed in fp32: the three      */
                  /* GEMMs on fp32 MFMA where H, V are multiples of 4 from 64 on, else plain FMA */
    RNNT_BF16 = 1 /* enc, pred, W_out are bfloat16; the three GEMMs run on bf16 MFMA with     */
                  /* fp32 accumulation, tanh/softmax/lattice in fp32                          */
} rnnt_dtype;

/* Problem description.  Lattice of sample b: 0 <= t < T_len[b], 0 <= u <= U_len[b]. */
typedef struct {
    int32_t B;      /* samples, >= 1                                                         */
    int32_t T_max;  /* rows of enc per sample, >= 1                                          */
    int32_t U_max;  /* label slots per sample, >= 0; pred has U_max + 1 rows, U_max <= 1023  */
    int32_t H;      /* joint size.  RNNT_BF16: multiple of 128, <= 1024.  RNNT_F32: 1..4096   */
    int32_t V;      /* vocabulary incl. blank.  RNNT_BF16: multiple of 256.  RNNT_F32: 2..16384 */
                    /* (another size: pad W_out with zero columns and b_out with -1e4 there; the  */
                    /* padding then has probability 0 and zero gradients)                         */
    int32_t blank;  /* index of the blank symbol, in [0,V)                                   */
    int32_t dtype;  /* rnnt_dtype                                                            */
    int32_t accumulate_params; /* 0: dW_out, db_out are overwritten; 1: added to (Alg. 1, line 3 / 8) */
    int32_t keep_scores;       /* RNNT_BF16 only.  0: the backward pass computes the scores a second time
                                  (the paper's trade: time for memory, Section 4).  1: the forward pass keeps
                                  the joint activations and the scores (fp16, relative to running row maxima)
                                  of a group of samples in the workspace and the backward pass reads them:
                                  three GEMMs per row instead of four, for 2 (H + V) more workspace bytes per
                                  lattice node of a group (the paper's outlook on other memory trade-offs,
                                  Section 6)                                                           */
    int32_t input_grads_bf16;  /* RNNT_BF16 only.  0: d_enc, d_pred are float.  1: they are bfloat16 arrays of
                                  the same shape (half the bytes of the two largest outputs): the sums are
                                  formed in float for one group of samples at a time in the workspace and
                                  rounded once (nearest even) on their way out (mixed precision, Section 6) */
    int32_t skip_below_log2;   /* Which 64-node lattice tiles take part in the backward pass (f^W_4 and Algorithm 1
                                  lines 8, 10, 11).  Every entry of a node's score gradient is at most the node's
                                  posterior gamma = exp(alpha + beta - ln P) in magnitude, and the alignments that
                                  carry the probability pass through a narrow band of a long lattice.
                                  0 (default): with RNNT_BF16, tiles in which every node has gamma < 2^-135 are
                                     left out: as bfloat16 MFMA operands their score gradients are all exactly zero
                                     (a magnitude below 2^-134 rounds to zero), so no term of any sum changes; only
                                     the order of the floating-point additions can.  With RNNT_F32 no tile is left
                                     out.
                                  -1: no tile is left out, anywhere.
                                  k = 1..126 (RNNT_BF16, else RNNT_ERR_UNSUPPORTED): tiles in
                                     which every node has gamma < 2^-k are left out; each gradient entry changes
                                     by less than 2^-k times the number of lattice nodes that add to it (with
                                     k = 30 four fifths of the tiles of a 750 x 140 lattice drop out).
                                  The loss is never affected.                                                  */
} rnnt_desc;

/* What the host scheduler decided for a call (Section 4.1.2 analogue; see rnnt_joint_loss_plan). */
typedef struct {
    int64_t rows_total;       /* sum_b T_len[b] * (U_len[b] + 1): lattice nodes without padding */
    int64_t rows_padded;      /* B * T_max * (U_max + 1)                                       */
    int64_t tiles_total;      /* 64-node lattice tiles (8 x 8 or 16 x 4 per sample) over all samples */
    int32_t n_groups;         /* launches of the forward/lattice stage; samples of a group run together */
    int32_t n_chunks;         /* launches of the backward stage (row ranges of <= chunk_rows)  */
    int64_t group_rows_cap;   /* lattice rows that fit one group                               */
    int64_t chunk_rows;       /* rows per backward chunk: tile-padded (bf16), lattice nodes    */
                              /* (fp32 GEMM form), 0 for the plain fp32 kernels                */
    size_t  workspace_bytes;  /* bytes the plan uses                                           */
    size_t  lattice_bytes;    /* part of it: lse, lpb, lpy, alpha, beta of one group           */
    size_t  chunk_bytes;      /* part of it: bf16 score-gradient / joint chunk buffers         */
} rnnt_plan_info;

const char* rnnt_status_string(rnnt_status s);
/* After a call returned RNNT_ERR_HIP: name and text of the HIP error and the library source line of the
 * call that reported it ("" if none so far).  Process-wide, overwritten by the next such failure. */
const char* rnnt_last_hip_error(void);

/*
 * Workspace size for a call (host only, no GPU needed).
 *   budget_bytes = 0: the library's default trade-off (never more than 1088 MiB plus, for bf16,
 *   the two packed copies of W_out and the partial sums of the dW GEMM, which depend on H and V
 *   only (partial sums: about 64 MiB while H*V <= 2^21, 32 bytes per element of W_out beyond),
 *   plus what the largest single sample needs; with desc->keep_scores the chunk buffers of that default
 *   hold up to 8 GiB, never more than the call's tile rows need, and the smallest plan holds the largest
 *   sample's rows: 2 (V + 64) + 2 (H + 64) + V / 16 bytes per row of its 64-node lattice tiles; with
 *   desc->input_grads_bf16 up to 256 MiB more, for the float sums of d_enc and d_pred of one group).
 *   RNNT_F32 with H and V multiples of 4, both >= 64, has chunk buffers too: 4 V + 8 H bytes per lattice node of a
 *   chunk (scores, joint activations and their gradients as float), 128 nodes in the smallest plan.
 *   Otherwise the largest plan not exceeding budget_bytes; if
 *   even the smallest workable plan (one sample per group, one tile row per chunk) exceeds it,
 *   that smallest size is returned, so a result > budget_bytes means "budget too small".
 * Returns 0 on invalid arguments.  Once the default cap is reached the result grows with B only by the
 * tables (28 bytes per sample, 8 bytes per 64-node lattice tile; Section 5.2: memory almost independent of
 * batch size).
 */
size_t rnnt_joint_loss_workspace_bytes(const rnnt_desc* desc, const int32_t* T_len_host,
                                       const int32_t* U_len_host, size_t budget_bytes);

/*
 * The schedule a call with this workspace size would use (host only).  sample_group, if not NULL,
 * receives for each of the B samples the index of the group it is processed in (every sample
 * is in exactly one group; a group's lattice state fits the workspace).
 */
rnnt_status rnnt_joint_loss_plan(const rnnt_desc* desc, const int32_t* T_len_host,
                                 const int32_t* U_len_host, size_t workspace_bytes,
                                 rnnt_plan_info* info, int32_t* sample_group);

/* Eq. (11): the paper's number of concurrently processed samples, 2^max(0,min(4,floor(log2(1e9/(4TUV))))).
 * Kept for reference next to this library's own grouping rule; returns 0 on non-positive input. */
int32_t rnnt_parallel_iterations(int64_t T, int64_t U, int64_t V);

/* Host-side label check: RNNT_ERR_LABEL if some labels[b*U_max + u], u < U_len[b], is outside [0,V).
 * The GPU path never indexes memory with a label; an out-of-range label there yields loss = +inf. */
rnnt_status rnnt_validate_labels_host(const rnnt_desc* desc, const int32_t* labels_host,
                                      const int32_t* U_len_host);

/*
 * Loss and gradients (Algorithm 1, lines 4-12, for all samples; Eqs. 4, 6, 7-10).
 *
 *   z[b,t,u,:] = tanh(enc[b,t,:] + pred[b,u,:])                (Eq. 4; the projections W^A, W^L, b^Z
 *                                                               are applied by the caller beforehand)
 *   h[b,t,u,:] = z[b,t,u,:] W_out + b_out                      (Eq. 6; W_out is the transpose of the
 *                                                               paper's W^O in R^{V x H})
 *   loss[b]    = -ln P(y_b | x_b), natural log                 (Eqs. 7-9)
 *   dW_out, db_out, d_enc, d_pred: gradients of sum_b loss[b]  (Eq. 10; Alg. 1 lines 8, 10, 11)
 *
 * enc      dev  [B, T_max, H]      desc->dtype; rows t >= T_len[b] are never read
 * pred     dev  [B, U_max+1, H]    desc->dtype; rows u >  U_len[b] are never read
 * W_out    dev  [H, V]             desc->dtype
 * b_out    dev  [V]                float
 * labels   dev  [B, U_max]         int32, entries u >= U_len[b] are never read
 * T_len    HOST [B]                1..T_max
 * U_len    HOST [B]                0..U_max
 * loss     dev  [B]                float, out
 * d_enc    dev  [B, T_max, H]      float (bfloat16 if desc->input_grads_bf16), out, fully overwritten
 *                                  (zeros in padded rows)
 * d_pred   dev  [B, U_max+1, H]    the same type, out, fully overwritten (zeros in padded rows)
 * dW_out   dev  [H, V]             float, out (overwritten or accumulated, see desc)
 * db_out   dev  [V]                float, out (same)
 * enc, pred, W_out, b_out, d_enc, d_pred, dW_out, db_out are 16-byte aligned (RNNT_ERR_UNSUPPORTED otherwise;
 * not required for RNNT_F32 shapes that take the plain FMA kernels).
 * workspace dev, 256-byte aligned, workspace_bytes >= rnnt_joint_loss_workspace_bytes(...);
 *          a larger workspace lets more samples share a launch
 * hip_stream  a hipStream_t (NULL = the default stream)
 *
 * Floating-point sums into d_enc, d_pred and db_out (on the fp32 path also dW_out) use atomic
 * adds, so those results can differ in the last bits from run to run; the bf16 path's dW_out is
 * summed in a fixed order.  Calls that share a workspace must be ordered on one stream.
 * The call enqueues its launches and returns without waiting; it must not be recorded into a HIP graph:
 * its first operation copies the length tables from host memory the call owns only until it returns, and
 * the schedule (number and size of the launches) is a function of those lengths.
 */
rnnt_status rnnt_joint_loss_fwd_bwd(const rnnt_desc* desc,
                                    const void* enc, const void* pred, const void* W_out,
                                    const float* b_out, const int32_t* labels,
                                    const int32_t* T_len_host, const int32_t* U_len_host,
                                    float* loss, void* d_enc, void* d_pred,
                                    float* dW_out, float* db_out,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The same with one weight per sample: loss[b] is still -ln P(y_b|x_b), the gradients are those of
 * sum_b sample_weight[b] * loss[b] (Section 3: the criterion is a sum over the samples, so a
 * training loop's mean reduction, loss masks or gradient scaling are such weights; Algorithm 1
 * lines 8-11 with every sample's posterior weights scaled).  sample_weight: HOST [B], every entry
 * finite and >= 0 (else RNNT_ERR_WEIGHT, before any launch); NULL means all ones, i.e. exactly
 * rnnt_joint_loss_fwd_bwd.  A weight of 0 leaves that sample out of every gradient.  Everything
 * else (layouts, workspace, ownership, errors, stream order) as above.
 */
rnnt_status rnnt_joint_loss_fwd_bwd_weighted(const rnnt_desc* desc,
                                             const void* enc, const void* pred, const void* W_out,
                                             const float* b_out, const int32_t* labels,
                                             const int32_t* T_len_host, const int32_t* U_len_host,
                                             const float* sample_weight_host,
                                             float* loss, void* d_enc, void* d_pred,
                                             float* dW_out, float* db_out,
                                             void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * rnnt_joint_loss_fwd_bwd for callers that cannot allocate device memory or provide a workspace (code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the workspace is an array of
 * RNNT_STATIC_SCRATCH_BYTES that is part of the library's device code, one copy per GPU the library runs on, held
 * until the process ends.  The call allocates nothing, on the device or through the runtime: no hipMalloc /
 * hipFree, and the length tables reach the GPU as kernel arguments instead of through a host-to-device copy.
 * Same inputs, outputs, layouts and results as rnnt_joint_loss_fwd_bwd with a workspace of that size (the same
 * schedule, so dW_out is bit-identical and the other sums agree up to the order of their atomic additions).
 *   RNNT_ERR_WORKSPACE  the call's smallest plan does not fit the array (the packed copies of W_out, 4 H V bytes,
 *                       the dW partial sums, about 64 MiB while H V <= 2^21, 20 bytes per lattice node of the
 *                       largest sample and one 128-row backward chunk must fit), or B > RNNT_STATIC_MAX_B
 *   other errors as rnnt_joint_loss_fwd_bwd
 * Nothing in the array has to be cleared between calls (every part is written before it is read within a call);
 * it keeps the last call's contents.  All calls on one GPU share the one array: calls that overlap on a GPU
 * (different streams or threads) race; order them on one stream.
 */
#define RNNT_STATIC_SCRATCH_BYTES (128u << 20)
#define RNNT_STATIC_MAX_B 8192
rnnt_status rnnt_joint_loss_fwd_bwd_static(const rnnt_desc* desc,
                                           const void* enc, const void* pred, const void* W_out,
                                           const float* b_out, const int32_t* labels,
                                           const int32_t* T_len_host, const int32_t* U_len_host,
                                           float* loss, void* d_enc, void* d_pred,
                                           float* dW_out, float* db_out, void* hip_stream);

/*
 * The same call for a training loop that repeats one batch geometry (Algorithm 1's loop body is run once per
 * training step): the schedule of Section 4.1.2's analogue is worked out once and kept in a handle, so a call
 * neither rebuilds it nor touches pageable host memory.
 *
 * rnnt_plan_create      checks desc and the lengths, builds the schedule for budget_bytes (meaning as in
 *                       rnnt_joint_loss_workspace_bytes; 0 = default) and stores the length tables in pinned host
 *                       memory (ordinary memory if no GPU is present or pinning fails).  overlap_lattice = 1 lays
 *                       the workspace out with room for the lattice state of two groups of samples (each then
 *                       half as large by default), which lets a call run every group's lattice sweep (f^W_2,
 *                       depth T + U, a few workgroups per sample) on a second stream beside the previous group's
 *                       backward pass.  The handle is host memory owned by the caller; HIP events are added to it
 *                       by the first call that uses a second stream.  Not thread-safe per handle.
 * rnnt_plan_workspace_bytes   workspace size calls with this handle need (0 for NULL)
 * rnnt_plan_describe    the schedule, as rnnt_joint_loss_plan reports it
 * rnnt_plan_destroy     frees the handle (NULL is allowed); the caller makes sure no call using it is still
 *                       running on the GPU
 * rnnt_joint_loss_fwd_bwd_planned   rnnt_joint_loss_fwd_bwd_weighted for the handle's desc and lengths
 *                       (sample_weight_host NULL = all ones).  hip_stream_lattice: NULL, or a second stream of
 *                       the same priority on the same device; used only if the handle was created with
 *                       overlap_lattice = 1, the call has more than one group and desc->keep_scores = 0.  The
 *                       lattice sweeps then run there, ordered against hip_stream by events (no host wait);
 *                       when the call returns, everything the second stream was given is ordered before the
 *                       end of the work on hip_stream, so the caller synchronises hip_stream only.  Results are
 *                       those of the one-stream call with the same schedule.
 */
typedef struct rnnt_plan_handle rnnt_plan_handle;
rnnt_status rnnt_plan_create(const rnnt_desc* desc, const int32_t* T_len_host, const int32_t* U_len_host,
                             size_t budget_bytes, int32_t overlap_lattice, rnnt_plan_handle** plan);
size_t rnnt_plan_workspace_bytes(const rnnt_plan_handle* plan);
rnnt_status rnnt_plan_describe(const rnnt_plan_handle* plan, rnnt_plan_info* info);
void rnnt_plan_destroy(rnnt_plan_handle* plan);
rnnt_status rnnt_joint_loss_fwd_bwd_planned(rnnt_plan_handle* plan,
                                            const void* enc, const void* pred, const void* W_out,
                                            const float* b_out, const int32_t* labels,
                                            const float* sample_weight_host,
                                            float* loss, void* d_enc, void* d_pred,
                                            float* dW_out, float* db_out,
                                            void* workspace, size_t workspace_bytes,
                                            void* hip_stream, void* hip_stream_lattice);

/*
 * Loss only (Eqs. 4, 6, 7-9): same inputs, no gradient outputs, same workspace rule
 * (the chunk buffers stay unused).
 */
rnnt_status rnnt_joint_loss_fwd(const rnnt_desc* desc,
                                const void* enc, const void* pred, const void* W_out,
                                const float* b_out, const int32_t* labels,
                                const int32_t* T_len_host, const int32_t* U_len_host,
                                float* loss, void* workspace, size_t workspace_bytes,
                                void* hip_stream);

/*
 * The same path with the joint network of Eq. (4) complete: the two input projections run inside
 * the call and the gradients are chained back through them (Algorithm 1 line 9 for theta^J, lines
 * 10-11 for the encodings).
 *
 *   enc[b,t,:]  = hA[b,t,:] W_A + b_Z          pred[b,u,:] = hL[b,u,:] W_L
 *   z[b,t,u,:]  = tanh(enc[b,t,:] + pred[b,u,:])                                      (Eq. 4)
 *   then as rnnt_joint_loss_fwd_bwd; in addition
 *   d_hA = d_enc W_A^T, dW_A = sum_{b,t} hA^T d_enc, db_Z = sum_{b,t} d_enc,
 *   d_hL = d_pred W_L^T, dW_L = sum_{b,u} hL^T d_pred.
 *
 * W_A [H_A, H] and W_L [H_L, H] are the transposes of the paper's W^A, W^L (H contiguous).
 * bf16: hA, hL, W_A, W_L bf16; the projections accumulate in fp32, add b_Z and are rounded to bf16
 * (they are the bf16 inputs of the joint kernels); d_enc, d_pred are rounded to bf16 as MFMA
 * operands of the three backward GEMMs.  H_A and H_L must be multiples of 128 (bf16) and at most 4096.
 *
 * hA    dev [B, T_max, H_A]    desc->dtype; rows t >= T_len[b] are never used (may hold NaN)
 * hL    dev [B, U_max+1, H_L]  desc->dtype; rows u >  U_len[b] are never used
 * W_A   dev [H_A, H], W_L dev [H_L, H]   desc->dtype;   b_Z dev [H] float
 * d_hA  dev [B, T_max, H_A] float, d_hL dev [B, U_max+1, H_L] float: out, fully overwritten, zeros in padded rows
 * dW_A, dW_L, db_Z: float, out; overwritten or accumulated like dW_out (desc->accumulate_params)
 * Everything else as in rnnt_joint_loss_fwd_bwd.  All device pointers 16-byte aligned.
 * workspace_bytes >= rnnt_joint_proj_workspace_bytes(...): the projected encodings and their
 * gradients ([B,T_max,H] and [B,U_max+1,H], desc->dtype resp. float) live there, in front of the
 * workspace of the inner path; budget_bytes (0 = default) applies to that inner part.
 */
size_t rnnt_joint_proj_workspace_bytes(const rnnt_desc* desc, int32_t H_A, int32_t H_L,
                                       const int32_t* T_len_host, const int32_t* U_len_host,
                                       size_t budget_bytes);
rnnt_status rnnt_joint_proj_loss_fwd_bwd(const rnnt_desc* desc, int32_t H_A, int32_t H_L,
                                         const void* hA, const void* hL, const void* W_A,
                                         const float* b_Z, const void* W_L,
                                         const void* W_out, const float* b_out, const int32_t* labels,
                                         const int32_t* T_len_host, const int32_t* U_len_host,
                                         float* loss, float* d_hA, float* d_hL, float* dW_A,
                                         float* db_Z, float* dW_L, float* dW_out, float* db_out,
                                         void* workspace, size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* RNNT_JOINT_LOSS_H */
