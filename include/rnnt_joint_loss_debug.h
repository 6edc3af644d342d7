/*
 * rnnt_joint_loss_debug.h - test and measurement hooks of the transducer joint -> loss -> gradient library.
 *
 * None of these is an operation of the method (arxiv 2211.16270); they exist so that tests can look at the
 * forward/backward variables the lattice pass leaves in the workspace, and so that the benchmark can time the
 * library's launches one by one and calibrate counters and peaks.  Same conventions as rnnt_joint_loss.h.
 * The timing hooks keep process-wide state and are not thread-safe.
 */
#ifndef RNNT_JOINT_LOSS_DEBUG_H
#define RNNT_JOINT_LOSS_DEBUG_H

#include "rnnt_joint_loss.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Test hook: copies the forward/backward variables of sample b (as left in the workspace by the
 * most recent call on this workspace, after the caller synchronised the stream) to host arrays
 * alpha_host, beta_host [T_len[b] * (U_len[b]+1)], undoing the per-sample offset the lattice
 * kernel works with, so they are the alpha, beta of Section 2 (f^W_2).  Only valid when the
 * call used a single group (info.n_groups == 1).  Synchronous.
 */
rnnt_status rnnt_debug_read_lattice(const rnnt_desc* desc, const int32_t* T_len_host,
                                    const int32_t* U_len_host, const void* workspace,
                                    size_t workspace_bytes, int32_t b,
                                    float* alpha_host, float* beta_host);

/*
 * Test and measurement hook: after a call with desc->skip_below_log2 > 0 on this workspace (same desc, lengths
 * and workspace size; stream synchronised by this function), the number of lattice tiles that went through the
 * backward pass and the number of all tiles.  With skip_below_log2 = 0 both are the number of all tiles.
 */
rnnt_status rnnt_debug_read_active_tiles(const rnnt_desc* desc, const int32_t* T_len_host,
                                         const int32_t* U_len_host, const void* workspace,
                                         size_t workspace_bytes, int64_t* active_tiles, int64_t* all_tiles);

/*
 * Measurement support, not a paper operation: copies n floats (n a multiple of 4, both dev, 16-byte
 * aligned) with a plain grid-stride kernel.  Its known size calibrates the HBM byte counters that
 * the per-kernel traffic figures are read from.  Enqueues on hip_stream, does not wait.
 */
rnnt_status rnnt_debug_copy_f32(const float* src, float* dst, size_t n, void* hip_stream);

/*
 * Measurement support (not a paper operation): a loop of nothing but bf16 MFMAs (32x32x16, fp32
 * accumulation) on operand values the caller chooses, to see what the matrix units sustain on such
 * values next to the published peak that the MFMA-bound kernels are priced against.
 *   frags  dev  32 fragments of 64 lanes x 8 bf16 (32 KiB): wave w of a workgroup uses fragments
 *               8w .. 8w+3 as A operands and 8w+4 .. 8w+7 as B operands
 *   out    dev  workgroups * 256 floats, overwritten (a checksum that keeps the loop alive)
 *   workgroups 1..65536 of 256 threads; iters 1..1000000 iterations of 16 MFMAs per wave:
 *               2 * 32*32*16 * 16 * iters * 4 * workgroups flop per launch
 * Enqueues on hip_stream, does not wait.  RNNT_ERR_NULL / RNNT_ERR_SHAPE on bad arguments.
 */
rnnt_status rnnt_debug_mfma_loop(const void* frags, float* out, int32_t workgroups, int32_t iters,
                                 void* hip_stream);
/* The same loop on the fp8 MFMA (e4m3 operands, 32x32x64, unit block scales, fp32 accumulation): frags holds 32
 * fragments of 64 lanes x 32 bytes (64 KiB); 2 * 32*32*64 * 16 * iters * 4 * workgroups flop per launch.  The path
 * itself has no fp8 kernel; this tells what one could gain. */
rnnt_status rnnt_debug_mfma_loop_fp8(const void* frags, float* out, int32_t workgroups, int32_t iters,
                                     void* hip_stream);

/*
 * Measurement support (not a paper operation): every workgroup (256 threads) reads the same array, 16 bytes per
 * lane and 1 KB per wave instruction, as the score kernels stream their W_out fragments.  With an array that stays
 * in the L2 this tells what the path from the L2 to the compute units delivers when all of them pull at once, the
 * other resource (besides the matrix units) those kernels depend on.
 *   src    dev  bytes to read: a multiple of 32 KiB, at most 4 GiB, 16-byte aligned
 *   out    dev  workgroups * 4096 bytes, overwritten (a checksum that keeps the loads alive)
 *   workgroups 1..65536; iters 1..1000000 passes over the array per workgroup:
 *               bytes * iters * workgroups bytes reach the compute units per launch
 * Enqueues on hip_stream, does not wait.  RNNT_ERR_NULL / RNNT_ERR_SHAPE on bad arguments.
 */
rnnt_status rnnt_debug_stream_read(const void* src, size_t bytes, void* out, int32_t workgroups, int32_t iters,
                                   void* hip_stream);

/*
 * Per-kernel timing for the benchmark (not a paper operation; measurement support for the
 * throughput figures reported against Table 1's cost terms).  While enabled, every launch made
 * by the entry points of rnnt_joint_loss.h is bracketed by HIP events recorded on the caller's stream
 * (process-wide state, not thread-safe).
 *   rnnt_profile_enable(1/0)    start (and clear) / stop recording
 *   rnnt_profile_kernel_count() number of kernel classes n
 *   rnnt_profile_kernel_name(i) name of class i, "" if out of range
 *   rnnt_profile_read(n, launches, total_ms)  waits for the recorded events, writes per class the
 *                               number of launches and the summed event time in ms (host arrays of
 *                               at least n entries), then clears the records
 */
rnnt_status rnnt_profile_enable(int32_t enable);
int32_t rnnt_profile_kernel_count(void);
const char* rnnt_profile_kernel_name(int32_t cls);
rnnt_status rnnt_profile_read(int32_t n, int64_t* launches_host, double* total_ms_host);

#ifdef __cplusplus
}
#endif
#endif /* RNNT_JOINT_LOSS_DEBUG_H */
