"""Sweeps shaped like the paper's experiments (Section 5.1-5.2): joint size H = 1024, vocabulary V = 4096,
batch of 16 over a grid of T x U from 50 x 10 to 500 x 100, and batch sizes 1..1024 at 500 x 100, with the
paper's zero-padding scheme (padding grows linearly over the batch: acoustic 0 -> 9.3 %, labels 0 -> 45.8 %).

    python -m paper_2211_16270_amd.sweep grid     # speed over the T x U grid, three ways of running the batch
    python -m paper_2211_16270_amd.sweep batch    # speed and peak memory over the batch size
    python -m paper_2211_16270_amd.sweep keep     # scores kept (keep_scores = 1) against computed twice
    python -m paper_2211_16270_amd.sweep keep16   # the same at B = 16 only, with the time of each kernel
    python -m paper_2211_16270_amd.sweep fp32     # the grid and three batch sizes with fp32 inputs and arithmetic

Inputs are seeded random tensors made on the GPU, as in the paper's benchmark; bf16 inputs unless stated.
`run_case(..., return_tensors=True)` also hands back the inputs, lengths and outputs of the last step, which is
how the GPU tests check every way of running a batch against the float64 checker on the same tensors.
Ways of running a batch:
  packed      one call, true lengths: this library's default (padding removed, samples share launches)
  padded      one call, every length set to the maximum: what a computation on the padded batch costs
  one_by_one  B calls of one sample each, true lengths: the sample-wise loop without parallel iterations
  kept        packed, with keep_scores = 1 in the descriptor
Prints one markdown table.
"""
from __future__ import annotations

import sys
import time

import numpy as np


def paper_lengths(B: int, T: int, U: int):
    """Section 5.1: padding grows linearly over the batch, 0 -> 9.3 % of T and 0 -> 45.8 % of U."""
    f = np.arange(B, dtype=np.float64) / max(B - 1, 1)
    T_len = np.maximum(1, np.floor(T * (1.0 - 0.093 * f) + 0.5)).astype(np.int32)
    U_len = np.maximum(0, np.floor(U * (1.0 - 0.458 * f) + 0.5)).astype(np.int32)
    return T_len, U_len


def run_case(B, T, U, H, V, mode, steps=3, warmup=1, seed=2211, dtype="bf16", return_tensors=False):
    import torch
    from . import binding as Bd

    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    g = torch.Generator(device="cuda").manual_seed(seed)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    rdt = Bd.RNNT_BF16 if dtype == "bf16" else Bd.RNNT_F32
    enc = torch.randn(B, T, H, generator=g, device="cuda").to(tdt)
    pred = torch.randn(B, U + 1, H, generator=g, device="cuda").to(tdt)
    W = (torch.randn(H, V, generator=g, device="cuda") / H ** 0.5).to(tdt)
    b_out = torch.zeros(V, dtype=torch.float32, device="cuda")
    labels = torch.randint(1, V, (B, max(U, 1)), generator=g, device="cuda", dtype=torch.int32)
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()       # from here on: inputs (resident) + outputs + workspace
    T_len, U_len = paper_lengths(B, T, U)
    if mode == "padded":
        T_len[:] = T
        U_len[:] = U
    f32 = dict(dtype=torch.float32, device="cuda")
    loss = torch.empty(B, **f32)
    d_enc, d_pred = torch.empty(B, T, H, **f32), torch.empty(B, U + 1, H, **f32)
    dW, db = torch.empty(H, V, **f32), torch.empty(V, **f32)
    stream = torch.cuda.current_stream()
    if mode == "one_by_one":
        desc1 = Bd.make_desc(1, T, U, H, V, 0, rdt, accumulate_params=1)
        nb = max(Bd.rnnt_joint_loss_workspace_bytes(desc1, T_len[b:b + 1], U_len[b:b + 1]) for b in range(B))
        ws = Bd.Workspace(nb)

        def step():
            dW.zero_()
            db.zero_()
            for b in range(B):
                s = Bd.rnnt_joint_loss_fwd_bwd(desc1, enc[b:b + 1], pred[b:b + 1], W, b_out, labels[b:b + 1],
                                               T_len[b:b + 1], U_len[b:b + 1], loss[b:b + 1], d_enc[b:b + 1],
                                               d_pred[b:b + 1], dW, db, ws.buf, stream)
                assert s == 0, s
    else:
        desc = Bd.make_desc(B, T, U, H, V, 0, rdt, keep_scores=1 if mode == "kept" else 0)
        nb = Bd.rnnt_joint_loss_workspace_bytes(desc, T_len, U_len)
        ws = Bd.Workspace(nb)

        def step():
            s = Bd.rnnt_joint_loss_fwd_bwd(desc, enc, pred, W, b_out, labels, T_len, U_len, loss, d_enc, d_pred, dW, db,
                                           ws.buf, stream)
            assert s == 0, s

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    assert bool(torch.isfinite(loss).all())
    rows = int(np.sum(T_len.astype(np.int64) * (U_len + 1)))
    # share of the lattice tiles the backward pass worked on (tiles whose score gradients are all zero as bf16
    # operands are left out by default on the path that computes the scores twice)
    share = 1.0
    if mode != "one_by_one":
        st, act, tot = Bd.rnnt_debug_read_active_tiles(desc, T_len, U_len, ws.buf)
        assert st == 0, st
        share = act / tot
    res = dict(ms=dt * 1e3, samples_per_s=B / dt, peak_gb=torch.cuda.max_memory_allocated() / 1e9,
               workspace_gb=nb / 1e9, rows=rows, tile_share=share,
               pflops_exec=(2.0 + (4.0 if mode == "kept" else 6.0) * share) * rows * H * V / dt / 1e15,
               pflops_dense=6.0 * rows * H * V / dt / 1e15)
    if return_tensors:
        res["tensors"] = dict(enc=enc, pred=pred, W_out=W, b_out=b_out, labels=labels, T_len=T_len, U_len=U_len,
                              loss=loss, d_enc=d_enc, d_pred=d_pred, dW_out=dW, db_out=db)
    return res


def main(argv):
    which = argv[1] if len(argv) > 1 else "grid"
    H, V = 1024, 4096
    if which == "grid":
        print(f"B = 16, H = {H}, V = {V}, bf16; ms per step (samples/s)\n")
        print("| T x U | packed | padded | one_by_one | packed vs one_by_one | peak GB (packed) | tiles in the backward pass (packed) |")
        print("|---|---|---|---|---|---|---|")
        for T, U in [(50, 10), (100, 20), (139, 27), (232, 46), (300, 60), (400, 80), (500, 100)]:
            r = {m: run_case(16, T, U, H, V, m, steps=5 if T <= 232 else 3) for m in ("packed", "padded", "one_by_one")}
            print(f"| {T} x {U} | " + " | ".join(f"{r[m]['ms']:.2f} ({r[m]['samples_per_s']:.0f})"
                                                   for m in ("packed", "padded", "one_by_one"))
                  + f" | {r['one_by_one']['ms'] / r['packed']['ms']:.2f}x | {r['packed']['peak_gb']:.2f} | {r['packed']['tile_share']:.3f} |", flush=True)
    elif which == "batch":
        T, U = 500, 100
        print(f"T x U = {T} x {U}, H = {H}, V = {V}, bf16, packed\n")
        print("| B | ms per step | samples/s | tiles in the backward pass | executed PFLOP/s | 6 R H V / time, PFLOP/s | workspace GB | peak GB (inputs + outputs + workspace) |")
        print("|---|---|---|---|---|---|---|---|")
        for B in (1, 4, 16, 64, 256, 1024):
            r = run_case(B, T, U, H, V, "packed", steps=3 if B <= 64 else 2)
            print(f"| {B} | {r['ms']:.1f} | {r['samples_per_s']:.1f} | {r['tile_share']:.3f} | {r['pflops_exec']:.3f} | {r['pflops_dense']:.3f} | "
                  f"{r['workspace_gb']:.2f} | {r['peak_gb']:.2f} |", flush=True)
    elif which == "keep":
        T, U = 500, 100
        print(f"T x U = {T} x {U}, bf16, packed; ms per step and peak GB (inputs + outputs + workspace)\n")
        print("| H | V | B | computed twice: ms | peak GB | kept: ms | peak GB | time kept / twice |")
        print("|---|---|---|---|---|---|---|---|")
        for Hx, Vx, Bs in [(1024, 4096, (1, 16, 256, 1024)), (768, 4096, (16,)), (1024, 1024, (16,)), (640, 1024, (16,)),
                           (512, 8192, (16,))]:
            for B in Bs:
                r = {m: run_case(B, T, U, Hx, Vx, m, steps=3 if B <= 64 else 2) for m in ("packed", "kept")}
                print(f"| {Hx} | {Vx} | {B} | {r['packed']['ms']:.2f} | {r['packed']['peak_gb']:.2f} | {r['kept']['ms']:.2f} | "
                      f"{r['kept']['peak_gb']:.2f} | {r['kept']['ms'] / r['packed']['ms']:.3f} |", flush=True)
    elif which == "keep16":
        from . import binding as Bd
        Bd.rnnt_profile_enable(True)
        for mode in ("packed", "kept"):
            Bd.rnnt_profile_read()
            r = run_case(16, 500, 100, H, V, mode, steps=3, warmup=1)
            prof = Bd.rnnt_profile_read()
            print(f"{mode}: {r['ms']:.3f} ms per step, rows {r['rows']}, workspace {r['workspace_gb']:.2f} GB")
            for k, (c, ms) in prof.items():
                if c:
                    print(f"    {k:24s} launches per step {c // 4:3d}   {ms / 4:8.3f} ms per step")
    elif which == "fp32":
        print(f"H = {H}, V = {V}, fp32 inputs and arithmetic (fp32 MFMA GEMMs over chunks of lattice nodes), packed\n")
        print("| B | T x U | ms per step | samples/s | executed TFLOP/s | workspace GB | peak GB (inputs + outputs + workspace) |")
        print("|---|---|---|---|---|---|---|")
        cases = [(16, T, U) for T, U in [(50, 10), (100, 20), (139, 27), (232, 46), (300, 60), (400, 80), (500, 100)]]
        for B, T, U in cases + [(1, 500, 100), (64, 500, 100)]:
            r = run_case(B, T, U, H, V, "packed", steps=2, warmup=1, dtype="f32")
            print(f"| {B} | {T} x {U} | {r['ms']:.1f} | {r['samples_per_s']:.1f} | {r['pflops_exec'] * 1e3:.1f} | "
                  f"{r['workspace_gb']:.2f} | {r['peak_gb']:.2f} |", flush=True)
    else:
        raise SystemExit("usage: python -m paper_2211_16270_amd.sweep grid|batch|keep|keep16|fp32")


if __name__ == "__main__":
    main(sys.argv)
