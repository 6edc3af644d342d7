#!/usr/bin/env python3
"""Benchmark of the fused joint + RNN-T loss + gradient call on one MI355X.

A step is one call of rnnt_joint_loss_fwd_bwd over one synthetic batch (the whole path:
joint tiles, score GEMM, softmax statistics, lattice, score gradients, backward GEMMs), with
all inputs already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C4|C2|C3|C5|C1|P16|P16F32] [--no-cpu-baseline]

The default workload is C4, the largest one a single GPU holds and the one the target is stated on
(B = 1024, T <= 1000, U <= 200, H = 512, V = 1024, bf16).  `value` is samples/s over K timed steps (whole
job, one GPU).  `roofline` describes the kernel that takes the most time: its ALGORITHMIC flops per launch
(2 H V per lattice node and contraction the method asks for: the scores once, dW_out, dz; scores that a
backward kernel computes a second time count as executed work only) divided by its average launch duration,
measured with HIP events recorded on the call's stream in a second pass over the same K steps (the events
are kept out of the pass that yields `value`); `exec_flops_per_launch` / `frac_exec` count what the kernel
really multiplies.  `roofline.traffic` is read from the committed rocprofv3 counter summary of this workload
under profiles/ (it is not measured in this run).  `cpu_baseline` is the float64 checker timed on the host
cores on a few samples of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_FLOPS = 2.5e15     # MI355X dense bf16 MFMA
PEAK_F32_FLOPS = 157.3e12    # MI355X fp32, vector and MFMA alike
CPU_SAMPLE = {"C1": 2, "C2": 32, "C3": 12, "C4": 12, "C5": 8}  # samples the checker is timed on (10-30 s)
COPY_BYTES = 256 << 20


def read_traffic(path):
    """{kernel: HBM bytes per launch} from a counter summary under profiles/ (lines of
    `kernel launches fetch_KiB write_KiB fetch_bytes write_bytes hbm_bytes_per_launch`)."""
    res = {}
    if not os.path.exists(path):
        return res
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        parts = line.split()
        res[parts[0]] = float(parts[-1])
    return res


def mfma_operand_patterns():
    """Operand fragments (bit patterns) for the MFMA-only loop: bf16 32 x 64 lanes x 8, e4m3 32 x 64 lanes x 32."""
    rng = np.random.Generator(np.random.PCG64(2211))
    n = 32 * 64 * 8
    sign = rng.integers(0, 2, n, dtype=np.uint16) << 15
    expo = (118 + rng.integers(0, 8, n, dtype=np.uint16)) << 7          # magnitudes 2^-9 .. 2^-2
    mant = rng.integers(0, 128, n, dtype=np.uint16)
    bf16 = [("zeros", np.zeros(n, dtype=np.uint16)), ("ones", np.full(n, 0x3F80, dtype=np.uint16)),
            ("random, 3 mantissa bits", sign | np.uint16(122 << 7) | (mant & 0x70)), ("random bf16", sign | expo | mant)]
    rng = np.random.Generator(np.random.PCG64(2212))
    n = 32 * 64 * 32
    rnd = rng.integers(0, 256, n, dtype=np.uint8)
    rnd = np.where((rnd & 0x7F) == 0x7F, rnd & 0xF0, rnd).astype(np.uint8)          # no NaN encodings
    mid = ((rng.integers(0, 2, n, dtype=np.uint8) << 7) | ((4 + rng.integers(0, 6, n, dtype=np.uint8)) << 3)
           | rng.integers(0, 8, n, dtype=np.uint8)).astype(np.uint8)                 # magnitudes 2^-3 .. 2^2
    fp8 = [("zeros", np.zeros(n, dtype=np.uint8)), ("ones", np.full(n, 0x38, dtype=np.uint8)),
           ("random e4m3, exponents 4..9", mid), ("random bytes", rnd)]
    return bf16, fp8


def mfma_loop_tflops(Bd, torch, bits, fp8, workgroups, iters):
    """Best of three launches of the library's MFMA-only loop (no memory access inside) on these operand bits."""
    frags = torch.from_numpy(bits.copy()).cuda() if fp8 else \
        torch.from_numpy(bits.view(np.int16).copy()).cuda().view(torch.bfloat16)
    out = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda")
    best = None
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        st = (Bd.rnnt_debug_mfma_loop_fp8 if fp8 else Bd.rnnt_debug_mfma_loop)(frags, out, workgroups, iters)
        e1.record()
        assert st == 0, st
        e1.synchronize()
        ms = e0.elapsed_time(e1)
        best = ms if best is None else min(best, ms)
    k = 64 if fp8 else 16
    return 2.0 * 32 * 32 * k * 16 * iters * 4 * workgroups / (best * 1e-3) / 1e12, best


def mfma_table(Bd, torch):
    """What the matrix units sustain on chosen operand values, next to the published peaks (the text kept as
    profiles/mfma_rate_by_operand_values.txt)."""
    bf16, fp8 = mfma_operand_patterns()
    for title, pats, is8, iters, peak in (("v_mfma_f32_32x32x16_bf16", bf16, False, 20000, 2500.0),
                                         ("v_mfma_f32_32x32x64_f8f6f4 (e4m3)", fp8, True, 10000, 5000.0)):
        print(f"# MFMA-only loop, {title}, {iters} iterations of 16 MFMAs per wave, 256 compute units")
        print(f"# operand values, waves per SIMD, ms per launch, TFLOP/s, fraction of the published {peak / 1e3:.1f} PFLOP/s")
        for name, bits in pats:
            for wgs in (256, 512):
                tf, ms = mfma_loop_tflops(Bd, torch, bits, is8, wgs, iters)
                print(f"{name}, {wgs // 256}, {ms:.2f}, {tf:.0f}, {tf / peak:.3f}", flush=True)


def stream_table(Bd, torch):
    """What the compute units get when all of them read one shared array the way the score kernels stream their
    W_out fragments (the text kept as profiles/shared_array_read_rate.txt)."""
    print("# every workgroup (256 threads) reads the same array, 16 bytes per lane, eight loads in flight per wave; 256 compute units")
    print("# array MiB, workgroups per compute unit, ms per launch, TB/s into the compute units, bytes per clock and "
          "compute unit at 2.4 GHz")
    for mib in (1, 2, 16, 128, 1024):
        src = torch.randint(0, 2 ** 31 - 1, (mib << 18,), dtype=torch.int32, device="cuda")
        for wpc in (1, 2, 4, 8):
            wgs = 256 * wpc
            iters = max(1, (128 if mib <= 16 else 8) * 16 // mib // wpc * 2)
            out = torch.empty(wgs * 1024, dtype=torch.int32, device="cuda")
            best = None
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                st = Bd.rnnt_debug_stream_read(src, out, wgs, iters)
                e1.record()
                assert st == 0, st
                e1.synchronize()
                ms = e0.elapsed_time(e1)
                best = ms if best is None else min(best, ms)
            tb = float(mib << 20) * iters * wgs / (best * 1e-3) / 1e12
            print(f"{mib}, {wpc}, {best:.2f}, {tb:.2f}, {tb * 1e12 / 256 / 2.4e9:.1f}", flush=True)
        del src


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C4")
    ap.add_argument("--budget-mib", type=int, default=0, help="workspace budget (0 = library default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--batch", type=int, default=0, help="use only the first N samples (profiling aid)")
    ap.add_argument("--bf16-grads", action="store_true",
                    help="input_grads_bf16 = 1 in the descriptor: d_enc and d_pred are bfloat16 arrays")
    ap.add_argument("--keep-scores", action="store_true",
                    help="keep_scores = 1 in the descriptor: the backward pass reads the scores the forward pass kept")
    ap.add_argument("--projections", type=int, default=0, metavar="D",
                    help="time the entry point with the joint network's input projections inside "
                         "(Eq. 4 complete), encoder / prediction width D (0 = the north-star entry point)")
    ap.add_argument("--skip-below", type=int, default=0, metavar="K",
                    help="skip_below_log2 = K in the descriptor: lattice tiles whose posteriors all lie below 2^-K stay "
                         "out of the backward pass.  0 = the library's default and the headline (only tiles whose score "
                         "gradients are exactly zero as bf16 operands are left out), -1 = every tile is multiplied")
    ap.add_argument("--no-skip-variant", action="store_true",
                    help="leave out the two further measurements (the same steps with skip_below_log2 = -1 and 30) that "
                         "the default bf16 line carries; for profiler runs that should hold the default path only")
    ap.add_argument("--planned", action="store_true",
                    help="call through a plan handle (rnnt_plan_create once, rnnt_joint_loss_fwd_bwd_planned per step)")
    ap.add_argument("--lattice-stream", action="store_true",
                    help="with --planned: the lattice sweeps run on a second stream beside the previous group's backward pass")
    ap.add_argument("--mfma-table", action="store_true",
                    help="only print what the MFMA-only loop sustains on chosen operand values (bf16 and fp8) and exit")
    ap.add_argument("--stream-table", action="store_true",
                    help="print what the compute units get when all of them read one shared array (L2, last-level "
                         "cache, HBM) and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch the 256 MiB plain copy kernel 5 times (HBM counter calibration under rocprofv3)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one MI355X per box); --gpus must be 1. "
              "Sharding over GPUs is a design note only (samples over GPUs, one all-reduce of dW_out and db_out); it is not implemented.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2211_16270_amd import binding as Bd
    from paper_2211_16270_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.mfma_table:
        mfma_table(Bd, torch)
        return
    if args.stream_table:
        stream_table(Bd, torch)
        return
    if args.config in ("P16", "P16F32"):
        # shaped like the paper's benchmark (Section 5.1): 16 samples of up to 500 x 100, joint size 1024,
        # 4096 word pieces; lengths drawn uniformly down to the paper's largest padding (9.3 % / 45.8 %)
        # P16F32: the same in fp32 (the paper's own precision), on the fp32 MFMA GEMM form of the path
        wl = synth.custom_workload(args.config, B=16, T_max=500, U_max=100, H=1024, V=4096,
                                   dtype="bf16" if args.config == "P16" else "f32", index=5,
                                   t_rule="uniform", t_lo=454, u_rule="uniform", u_lo=54)
    else:
        wl = synth.WORKLOADS[args.config]
    steps = args.steps if args.steps is not None else {"C1": 100, "C2": 100, "C3": 20, "C4": 10, "C5": 10}.get(wl.name, 10)
    t0 = time.time()
    if args.batch:
        import dataclasses
        batch = synth.make_batch(wl, sample_ids=list(range(args.batch)), pad="zero")
        wl = dataclasses.replace(wl, B=args.batch)
        batch.wl = wl
    else:
        batch = synth.make_batch(wl, pad="zero")
    gen_s = time.time() - t0
    dev = Bd.to_device(batch)
    dt = Bd.RNNT_BF16 if wl.dtype == "bf16" else Bd.RNNT_F32
    desc = Bd.make_desc(wl.B, wl.T_max, wl.U_max, wl.H, wl.V, wl.blank, dt, keep_scores=int(args.keep_scores),
                        input_grads_bf16=int(args.bf16_grads), skip_below_log2=args.skip_below)
    plan = side = None
    if args.planned or args.lattice_stream:
        plan = Bd.PlanHandle(desc, dev["T_len"], dev["U_len"], args.budget_mib << 20, overlap_lattice=args.lattice_stream)
        nbytes, info = plan.workspace_bytes, plan.describe()
        side = torch.cuda.Stream() if args.lattice_stream else None
    else:
        nbytes = Bd.rnnt_joint_loss_workspace_bytes(desc, dev["T_len"], dev["U_len"], args.budget_mib << 20)
        st, info, _ = Bd.rnnt_joint_loss_plan(desc, dev["T_len"], dev["U_len"], nbytes)
        assert st == 0, st
    torch.cuda.reset_peak_memory_stats()
    ws = Bd.Workspace(nbytes)
    loss = torch.empty(wl.B, dtype=torch.float32, device="cuda")
    gdt = torch.bfloat16 if args.bf16_grads else torch.float32
    d_enc = torch.empty(wl.B, wl.T_max, wl.H, dtype=gdt, device="cuda")
    d_pred = torch.empty(wl.B, wl.U_max + 1, wl.H, dtype=gdt, device="cuda")
    dW = torch.empty(wl.H, wl.V, dtype=torch.float32, device="cuda")
    db = torch.empty(wl.V, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    if args.projections:
        D = args.projections
        proj = synth.make_proj_inputs(batch, D, D, pad="zero")
        devp = Bd.proj_to_device(proj, wl.dtype)
        nbytes = Bd.rnnt_joint_proj_workspace_bytes(desc, D, D, dev["T_len"], dev["U_len"], args.budget_mib << 20)
        del ws, d_enc, d_pred, dev["enc"], dev["pred"]
        torch.cuda.reset_peak_memory_stats()
        ws = Bd.Workspace(nbytes)
        f32 = dict(dtype=torch.float32, device="cuda")
        d_hA, d_hL = torch.empty(wl.B, wl.T_max, D, **f32), torch.empty(wl.B, wl.U_max + 1, D, **f32)
        dWA, dbZ, dWL = torch.empty(D, wl.H, **f32), torch.empty(wl.H, **f32), torch.empty(D, wl.H, **f32)

    def step():
        if args.projections:
            s = Bd.rnnt_joint_proj_loss_fwd_bwd(desc, D, D, devp["hA"], devp["hL"], devp["W_A"], devp["b_Z"],
                                                devp["W_L"], dev["W_out"], dev["b_out"], dev["labels"], dev["T_len"],
                                                dev["U_len"], loss, d_hA, d_hL, dWA, dbZ, dWL, dW, db, ws.buf, stream)
            if s != 0:
                raise Bd.RnntError(s, "rnnt_joint_proj_loss_fwd_bwd")
            return
        if plan is not None:
            s = Bd.rnnt_joint_loss_fwd_bwd_planned(plan, dev["enc"], dev["pred"], dev["W_out"], dev["b_out"], dev["labels"],
                                                   None, loss, d_enc, d_pred, dW, db, ws.buf, stream, side)
        else:
            s = Bd.rnnt_joint_loss_fwd_bwd(desc, dev["enc"], dev["pred"], dev["W_out"], dev["b_out"], dev["labels"],
                                           dev["T_len"], dev["U_len"], loss, d_enc, d_pred, dW, db, ws.buf, stream)
        if s != 0:
            raise Bd.RnntError(s, "rnnt_joint_loss_fwd_bwd")

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]   # one event record between steps
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / steps * 1e3
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    value = wl.B / (elapsed / steps)
    assert bool(torch.isfinite(loss).all()), "non-finite loss"
    peak_bytes = torch.cuda.max_memory_allocated()

    # share of the lattice tiles the backward pass worked on (tiles whose bf16 score gradients are all zero are left out)
    share_main = 1.0
    if plan is None and not (args.projections and args.budget_mib):
        inner = ws.buf
        if args.projections:
            # the joint path's own workspace lies behind the projected encodings and their gradients
            inner = ws.buf[nbytes - Bd.rnnt_joint_loss_workspace_bytes(desc, dev["T_len"], dev["U_len"], args.budget_mib << 20):]
        st, act, tot = Bd.rnnt_debug_read_active_tiles(desc, dev["T_len"], dev["U_len"], inner)
        assert st == 0, st
        share_main = act / tot

    # second pass: the same K steps with every launch bracketed by HIP events on the same stream
    Bd.rnnt_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed_prof = time.perf_counter() - t0
    prof = Bd.rnnt_profile_read()
    Bd.rnnt_profile_enable(False)

    if args.calibrate_copy:
        src = torch.ones(COPY_BYTES // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            assert Bd.rnnt_debug_copy_f32(src, dst) == 0
        torch.cuda.synchronize()
        del src, dst

    # the same steps with other values of skip_below_log2 (not the headline): -1 = every lattice tile goes through the
    # backward pass, also those whose score gradients are exactly zero as bf16 operands; 30 = only tiles with a node of
    # posterior >= 2^-30
    variants = None
    if (wl.dtype == "bf16" and wl.H <= 640 and not (args.skip_below or args.keep_scores or args.projections
                                                     or args.bf16_grads or args.no_skip_variant or args.batch
                                                     or plan is not None)):
        loss_default = loss.clone()
        variants = {}
        for key, k_skip, what in (("every_tile", -1, "skip_below_log2 = -1: every lattice tile goes through the backward "
                                   "pass, also those whose score gradients are all zero as bf16 operands"),
                                  ("negligible_tiles_skipped", 30, "skip_below_log2 = 30: backward pass only over lattice "
                                   "tiles with a node of posterior >= 2^-30; same loss, gradients within rounding of the "
                                   "full computation (tests)")):
            desc2 = Bd.make_desc(wl.B, wl.T_max, wl.U_max, wl.H, wl.V, wl.blank, dt, skip_below_log2=k_skip)
            n2 = Bd.rnnt_joint_loss_workspace_bytes(desc2, dev["T_len"], dev["U_len"], args.budget_mib << 20)
            del ws
            ws = Bd.Workspace(n2)

            def step2():
                s = Bd.rnnt_joint_loss_fwd_bwd(desc2, dev["enc"], dev["pred"], dev["W_out"], dev["b_out"], dev["labels"],
                                               dev["T_len"], dev["U_len"], loss, d_enc, d_pred, dW, db, ws.buf, stream)
                if s != 0:
                    raise Bd.RnntError(s, "rnnt_joint_loss_fwd_bwd")
            k2 = max(2, min(steps, 6))
            step2()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(k2):
                step2()
            torch.cuda.synchronize()
            dt2 = (time.perf_counter() - t0) / k2
            st, act, tot = Bd.rnnt_debug_read_active_tiles(desc2, dev["T_len"], dev["U_len"], ws.buf)
            assert st == 0 and bool(torch.equal(loss, loss_default))
            variants[key] = {"skip_below_log2": k_skip, "value": wl.B / dt2, "unit": "samples/s",
                             "ms_per_step": dt2 * 1e3, "steps": k2, "backward_tile_share": act / tot, "what": what}

    R = int(info["rows_total"])
    HV = wl.H * wl.V
    # share of the lattice tiles the backward pass worked on
    bwd_share = share_main
    # flops per step of each MFMA kernel, 2*H*V per lattice node and contraction.  Algorithmic: the three
    # contractions the method asks for (scores, dW_out, dz), each counted once, where it is first computed;
    # executed: what the kernel multiplies, i.e. also the scores a backward kernel computes a second time.
    alg_flops_per_step = {"joint_scores_fwd": 2.0 * R * HV, "joint_scores_bwd": 0.0,
                          "joint_scores_fwd_keep": 2.0 * R * HV,
                          "gemm_dz": 2.0 * R * HV, "gemm_dw_db": 2.0 * R * HV, "joint_bwd_fused": 2.0 * R * HV,
                          "fwd_f32": 2.0 * R * HV, "bwd_f32": 4.0 * R * HV}
    exec_flops_per_step = dict(alg_flops_per_step, joint_scores_bwd=2.0 * R * HV, bwd_f32=6.0 * R * HV,
                               joint_bwd_fused=(2.0 if args.keep_scores else 4.0) * R * HV)
    if bwd_share < 1.0:
        # tiles of negligible posterior are left out: both counts cover only the rows the kernels worked on
        for name in ("joint_bwd_fused", "gemm_dw_db"):
            alg_flops_per_step[name] *= bwd_share
            exec_flops_per_step[name] *= bwd_share
    kernels = {}
    for name, (cnt, ms) in prof.items():
        if cnt:
            kernels[name] = {"launches_per_step": cnt / steps, "ms_per_step": ms / steps,
                             "avg_launch_us": ms / cnt * 1e3}
    gpu_ms = sum(k["ms_per_step"] for k in kernels.values())
    # the kernel that takes the most time among those that carry algorithmic work (a kernel that only multiplies the
    # scores a second time carries none)
    cands = [n for n in kernels if alg_flops_per_step.get(n, 0.0) > 0.0] or [n for n in kernels if n in alg_flops_per_step]
    dom = max(cands, key=lambda n: kernels[n]["ms_per_step"])
    launches = kernels[dom]["launches_per_step"]
    avg_s = kernels[dom]["avg_launch_us"] * 1e-6
    flops_per_launch = alg_flops_per_step[dom] / launches
    exec_per_launch = exec_flops_per_step[dom] / launches
    peak = PEAK_BF16_FLOPS if wl.dtype == "bf16" else PEAK_F32_FLOPS
    achieved = flops_per_launch / avg_s
    for name, k in kernels.items():
        if name in alg_flops_per_step:
            k["frac_alg"] = alg_flops_per_step[name] / (k["ms_per_step"] * 1e-3) / peak
            k["frac_exec"] = exec_flops_per_step[name] / (k["ms_per_step"] * 1e-3) / peak
    # HBM bytes per launch from the committed rocprofv3 counter summary of this workload, if any
    tname = f"hbm_traffic_{wl.name}" + ("_keep_scores" if args.keep_scores else "") + ".txt"
    traffic = read_traffic(os.path.join(ROOT, "profiles", tname)) if not args.batch else {}
    # fp32: GEMMs on the fp32 MFMA instruction where the plan has chunk buffers (H, V multiples of 128; `kernel` is
    # then the group of launches of one chunk: three GEMMs and the row kernels between them), else plain FMA
    roofline = {"bound": "mfma" if (wl.dtype == "bf16" or info["chunk_rows"] > 0) else "alu", "kernel": dom,
                "achieved": achieved / 1e12, "peak": peak / 1e12, "unit": "TFLOP/s", "frac": achieved / peak,
                "traffic": traffic.get(dom), "traffic_source": ("profiles/" + tname) if traffic.get(dom) else None,
                "alg_flops_per_launch": flops_per_launch, "exec_flops_per_launch": exec_per_launch,
                "frac_exec": exec_per_launch / avg_s / peak, "avg_launch_us": kernels[dom]["avg_launch_us"]}
    # what the matrix units sustain on operands like this path's (random bf16 values): an MFMA-only loop, no
    # memory access; the chip lowers its clock under its power limit, so this is below the published peak
    pats, _ = mfma_operand_patterns()
    measured_peak = {name: mfma_loop_tflops(Bd, torch, bits, False, 512, 4000)[0]
                     for name, bits in pats if name in ("zeros", "random bf16")} if wl.dtype == "bf16" else None
    step_s = elapsed / steps
    util_alg = (2.0 + 4.0 * bwd_share) * R * HV / step_s / peak
    util_exec = (2.0 + (4.0 if args.keep_scores else 6.0) * bwd_share) * R * HV / step_s / peak
    lat = kernels.get("lattice")
    # lattice pass: bytes per launch from the committed FETCH_SIZE / WRITE_SIZE summary where there is one,
    # next to the figure from the 24 bytes per node the sweep has to move (emissions read twice, alpha, beta written)
    lattice_alg_gbs = (24.0 * R / (lat["ms_per_step"] * 1e-3) / 1e9) if lat else None
    lattice_gbs = (traffic["lattice"] * lat["launches_per_step"] / (lat["ms_per_step"] * 1e-3) / 1e9) \
        if lat and traffic.get("lattice") else None

    out = {
        "metric": "samples/s fused joint+RNN-T loss+grads" + (" incl. input projections" if args.projections else ""),
        "value": value, "unit": "samples/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={wl.B} T_max={wl.T_max} U_max={wl.U_max} H={wl.H} V={wl.V} "
                               f"{wl.dtype}, ragged lengths, {R} lattice nodes ({100.0 * R / info['rows_padded']:.1f}% of padded)",
                   "entry_point": "rnnt_joint_proj_loss_fwd_bwd, H_A = H_L = %d" % args.projections
                   if args.projections else ("rnnt_joint_loss_fwd_bwd_planned" + (", lattice sweeps on a second stream"
                                                                                   if side is not None else "")
                                             if plan is not None else "rnnt_joint_loss_fwd_bwd"),
                   "keep_scores": int(args.keep_scores), "input_grads_bf16": int(args.bf16_grads),
                   "skip_below_log2": args.skip_below, "backward_tile_share": bwd_share,
                   "groups": info["n_groups"], "chunks": info["n_chunks"],
                   "workspace_bytes": int(nbytes)},
        "mfma_util_alg": util_alg, "mfma_util_exec": util_exec,
        # 6 R H V over the step time: what an implementation that multiplies every lattice node would have to sustain
        # for this step time (equal to mfma_util_alg when backward_tile_share is 1)
        "mfma_util_dense_equivalent": 6.0 * R * HV / step_s / peak,
        "peak_hbm_gb": peak_bytes / 1e9,
        "lattice_gb_per_s": lattice_gbs, "lattice_gb_per_s_from_24B_per_node": lattice_alg_gbs,
        "ms_per_step_with_events": elapsed_prof / steps * 1e3,
        "gpu_kernel_ms_per_step": gpu_ms,
        "roofline": roofline,
        "other_tile_selections": variants,
        "measured_mfma_peak": None if measured_peak is None else
        {"unit": "TFLOP/s", "what": "MFMA-only loop, 32x32x16 bf16, two waves per SIMD, no memory access",
         "zeros": measured_peak["zeros"], "random_bf16": measured_peak["random bf16"]},
        "kernels": kernels,
    }

    if not args.no_cpu_baseline:
        from oracle import rnnt_oracle as O
        n = min(CPU_SAMPLE.get(wl.name, 1), wl.B)
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        f64 = lambda x: np.asarray(x[:n], dtype=np.float64)
        t0 = time.perf_counter()
        if args.projections:
            ref = O.rnnt_joint_proj_loss(f64(proj.hA), f64(proj.hL), proj.W_A.astype(np.float64),
                                         proj.b_Z.astype(np.float64), proj.W_L.astype(np.float64),
                                         batch.W_out.astype(np.float64), batch.b_out.astype(np.float64),
                                         batch.labels[:n], batch.T_len[:n], batch.U_len[:n], wl.blank)
        else:
            ref = O.rnnt_joint_loss(f64(batch.enc), f64(batch.pred), batch.W_out.astype(np.float64),
                                    batch.b_out.astype(np.float64), batch.labels[:n], batch.T_len[:n],
                                    batch.U_len[:n], wl.blank)
        cpu_s = time.perf_counter() - t0
        rel = float(np.max(np.abs(loss[:n].cpu().numpy() - ref["loss"]) / np.abs(ref["loss"])))
        out["cpu_baseline"] = {"value": n / cpu_s, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"first {n} of {wl.B} samples of {wl.name}, float64 numpy, {cpu_s:.1f} s",
                               "gpu_loss_rel_err_on_sample": rel}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
