"""GPU parity on the named workloads at their real shapes: sub-batches the float64 checker finishes in
seconds, every one of the five outputs compared element by element (loss, d_enc, d_pred, dW_out, db_out),
in the default plan that bench.py times and in plans a small workspace cuts into several groups of samples
and several backward chunks (run with -m gpu on an MI355X)."""
import numpy as np
import pytest

from paper_2211_16270_amd import binding as Bd
from paper_2211_16270_amd import synth
from tests.gpu_util import assert_padding_zero, assert_parity, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _rows(wl):
    T, U, _ = synth.draw_lengths_labels(wl)
    return T.astype(np.int64) * (U.astype(np.int64) + 1), T, U


def _ids_spanning(wl, n, max_rows=None):
    """n sample ids of a workload: the one with the fewest lattice nodes, the one with the most (at most
    max_rows, if given) and the first others."""
    rows, _, _ = _rows(wl)
    ok = np.arange(wl.B) if max_rows is None else np.nonzero(rows <= max_rows)[0]
    lo = int(ok[np.argmin(rows[ok])])
    hi = int(ok[np.argmax(rows[ok])])
    ids = [lo, hi]
    for b in ok:
        if len(ids) >= n:
            break
        if int(b) not in ids:
            ids.append(int(b))
    return ids


def _budget_with_several_groups_and_chunks(batch, desc_opts, frac=0.5):
    """A workspace size between the smallest plan and the default one that cuts the sub-batch into at
    least two groups of samples and more backward chunks than groups."""
    wl = batch.wl
    desc = Bd.make_desc(batch.B, wl.T_max, wl.U_max, wl.H, wl.V, wl.blank, Bd.RNNT_BF16, 0, **desc_opts)
    nmin = Bd.rnnt_joint_loss_workspace_bytes(desc, batch.T_len, batch.U_len, 1)
    ndef = Bd.rnnt_joint_loss_workspace_bytes(desc, batch.T_len, batch.U_len, 0)
    for f in (frac, 0.25, 0.1, 0.03, 0.0):
        budget = int(nmin + f * (ndef - nmin))
        st, info, _ = Bd.rnnt_joint_loss_plan(desc, batch.T_len, batch.U_len, budget)
        assert st == 0
        if info["n_groups"] >= 2 and info["n_chunks"] > info["n_groups"]:
            return budget, info
    raise AssertionError("no budget cuts this sub-batch into several groups and chunks")


def test_c2_full_batch_all_outputs():
    # the whole B = 32 batch (the checker takes a few seconds): default plan = one group, one chunk
    batch = synth.make_batch("C2")
    ref = run_oracle(batch)
    got = run_gpu(batch)
    e, errs = assert_parity(got, ref, "bf16", "C2 full")
    _say("C2 full errs", e, errs)
    assert_padding_zero(got, batch)
    kept = run_gpu(batch, keep_scores=1)
    e, errs = assert_parity(kept, ref, "bf16", "C2 full, kept scores")
    _say("C2 full kept errs", e, errs)


def test_c4_subbatch_all_outputs_default_and_small_workspace():
    # memory-headline workload (B = 1024, T <= 1000, U <= 200, H = 512, V = 1024): 12 of its samples, among them
    # the one with the fewest and the one with the most lattice nodes (multi-wave lattice kernel, U + 1 > 64)
    wl = synth.WORKLOADS["C4"]
    ids = _ids_spanning(wl, 12)
    batch = synth.make_batch(wl, sample_ids=ids)
    _say("C4 ids", ids, batch.T_len.tolist(), batch.U_len.tolist())
    ref = run_oracle(batch)
    _say("C4 checker done")
    got = run_gpu(batch)
    e, errs = assert_parity(got, ref, "bf16", "C4 sub-batch")
    _say("C4 sub-batch errs", e, errs)
    assert_padding_zero(got, batch)
    budget, info = _budget_with_several_groups_and_chunks(batch, {})
    _say("C4 small plan", info)
    small = run_gpu(batch, budget_bytes=budget)
    e, errs = assert_parity(small, ref, "bf16", "C4 sub-batch, several groups and chunks")
    _say("C4 small-workspace errs", e, errs)
    assert_padding_zero(small, batch)


def test_c3_subbatch_all_outputs_default_small_workspace_and_kept_scores():
    # H = 640 (the widest joint the fused backward kernel takes), V = 4096: 8 samples incl. fewest / most nodes
    wl = synth.WORKLOADS["C3"]
    ids = _ids_spanning(wl, 8)
    batch = synth.make_batch(wl, sample_ids=ids)
    _say("C3 ids", ids, batch.T_len.tolist(), batch.U_len.tolist())
    ref = run_oracle(batch)
    _say("C3 checker done")
    got = run_gpu(batch)
    e, errs = assert_parity(got, ref, "bf16", "C3 sub-batch")
    _say("C3 sub-batch errs", e, errs)
    assert_padding_zero(got, batch)
    budget, info = _budget_with_several_groups_and_chunks(batch, {})
    _say("C3 small plan", info)
    small = run_gpu(batch, budget_bytes=budget)
    e, errs = assert_parity(small, ref, "bf16", "C3 sub-batch, several groups and chunks")
    _say("C3 small-workspace errs", e, errs)
    kept = run_gpu(batch, keep_scores=1)
    e, errs = assert_parity(kept, ref, "bf16", "C3 sub-batch, kept scores")
    _say("C3 kept errs", e, errs)
    assert_padding_zero(kept, batch)


def test_c5_subbatch_all_outputs_short_and_long_samples_together():
    # V = 8192, Zipf labels, log-uniform lengths: the shortest sample (50 x 16: single-wave lattice kernel, 16 x 4
    # tiles) next to long ones (U + 1 > 64: multi-wave lattice kernel, 8 x 8 tiles) in one launch.  The checker
    # forms a sample's [T, U+1, V] scores in float64 several times over, so the long ones are capped at 60 000
    # lattice nodes (4 GB per such array); the longest sample of the workload (800 x 241, 12.6 GB per array) is
    # left to the invariants of the full-size run below.
    wl = synth.WORKLOADS["C5"]
    ids = _ids_spanning(wl, 8, max_rows=60_000)
    batch = synth.make_batch(wl, sample_ids=ids)
    _say("C5 ids", ids, batch.T_len.tolist(), batch.U_len.tolist())
    assert batch.U_len.min() + 1 <= 64 < batch.U_len.max() + 1
    ref = run_oracle(batch)
    _say("C5 checker done")
    got = run_gpu(batch)
    e, errs = assert_parity(got, ref, "bf16", "C5 sub-batch")
    _say("C5 sub-batch errs", e, errs)
    assert_padding_zero(got, batch)
    kept = run_gpu(batch, keep_scores=1)
    e, errs = assert_parity(kept, ref, "bf16", "C5 sub-batch, kept scores")
    _say("C5 kept errs", e, errs)
    budget, info = _budget_with_several_groups_and_chunks(batch, {})
    _say("C5 small plan", info)
    small = run_gpu(batch, budget_bytes=budget)
    e, errs = assert_parity(small, ref, "bf16", "C5 sub-batch, several groups and chunks")
    _say("C5 small-workspace errs", e, errs)


def test_c5_longest_and_shortest_sample_packing_invariance():
    # the longest (800 x 241) and the shortest sample of C5 in one call against each of them alone: per-sample
    # outputs do not depend on what else shares the launch; the parameter gradients add up
    wl = synth.WORKLOADS["C5"]
    rows, _, _ = _rows(wl)
    lo, hi = int(np.argmin(rows)), int(np.argmax(rows))
    both = run_gpu(synth.make_batch(wl, sample_ids=[lo, hi]))
    a = run_gpu(synth.make_batch(wl, sample_ids=[lo]))
    b = run_gpu(synth.make_batch(wl, sample_ids=[hi]))
    assert np.all(np.isfinite(both["loss"]))
    np.testing.assert_allclose(both["loss"], np.concatenate([a["loss"], b["loss"]]), rtol=1e-6)
    for k in ("d_enc", "d_pred"):
        for i, single in enumerate((a, b)):
            d = np.abs(both[k][i] - single[k][0]).max() / np.abs(single[k][0]).max()
            assert d < 1e-3, (k, i, d)
    for k in ("dW_out", "db_out"):
        s = a[k].astype(np.float64) + b[k].astype(np.float64)
        d = np.abs(both[k] - s).max() / np.abs(s).max()
        assert d < 2e-3, (k, d)
    assert abs(float(both["db_out"].astype(np.float64).sum())) < 1e-2 * float(np.abs(both["db_out"]).sum())


@pytest.mark.parametrize("mode,dtype", [("packed", "bf16"), ("padded", "bf16"), ("one_by_one", "bf16"), ("kept", "bf16"),
                                        ("packed", "f32"), ("one_by_one", "f32")])
def test_paper_shaped_sweep_modes_against_the_checker(mode, dtype):
    # one small point of the paper-shaped sweeps (Section 5.1's padding scheme: lengths fall linearly over the
    # batch) in every way the sweep runs a batch; the checker gets the very tensors the sweep made on the GPU
    # and the lengths that way of running used (all at the maximum for "padded")
    from oracle import rnnt_oracle as O
    from paper_2211_16270_amd import sweep
    from tests.gpu_util import GRADS, TOL, rel_grad_err, rel_loss_err
    B, T, U, H, V = 4, 50, 10, 256, 512
    r = sweep.run_case(B, T, U, H, V, mode, steps=2, warmup=1, dtype=dtype, return_tensors=True)
    t = r["tensors"]
    if mode != "padded":
        Tp, Up = sweep.paper_lengths(B, T, U)
        assert np.array_equal(t["T_len"], Tp) and np.array_equal(t["U_len"], Up) and Tp.min() < T and Up.min() < U
    f64 = lambda x: x.float().cpu().numpy().astype(np.float64)
    ref = O.rnnt_joint_loss(f64(t["enc"]), f64(t["pred"]), f64(t["W_out"]), f64(t["b_out"]),
                            t["labels"].cpu().numpy(), t["T_len"], t["U_len"], 0)
    tol = TOL[dtype]
    e = rel_loss_err(f64(t["loss"]), ref["loss"])
    assert e <= tol["loss"], (mode, dtype, e)
    for k in GRADS:
        eg = rel_grad_err(f64(t[k]), ref[k])
        _say("sweep", mode, dtype, k, eg)
        assert eg <= tol["grad"], (mode, dtype, k, eg)
    assert r["rows"] == int(np.sum(t["T_len"].astype(np.int64) * (t["U_len"] + 1)))


def _run_planned(batch, plan, lattice_stream=None, sample_weight=None, workspace=None):
    import torch
    wl = batch.wl
    dev = Bd.to_device(batch)
    f32 = dict(dtype=torch.float32, device="cuda:0")
    out = dict(loss=torch.empty(batch.B, **f32), d_enc=torch.empty(batch.B, wl.T_max, wl.H, **f32),
               d_pred=torch.empty(batch.B, wl.U_max + 1, wl.H, **f32), dW_out=torch.empty(wl.H, wl.V, **f32),
               db_out=torch.empty(wl.V, **f32))
    ws = workspace or Bd.Workspace(plan.workspace_bytes)
    st = Bd.rnnt_joint_loss_fwd_bwd_planned(plan, dev["enc"], dev["pred"], dev["W_out"], dev["b_out"], dev["labels"],
                                            sample_weight, out["loss"], out["d_enc"], out["d_pred"], out["dW_out"],
                                            out["db_out"], ws.buf, lattice_stream=lattice_stream)
    assert st == 0, Bd.STATUS_NAMES[st]
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}, ws


def test_plan_handle_one_stream_equals_the_plain_call():
    batch = synth.make_batch("C2")
    desc = Bd.make_desc(batch.B, 250, 50, 512, 1024, 0, Bd.RNNT_BF16)
    plan = Bd.PlanHandle(desc, batch.T_len, batch.U_len)
    plain = run_gpu(batch)
    got, ws = _run_planned(batch, plan)
    np.testing.assert_array_equal(got["loss"], plain["loss"])
    np.testing.assert_array_equal(got["dW_out"], plain["dW_out"])          # same schedule, fixed summation order
    for k in ("d_enc", "d_pred", "db_out"):
        assert np.abs(got[k] - plain[k]).max() <= 1e-5 * np.abs(plain[k]).max(), k
    again, _ = _run_planned(batch, plan, workspace=ws)                      # the handle and workspace are reusable
    np.testing.assert_array_equal(again["loss"], got["loss"])
    np.testing.assert_array_equal(again["dW_out"], got["dW_out"])
    plan.close()


@pytest.mark.parametrize("name,n,frac", [("C2", 32, 0.005), ("C4", 12, 0.05)])
def test_lattice_sweeps_on_a_second_stream_against_the_checker(name, n, frac):
    # several groups of samples; every group's lattice sweep runs on a second stream beside the previous group's
    # backward pass (two lattice buffers).  Checked against the float64 checker, against the one-stream call with
    # the same handle, three calls in a row, and with per-sample weights.
    import torch
    wl = synth.WORKLOADS[name]
    ids = list(range(n)) if name == "C2" else _ids_spanning(wl, n)
    batch = synth.make_batch(wl, sample_ids=ids)
    desc = Bd.make_desc(batch.B, wl.T_max, wl.U_max, wl.H, wl.V, 0, Bd.RNNT_BF16)
    nmin = Bd.rnnt_joint_loss_workspace_bytes(desc, batch.T_len, batch.U_len, 1)
    ndef = Bd.rnnt_joint_loss_workspace_bytes(desc, batch.T_len, batch.U_len, 0)
    plan = Bd.PlanHandle(desc, batch.T_len, batch.U_len, budget_bytes=int(nmin + frac * (ndef - nmin)), overlap_lattice=True)
    info = plan.describe()
    _say("two-stream plan", name, info)
    assert info["n_groups"] >= 3
    ref = run_oracle(batch)
    side = torch.cuda.Stream()
    one, ws = _run_planned(batch, plan)
    assert_parity(one, ref, "bf16", f"{name} planned, one stream")
    for rep in range(3):
        two, _ = _run_planned(batch, plan, lattice_stream=side, workspace=ws)
        e, errs = assert_parity(two, ref, "bf16", f"{name} planned, lattice on a second stream, call {rep}")
        np.testing.assert_array_equal(two["loss"], one["loss"])
        np.testing.assert_array_equal(two["dW_out"], one["dW_out"])
    _say("two-stream errs", e, errs)
    assert_padding_zero(two, batch)
    w = np.linspace(0.0, 2.0, batch.B).astype(np.float32)
    refw = run_oracle(batch, sample_weight=w.astype(np.float64))
    tw, _ = _run_planned(batch, plan, lattice_stream=side, sample_weight=w, workspace=ws)
    assert_parity(tw, refw, "bf16", f"{name} planned, second stream, weighted")
    plan.close()


@pytest.mark.parametrize("name,n,k", [("C2", 32, 30), ("C4", 12, 30), ("C4", 12, 20), ("C3", 8, 30)])
def test_backward_pass_without_the_tiles_of_negligible_posterior(name, n, k):
    # skip_below_log2 = k: lattice tiles whose nodes all have a posterior below 2^-k stay out of the backward pass.
    # All five outputs against the checker at the usual tolerance, the loss bit-identical to the full call, the
    # gradients within 2^-k * (nodes that add to an entry) of it, and a real share of the tiles left out.
    wl = synth.WORKLOADS[name]
    ids = list(range(n)) if name == "C2" else _ids_spanning(wl, n)
    batch = synth.make_batch(wl, sample_ids=ids)
    ref = run_oracle(batch)
    full = run_gpu(batch, skip_below_log2=-1)               # every tile
    got = run_gpu(batch, skip_below_log2=k)
    e, errs = assert_parity(got, ref, "bf16", f"{name} without negligible tiles, k = {k}")
    assert_padding_zero(got, batch)
    np.testing.assert_array_equal(got["loss"], full["loss"])
    st, active, total = Bd.rnnt_debug_read_active_tiles(got["desc"], batch.T_len, batch.U_len, got["workspace"].buf)
    assert st == 0 and 0 < active <= total
    _say("negligible tiles", name, k, "active", active, "of", total, "errs", e, errs)
    for key in ("d_enc", "d_pred", "dW_out", "db_out"):
        d = np.abs(got[key].astype(np.float64) - full[key]).max() / np.abs(full[key]).max()
        assert d < 1e-4, (key, d)          # far inside the tolerance: what was left out is below 2^-20 per node
    if name != "C2":
        assert active < 0.6 * total        # long lattices: most tiles carry no posterior mass
    # a small workspace: several groups, several chunks per group, the list cut across chunks
    budget, info = _budget_with_several_groups_and_chunks(batch, {})
    small = run_gpu(batch, budget_bytes=budget, skip_below_log2=k)
    assert_parity(small, ref, "bf16", f"{name} without negligible tiles, small workspace")
    st, active2, total2 = Bd.rnnt_debug_read_active_tiles(small["desc"], batch.T_len, batch.U_len, small["workspace"].buf)
    assert st == 0 and (active2, total2) == (active, total)


def test_negligible_tile_option_edge_cases():
    # tiny lattices (every tile holds posterior mass: nothing is left out), a weight of zero (all of that sample's
    # tiles drop out), and shapes the option does not cover
    wl = synth.custom_workload("skipedge", B=4, T_max=37, U_max=19, H=128, V=256, dtype="bf16", index=170,
                               t_rule="uniform", t_lo=3, u_rule="uniform", u_lo=0)
    batch = synth.make_batch(wl)
    ref = run_oracle(batch)
    got = run_gpu(batch, skip_below_log2=30)
    assert_parity(got, ref, "bf16", "small lattices, k = 30")
    w = np.array([1.0, 0.0, 0.5, 2.0], dtype=np.float32)
    gw = run_gpu(batch, skip_below_log2=30, sample_weight=w)
    assert_parity(gw, run_oracle(batch, sample_weight=w.astype(np.float64)), "bf16", "weights, k = 30")
    assert np.all(gw["d_enc"][1] == 0.0) and np.all(gw["d_pred"][1] == 0.0)
    one = run_gpu(batch, skip_below_log2=1)            # gamma < 1/2 dropped: a coarse result, but a finite one
    assert all(np.all(np.isfinite(one[k2])) for k2 in ("loss", "d_enc", "d_pred", "dW_out", "db_out"))
    np.testing.assert_array_equal(one["loss"], got["loss"])
    for bad in (dict(dtype=Bd.RNNT_F32), dict(skip=127), dict(skip=-2)):
        d = Bd.make_desc(2, 8, 4, bad.get("H", 128), 256, 0, bad.get("dtype", Bd.RNNT_BF16),
                         keep_scores=bad.get("keep_scores", 0), skip_below_log2=bad.get("skip", 30))
        assert Bd.rnnt_joint_loss_workspace_bytes(d, [8, 8], [4, 4]) == 0, bad


@pytest.mark.parametrize("name,n", [("C4", 12), ("C3", 8), ("C5", 8), ("P1024", 4)])
def test_default_leaves_out_only_tiles_whose_score_gradients_are_zero_in_bf16(name, n):
    # skip_below_log2 = 0 (default): tiles whose posteriors all lie below 2^-135 stay out of the backward pass; as bf16
    # operands their score gradients are exactly zero, so against the pass over every tile (-1) only the order of the
    # floating-point additions differs: loss identical, gradients equal to a few units of fp32 rounding of the sums
    if name == "P1024":
        # the paper's own shape (joint size 1024, 4096 word pieces, 500 x 100): the unfused backward kernels
        wl = synth.custom_workload("P4", B=4, T_max=500, U_max=100, H=1024, V=4096, dtype="bf16", index=5,
                                   t_rule="uniform", t_lo=454, u_rule="uniform", u_lo=54)
        ids = list(range(n))
    else:
        wl = synth.WORKLOADS[name]
        ids = _ids_spanning(wl, n, max_rows=60_000 if name == "C5" else None)
    batch = synth.make_batch(wl, sample_ids=ids)
    dflt = run_gpu(batch)
    every = run_gpu(batch, skip_below_log2=-1)
    np.testing.assert_array_equal(dflt["loss"], every["loss"])
    for key in ("d_enc", "d_pred", "dW_out", "db_out"):
        d = np.abs(dflt[key].astype(np.float64) - every[key]).max() / np.abs(every[key]).max()
        _say("default vs every tile", name, key, d)
        assert d < 2e-6, (key, d)
    st, active, total = Bd.rnnt_debug_read_active_tiles(dflt["desc"], batch.T_len, batch.U_len, dflt["workspace"].buf)
    st2, a2, t2 = Bd.rnnt_debug_read_active_tiles(every["desc"], batch.T_len, batch.U_len, every["workspace"].buf)
    _say("default keeps", active, "of", total, "tiles")
    assert st == 0 and st2 == 0 and a2 == t2 == total and 0 < active < total


@pytest.mark.parametrize("name,n", [("C4", 12), ("C3", 8), ("P1024", 4)])
def test_kept_scores_with_the_tile_selection(name, n):
    # keep_scores = 1: the forward pass has written every tile's scores and joint rows into the chunk buffers before
    # the list exists, so the backward kernels and the dW_out GEMM pick the listed tiles' rows where they lie (fused
    # kernel for H <= 640, conversion pass + dz GEMM above).  Default against the checker and against the pass over
    # every tile (loss identical, gradients equal to rounding of the sums); k = 30 against the checker; a small
    # workspace (several groups) the same.
    if name == "P1024":
        wl = synth.custom_workload("P4", B=4, T_max=500, U_max=100, H=1024, V=4096, dtype="bf16", index=5,
                                   t_rule="uniform", t_lo=454, u_rule="uniform", u_lo=54)
        ids = list(range(n))
    else:
        wl = synth.WORKLOADS[name]
        ids = _ids_spanning(wl, n)
    batch = synth.make_batch(wl, sample_ids=ids)
    ref = run_oracle(batch)
    dflt = run_gpu(batch, keep_scores=1)
    e, errs = assert_parity(dflt, ref, "bf16", f"{name} kept scores, default tile selection")
    assert_padding_zero(dflt, batch)
    every = run_gpu(batch, keep_scores=1, skip_below_log2=-1)
    np.testing.assert_array_equal(dflt["loss"], every["loss"])
    for key in ("d_enc", "d_pred", "dW_out", "db_out"):
        d = np.abs(dflt[key].astype(np.float64) - every[key]).max() / np.abs(every[key]).max()
        _say("kept scores, default vs every tile", name, key, d)
        assert d < 2e-6, (key, d)
    st, active, total = Bd.rnnt_debug_read_active_tiles(dflt["desc"], batch.T_len, batch.U_len, dflt["workspace"].buf)
    _say("kept scores: default keeps", active, "of", total, "tiles; errs", e, errs)
    assert st == 0 and 0 < active < total
    k30 = run_gpu(batch, keep_scores=1, skip_below_log2=30)
    assert_parity(k30, ref, "bf16", f"{name} kept scores, k = 30")
    st, a30, _ = Bd.rnnt_debug_read_active_tiles(k30["desc"], batch.T_len, batch.U_len, k30["workspace"].buf)
    assert st == 0 and 0 < a30 < active
    # a workspace that cuts the sub-batch into several groups (with kept scores a group is one chunk)
    desc = Bd.make_desc(batch.B, wl.T_max, wl.U_max, wl.H, wl.V, wl.blank, Bd.RNNT_BF16, 0, keep_scores=1)
    nmin = Bd.rnnt_joint_loss_workspace_bytes(desc, batch.T_len, batch.U_len, 1)
    ndef = Bd.rnnt_joint_loss_workspace_bytes(desc, batch.T_len, batch.U_len, 0)
    budget = nmin + (ndef - nmin) // 3
    st, info, _ = Bd.rnnt_joint_loss_plan(desc, batch.T_len, batch.U_len, budget)
    assert st == 0 and info["n_groups"] >= 2, info
    small = run_gpu(batch, keep_scores=1, budget_bytes=budget)
    assert_parity(small, ref, "bf16", f"{name} kept scores, small workspace")
    np.testing.assert_array_equal(small["loss"], dflt["loss"])
