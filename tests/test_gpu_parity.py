"""GPU parity: the C-ABI library against the float64 checker, element by element, on the same
seeded inputs (run with -m gpu on an MI355X)."""
import os

import numpy as np
import pytest

from oracle import rnnt_oracle as O
from paper_2211_16270_amd import binding as Bd
from paper_2211_16270_amd import synth
from tests.gpu_util import (GRADS, TOL, assert_padding_zero, assert_parity, rel_grad_err, rel_loss_err,
                            run_gpu, run_oracle)

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------ fp32 path
def test_f32_smallest_workload_full_parity():
    batch = synth.make_batch("C1")
    _say("C1 fp32", batch.T_len, batch.U_len)
    got, ref = run_gpu(batch), run_oracle(batch)
    e, errs = assert_parity(got, ref, "f32", "C1")
    _say("C1 errs", e, errs)
    assert abs(float(got["db_out"].sum())) < 1e-3


@pytest.mark.parametrize("T_len,U_len,blank", [
    ([1, 1], [0, 0], 0),            # single-node lattices: loss = -ln p(blank)
    ([9, 4], [0, 0], 2),            # no labels
    ([1, 1], [5, 3], 0),            # single frame
    ([11, 7], [6, 2], 3),           # ragged, blank in the middle of the vocabulary
    ([13, 2], [1, 6], 0),
])
def test_f32_degenerate_and_ragged_lattices(T_len, U_len, blank):
    wl = synth.custom_workload("edge", B=2, T_max=13, U_max=6, H=24, V=11, dtype="f32", index=101)
    batch = synth.with_lengths(synth.make_batch(wl), T_len, U_len)
    batch.labels[0, :1] = blank if U_len[0] > 0 else batch.labels[0, :1]   # a label equal to the blank
    _say("edge f32", T_len, U_len, blank)
    got, ref = run_gpu(batch, blank=blank), run_oracle(batch, blank=blank)
    assert_parity(got, ref, "f32", f"edge {T_len} {U_len}")
    assert_padding_zero(got, batch)


def test_f32_moderate_shape_and_group_splitting():
    wl = synth.custom_workload("mid32", B=5, T_max=33, U_max=12, H=48, V=70, dtype="f32", index=102,
                               t_rule="uniform", t_lo=5, u_rule="uniform", u_lo=0)
    batch = synth.make_batch(wl)
    ref = run_oracle(batch)
    got = run_gpu(batch)
    assert_parity(got, ref, "f32", "mid32")
    assert_padding_zero(got, batch)
    # smallest possible workspace: one sample per group
    desc = got["desc"]
    nmin = Bd.rnnt_joint_loss_workspace_bytes(desc, batch.T_len, batch.U_len, 1)
    st, info, _ = Bd.rnnt_joint_loss_plan(desc, batch.T_len, batch.U_len, nmin)
    assert st == 0 and info["n_groups"] >= 2
    got2 = run_gpu(batch, budget_bytes=nmin)
    assert_parity(got2, ref, "f32", "mid32 min workspace")


# ------------------------------------------------------------------ fp32 MFMA GEMM form (H, V multiples of 4, >= 64)
@pytest.mark.parametrize("H,V", [(128, 128), (256, 384), (384, 128), (64, 64), (68, 100), (320, 1000), (132, 72)])
def test_f32_gemm_form_against_the_checker(H, V):
    wl = synth.custom_workload("g32", B=5, T_max=37, U_max=11, H=H, V=V, dtype="f32", index=131,
                               t_rule="uniform", t_lo=5, u_rule="uniform", u_lo=0)
    batch = synth.make_batch(wl)
    _say("fp32 GEMM form", H, V, batch.T_len, batch.U_len)
    ref = run_oracle(batch)
    got = run_gpu(batch)
    st, info, _ = Bd.rnnt_joint_loss_plan(got["desc"], batch.T_len, batch.U_len, 0)
    assert st == 0 and info["chunk_rows"] >= 128              # this shape runs as GEMMs over chunk buffers
    e, errs = assert_parity(got, ref, "f32", "fp32 GEMM form")
    _say("fp32 GEMM form errs", e, errs)
    assert_padding_zero(got, batch)
    # smallest workspace: one sample per group, chunks of 128 lattice nodes (several per sample)
    nmin = Bd.rnnt_joint_loss_workspace_bytes(got["desc"], batch.T_len, batch.U_len, 1)
    st, info, _ = Bd.rnnt_joint_loss_plan(got["desc"], batch.T_len, batch.U_len, nmin)
    assert st == 0 and info["chunk_rows"] == 128 and info["n_groups"] >= 2
    small = run_gpu(batch, budget_bytes=nmin)
    assert_parity(small, ref, "f32", "fp32 GEMM form, smallest workspace")
    assert_padding_zero(small, batch)
    # weighted sum of the losses, one sample left out
    w = np.array([0.5, 0.0, 2.0, 1.0 / 3.0, 1.0], dtype=np.float32)
    gw, rw = run_gpu(batch, sample_weight=w), run_oracle(batch, sample_weight=w.astype(np.float64))
    assert_parity(gw, rw, "f32", "fp32 GEMM form, weighted")
    assert np.all(gw["d_enc"][1] == 0.0) and np.all(gw["d_pred"][1] == 0.0)


@pytest.mark.parametrize("T_len,U_len,blank", [
    ([1, 1], [0, 0], 0),
    ([9, 4], [0, 0], 2),
    ([1, 1], [5, 3], 0),
    ([11, 7], [6, 2], 127),
    ([13, 2], [1, 6], 64),
])
def test_f32_gemm_form_edge_lattices(T_len, U_len, blank):
    wl = synth.custom_workload("edge32g", B=2, T_max=13, U_max=6, H=128, V=128, dtype="f32", index=132)
    batch = synth.with_lengths(synth.make_batch(wl), T_len, U_len)
    batch.labels[0, :1] = blank if U_len[0] > 0 else batch.labels[0, :1]
    _say("edge fp32 GEMM form", T_len, U_len, blank)
    got, ref = run_gpu(batch, blank=blank), run_oracle(batch, blank=blank)
    assert_parity(got, ref, "f32", f"edge {T_len} {U_len}")
    assert_padding_zero(got, batch)


def test_f32_gemm_form_several_chunks_and_accumulate():
    import torch
    wl = synth.custom_workload("g32b", B=6, T_max=90, U_max=20, H=256, V=512, dtype="f32", index=133,
                               t_rule="uniform", t_lo=40, u_rule="uniform", u_lo=5)
    batch = synth.make_batch(wl)
    ref = run_oracle(batch)
    got = run_gpu(batch)
    assert_parity(got, ref, "f32", "g32b")
    # a budget that cuts the call into several groups and chunks
    nmin = Bd.rnnt_joint_loss_workspace_bytes(got["desc"], batch.T_len, batch.U_len, 1)
    budget = nmin + (6 << 20)
    st, info, _ = Bd.rnnt_joint_loss_plan(got["desc"], batch.T_len, batch.U_len, budget)
    assert st == 0 and 128 < info["chunk_rows"] < info["rows_total"]
    mid = run_gpu(batch, budget_bytes=budget)
    assert_parity(mid, ref, "f32", "g32b with a budget")
    # accumulate_params: dW_out, db_out are added to what the arrays hold
    acc = (torch.full((wl.H, wl.V), 0.25, device="cuda"), torch.full((wl.V,), -0.5, device="cuda"))
    got2 = run_gpu(batch, accumulate_into=acc)
    assert rel_grad_err(got2["dW_out"] - 0.25, ref["dW_out"]) <= TOL["f32"]["grad"]
    assert rel_grad_err(got2["db_out"] + 0.5, ref["db_out"]) <= TOL["f32"]["grad"]
    # the loss-only entry point runs the forward chunks and the lattice alone
    dev = got["dev"]
    loss = torch.zeros(batch.B, dtype=torch.float32, device="cuda:0")
    st = Bd.rnnt_joint_loss_fwd(got["desc"], dev["enc"], dev["pred"], dev["W_out"], dev["b_out"], dev["labels"],
                                dev["T_len"], dev["U_len"], loss, got["workspace"].buf)
    torch.cuda.synchronize()
    assert st == 0
    np.testing.assert_array_equal(loss.cpu().numpy(), got["loss"])


def test_f32_long_lattices_keep_the_gradient_tolerance():
    # lattices near the largest of the named workloads (1000 x 200): the fp32 path's sweep accumulates in fp64, so
    # that the posteriors of a chain of 1100 dependent log-add-exps stay inside the fp32 gradient tolerance
    wl = synth.custom_workload("long32", B=2, T_max=1000, U_max=200, H=64, V=64, dtype="f32", index=135,
                               t_rule="uniform", t_lo=900, u_rule="uniform", u_lo=150)
    batch = synth.make_batch(wl)
    _say("long fp32 lattices", batch.T_len, batch.U_len)
    got, ref = run_gpu(batch), run_oracle(batch)
    e, errs = assert_parity(got, ref, "f32", "long32")
    _say("long32 errs", e, errs)
    assert_padding_zero(got, batch)


def test_f32_gemm_form_at_the_paper_joint_and_vocabulary_size():
    # H = 1024, V = 4096 (Section 5.1) in fp32, lengths with the paper's padding scheme scaled down; a budget that
    # cuts the backward pass into several chunks
    wl = synth.custom_workload("p32", B=4, T_max=96, U_max=20, H=1024, V=4096, dtype="f32", index=134,
                               t_rule="uniform", t_lo=80, u_rule="uniform", u_lo=10)
    batch = synth.make_batch(wl)
    _say("fp32 GEMM form 1024 x 4096", batch.T_len, batch.U_len)
    ref = run_oracle(batch)
    got = run_gpu(batch)
    e, errs = assert_parity(got, ref, "f32", "p32")
    _say("p32 errs", e, errs)
    assert_padding_zero(got, batch)
    nmin = Bd.rnnt_joint_loss_workspace_bytes(got["desc"], batch.T_len, batch.U_len, 1)
    budget = nmin + (40 << 20)
    st, info, _ = Bd.rnnt_joint_loss_plan(got["desc"], batch.T_len, batch.U_len, budget)
    assert st == 0 and 128 < info["chunk_rows"] < info["rows_total"]
    assert_parity(run_gpu(batch, budget_bytes=budget), ref, "f32", "p32 with a budget")


@pytest.mark.parametrize("seed", range(4))
def test_f32_gemm_form_random_shapes(seed):
    rng = np.random.default_rng(9500 + seed)
    H, V = int(rng.choice([128, 256, 384])), int(rng.choice([128, 256, 640]))
    B, T_max, U_max = int(rng.integers(1, 6)), int(rng.integers(1, 41)), int(rng.integers(0, 21))
    blank = int(rng.integers(0, V))
    wl = synth.custom_workload(f"rg{seed}", B=B, T_max=T_max, U_max=U_max, H=H, V=V, dtype="f32", index=340 + seed)
    T_len, U_len = rng.integers(1, T_max + 1, size=B), rng.integers(0, U_max + 1, size=B)
    batch = synth.with_lengths(synth.make_batch(wl), T_len, U_len)
    labels = rng.integers(0, V, size=batch.labels.shape).astype(np.int32)        # blank included on purpose
    for b in range(B):
        labels[b, U_len[b]:] = -1
    import dataclasses
    batch = dataclasses.replace(batch, labels=labels)
    smallest = bool(rng.integers(0, 2))
    _say("random fp32 GEMM form", seed, dict(B=B, T_max=T_max, U_max=U_max, H=H, V=V, blank=blank), T_len.tolist(),
         U_len.tolist(), "smallest workspace" if smallest else "")
    budget = 0
    if smallest:
        budget = Bd.rnnt_joint_loss_workspace_bytes(Bd.make_desc(B, T_max, U_max, H, V, blank, Bd.RNNT_F32), T_len, U_len, 1)
    got = run_gpu(batch, blank=blank, budget_bytes=budget)
    assert_parity(got, run_oracle(batch, blank=blank), "f32", f"random fp32 GEMM form {seed}")
    assert_padding_zero(got, batch)


# ------------------------------------------------------------------ bf16 MFMA path
def _mid_bf16(index=110, **kw):
    args = dict(B=4, T_max=37, U_max=19, H=128, V=256, dtype="bf16", index=index,
                t_rule="uniform", t_lo=3, u_rule="uniform", u_lo=0)
    args.update(kw)
    return synth.custom_workload("mid16", **args)


def test_bf16_mid_shape_full_parity_and_lattice():
    batch = synth.make_batch(_mid_bf16())
    _say("mid bf16", batch.T_len, batch.U_len)
    got, ref = run_gpu(batch), run_oracle(batch)
    e, errs = assert_parity(got, ref, "bf16", "mid16")
    _say("mid16 errs", e, errs)
    assert_padding_zero(got, batch)
    # forward/backward variables against the checker (fp32 lattice, bf16 GEMM inputs)
    b = 1
    st, al, be = Bd.rnnt_debug_read_lattice(got["desc"], batch.T_len, batch.U_len, got["workspace"].buf, b)
    assert st == 0
    T, U = int(batch.T_len[b]), int(batch.U_len[b])
    r = O.sample_loss_and_grads(batch.enc[b, :T], batch.pred[b, :U + 1], batch.W_out, batch.b_out,
                                batch.labels[b, :U], 0, want_intermediates=True)
    assert np.max(np.abs(al - r["alpha"])) < 2e-3 * max(1.0, np.abs(r["alpha"]).max())
    assert np.max(np.abs(be - r["beta"])) < 2e-3 * max(1.0, np.abs(r["beta"]).max())


@pytest.mark.parametrize("T_len,U_len,blank", [
    ([1, 1, 8, 9], [0, 7, 0, 8], 0),
    ([37, 16, 17, 1], [19, 15, 16, 19], 5),
    ([8, 8, 8, 8], [7, 7, 7, 7], 255),
    ([16, 8, 32, 5], [3, 7, 11, 2], 0),          # one 16 x 4 tile; one 8 x 8 tile; 16 x 4 tiles, three wide; one partly filled
])
def test_bf16_edge_lattices(T_len, U_len, blank):
    batch = synth.with_lengths(synth.make_batch(_mid_bf16(111, t_rule="full", u_rule="full")), T_len, U_len)
    batch.labels[1, :1] = blank
    _say("edge bf16", T_len, U_len, blank)
    got, ref = run_gpu(batch, blank=blank), run_oracle(batch, blank=blank)
    assert_parity(got, ref, "bf16", f"edge16 {T_len}")
    assert_padding_zero(got, batch)


@pytest.mark.parametrize("H,V", [(640, 256), (1024, 512), (256, 768), (896, 256)])
def test_bf16_other_hidden_sizes(H, V):
    # H > 512 takes the unfused backward (separate dz GEMM), H = 640 also the partial 256-wide tile of
    # the dW GEMM; V = 768 is a vocabulary that is not a multiple of the 512-entry step
    wl = synth.custom_workload("wide", B=3, T_max=21, U_max=11, H=H, V=V, dtype="bf16", index=115,
                               t_rule="uniform", t_lo=5, u_rule="uniform", u_lo=1)
    batch = synth.make_batch(wl)
    _say("wide bf16", H, V, batch.T_len, batch.U_len)
    got, ref = run_gpu(batch), run_oracle(batch)
    e, errs = assert_parity(got, ref, "bf16", f"H={H} V={V}")
    _say("errs", e, errs)
    assert_padding_zero(got, batch)


def test_bf16_grouping_and_chunking_do_not_change_the_result():
    batch = synth.make_batch(_mid_bf16(112, B=6))
    ref = run_oracle(batch)
    full = run_gpu(batch)
    desc = full["desc"]
    nmin = Bd.rnnt_joint_loss_workspace_bytes(desc, batch.T_len, batch.U_len, 1)
    st, info, _ = Bd.rnnt_joint_loss_plan(desc, batch.T_len, batch.U_len, nmin)
    _say("min plan", info)
    assert st == 0 and info["n_groups"] >= 2 and info["n_chunks"] > info["n_groups"]
    small = run_gpu(batch, budget_bytes=nmin)
    assert_parity(small, ref, "bf16", "min workspace")
    assert_parity(full, ref, "bf16", "default workspace")
    assert rel_loss_err(small["loss"], full["loss"]) < 1e-6     # the loss has no atomics in it
    # permuting the batch permutes the per-sample outputs
    perm = np.array([3, 0, 5, 1, 4, 2])
    pb = synth.Batch(batch.wl, batch.sample_ids[perm], batch.enc[perm], batch.pred[perm], batch.W_out,
                     batch.b_out, batch.labels[perm], batch.T_len[perm], batch.U_len[perm])
    p = run_gpu(pb)
    assert rel_loss_err(p["loss"], full["loss"][perm]) < 1e-6
    assert rel_grad_err(p["d_enc"], full["d_enc"][perm]) < 1e-5
    assert rel_grad_err(p["dW_out"], full["dW_out"]) < 1e-4


def test_bf16_accumulate_params_and_forward_only():
    import torch
    batch = synth.make_batch(_mid_bf16(113, B=2))
    first = run_gpu(batch)
    dW = torch.full((batch.wl.H, batch.wl.V), 0.5, dtype=torch.float32, device="cuda:0")
    db = torch.full((batch.wl.V,), -0.25, dtype=torch.float32, device="cuda:0")
    second = run_gpu(batch, accumulate_into=(dW, db))
    assert rel_grad_err(second["dW_out"] - 0.5, first["dW_out"]) < 1e-4
    assert rel_grad_err(second["db_out"] + 0.25, first["db_out"]) < 1e-4
    dev = first["dev"]
    loss = torch.zeros(batch.B, dtype=torch.float32, device="cuda:0")
    st = Bd.rnnt_joint_loss_fwd(first["desc"], dev["enc"], dev["pred"], dev["W_out"], dev["b_out"], dev["labels"],
                                dev["T_len"], dev["U_len"], loss, first["workspace"].buf)
    torch.cuda.synchronize()
    assert st == 0
    np.testing.assert_array_equal(loss.cpu().numpy(), first["loss"])


def _closed_form(T, U, V):
    with open(os.path.join(GOLD, "uniform_scores_closed_form.txt")) as f:
        for line in f:
            if line.startswith("#"):
                continue
            t, u, v, val = line.split()
            if (int(t), int(u), int(v)) == (T, U, V):
                return float(val)
    raise KeyError((T, U, V))


@pytest.mark.parametrize("opts", [{}, dict(keep_scores=1, input_grads_bf16=1)])
def test_uniform_scores_closed_form_at_the_largest_lattice(opts):
    # W_out = 0: every emission has probability 1/V; checks the lattice kernel at T=1000, U=200
    wl = synth.custom_workload("uni", B=2, T_max=1000, U_max=200, H=128, V=1024, dtype="bf16", index=114)
    batch = synth.make_batch(wl, pad="zero")
    batch.W_out[:] = 0.0
    batch = synth.with_lengths(batch, [1000, 250], [200, 50], pad="zero")
    got = run_gpu(batch, **opts)
    ref = np.array([_closed_form(1000, 200, 1024), _closed_form(250, 50, 1024)])
    _say("uniform", got["loss"], ref)
    assert rel_loss_err(got["loss"].astype(np.float64), ref) < 2e-6
    assert np.abs(got["d_enc"]).max() == 0.0          # dz = dh W^T = 0
    # dh = gamma/V - posteriors sums to zero over V at every node, hence db sums to zero
    assert abs(float(got["db_out"].astype(np.float64).sum())) < 1e-4 * float(np.abs(got["db_out"]).sum())
    # db[blank] = sum gamma / V - T: every alignment emits T blanks and gamma sums to T+U
    for_b = [(1000 + 200) / 1024 - 1000, (250 + 50) / 1024 - 250]
    assert abs(float(got["db_out"][0]) - sum(for_b)) < 1e-2 * abs(sum(for_b))


@pytest.mark.parametrize("scale", [8.0, 16.0])
def test_bf16_saturated_joint_and_peaked_softmax(scale):
    # inputs 8x and weights 4x the benchmark's scale (powers of two keep them bf16 values): tanh is
    # saturated for most elements, the scores reach several tens, the softmax is close to one-hot and
    # the per-sample loss is in the hundreds; nothing may overflow and the result must still match.
    # At 16x some inputs lie beyond +-40, where the joint tile is built from the sums instead of from
    # products of exponentials (and inputs of opposite sign and that size still cancel exactly).
    from dataclasses import replace
    wl = synth.custom_workload("peaky", B=3, T_max=29, U_max=13, H=256, V=512, dtype="bf16", index=124,
                               t_rule="uniform", t_lo=7, u_rule="uniform", u_lo=1)
    batch = synth.make_batch(wl)
    batch = replace(batch, enc=batch.enc * scale, pred=batch.pred * scale, W_out=batch.W_out * 4.0,
                    b_out=(np.arange(wl.V, dtype=np.float32) % 7 - 3.0) * 2.0)
    if scale > 8.0:
        # a frame and a label position whose inputs are large and cancel: z = tanh(0) there, not 0 * inf
        batch.enc[0, 2, :] = 64.0
        batch.pred[0, 1, :] = -64.0
    got, ref = run_gpu(batch), run_oracle(batch)
    _say("peaky loss", ref["loss"])
    e, errs = assert_parity(got, ref, "bf16", "peaky")
    _say("peaky errs", e, errs)
    assert_padding_zero(got, batch)


def test_mfma_loop_of_the_measurement_entry_point_multiplies():
    # ones times ones: every MFMA adds 16 to each accumulator element; the checksum of a lane is the sum of two
    # elements of each of its 16 accumulator tiles
    import torch
    frags = torch.ones(32 * 64 * 8, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(3 * 256, dtype=torch.float32, device="cuda")
    assert Bd.rnnt_debug_mfma_loop(frags, out, 3, 5) == 0
    torch.cuda.synchronize()
    assert bool((out == 16 * 2 * 16.0 * 5).all())


def test_fp8_mfma_loop_of_the_measurement_entry_point_multiplies():
    # e4m3 ones (0x38) times ones: every 32x32x64 MFMA adds 64 to each accumulator element
    import torch
    frags = torch.full((32 * 64 * 32,), 0x38, dtype=torch.uint8, device="cuda")
    out = torch.zeros(2 * 256, dtype=torch.float32, device="cuda")
    assert Bd.rnnt_debug_mfma_loop_fp8(frags, out, 2, 3) == 0
    torch.cuda.synchronize()
    assert bool((out == 16 * 2 * 64.0 * 3).all()), out[:4]


# ------------------------------------------------------------------ scores kept instead of computed twice
@pytest.mark.parametrize("H,V", [(128, 256), (640, 1024), (896, 256), (1024, 512), (256, 768), (1024, 4096)])
def test_bf16_kept_scores_match_the_checker_and_the_default_path(H, V):
    wl = synth.custom_workload("keep", B=5, T_max=27, U_max=12, H=H, V=V, dtype="bf16", index=130,
                               t_rule="uniform", t_lo=3, u_rule="uniform", u_lo=0)
    batch = synth.make_batch(wl)
    batch.labels[2, :1] = 0                                  # a label equal to the blank
    _say("keep", H, V, batch.T_len, batch.U_len)
    ref = run_oracle(batch)
    got = run_gpu(batch, keep_scores=1)
    e, errs = assert_parity(got, ref, "bf16", f"kept scores H={H} V={V}")
    _say("errs", e, errs)
    assert_padding_zero(got, batch)
    plain = run_gpu(batch)
    np.testing.assert_array_equal(got["loss"], plain["loss"])     # the same forward arithmetic
    # smallest workspace: several groups, each one backward chunk
    nmin = Bd.rnnt_joint_loss_workspace_bytes(got["desc"], batch.T_len, batch.U_len, 1)
    st, info, _ = Bd.rnnt_joint_loss_plan(got["desc"], batch.T_len, batch.U_len, nmin)
    assert st == 0 and info["n_groups"] == info["n_chunks"] > 1
    small = run_gpu(batch, budget_bytes=nmin, keep_scores=1)
    assert_parity(small, ref, "bf16", "kept scores, smallest workspace")
    np.testing.assert_array_equal(small["loss"], got["loss"])


def test_bf16_kept_scores_with_large_scores_and_weights():
    # scores of several tens: what is kept is the difference to a running maximum, so the size of the
    # scores does not enter the error; weights scale the posteriors in the pass that makes dh
    from dataclasses import replace
    wl = synth.custom_workload("peaky", B=3, T_max=29, U_max=13, H=256, V=512, dtype="bf16", index=124,
                               t_rule="uniform", t_lo=7, u_rule="uniform", u_lo=1)
    batch = synth.make_batch(wl)
    batch = replace(batch, enc=batch.enc * 8.0, pred=batch.pred * 8.0, W_out=batch.W_out * 4.0,
                    b_out=(np.arange(wl.V, dtype=np.float32) % 7 - 3.0) * 2.0)
    w = np.array([0.5, 0.0, 3.0], dtype=np.float32)
    got = run_gpu(batch, keep_scores=1, sample_weight=w)
    ref = run_oracle(batch, sample_weight=w.astype(np.float64))
    e, errs = assert_parity(got, ref, "bf16", "peaky, kept scores")
    _say("peaky kept errs", e, errs)
    assert_padding_zero(got, batch)
    assert not got["d_enc"][1].any() and not got["d_pred"][1].any()


def test_bf16_kept_scores_bench_workload_sampled():
    # the benchmark's smaller bf16 workload at full size: loss of every sample against the default path,
    # gradients against it within the two paths' rounding (both are checked against the checker on sub-batches)
    batch = synth.make_batch("C2")
    plain = run_gpu(batch)
    kept = run_gpu(batch, keep_scores=1)
    np.testing.assert_array_equal(kept["loss"], plain["loss"])
    for k in GRADS:
        err = rel_grad_err(kept[k], plain[k])
        _say("C2 kept vs default", k, err)
        assert err < TOL["bf16"]["grad"], k
    sub = synth.make_batch("C2", sample_ids=[3, 29])
    assert_parity(run_gpu(sub, keep_scores=1), run_oracle(sub), "bf16", "C2 sub-batch, kept scores")


# ------------------------------------------------------------------ d_enc, d_pred as bfloat16
@pytest.mark.parametrize("H,V,keep", [(128, 256, 0), (896, 256, 0), (512, 1024, 0), (256, 512, 1)])
def test_bf16_input_gradient_outputs(H, V, keep):
    wl = synth.custom_workload("g16", B=6, T_max=29, U_max=12, H=H, V=V, dtype="bf16", index=140,
                               t_rule="uniform", t_lo=3, u_rule="uniform", u_lo=0)
    batch = synth.make_batch(wl)
    _say("bf16 grads", H, V, keep, batch.T_len, batch.U_len)
    ref = run_oracle(batch)
    got = run_gpu(batch, input_grads_bf16=1, keep_scores=keep)
    e, errs = assert_parity(got, ref, "bf16", f"bf16 d_enc/d_pred H={H} V={V}")
    _say("errs", e, errs)
    assert_padding_zero(got, batch)
    # the float outputs of the default call, rounded, are the same numbers up to the order of the float sums
    plain = run_gpu(batch, keep_scores=keep)
    np.testing.assert_array_equal(got["loss"], plain["loss"])
    for k in ("d_enc", "d_pred"):
        assert rel_grad_err(got[k], plain[k]) < 5e-3, k
    # smallest workspace: one sample per group, every group converted on its own
    nmin = Bd.rnnt_joint_loss_workspace_bytes(got["desc"], batch.T_len, batch.U_len, 1)
    st, info, _ = Bd.rnnt_joint_loss_plan(got["desc"], batch.T_len, batch.U_len, nmin)
    assert st == 0 and info["n_groups"] == batch.B
    small = run_gpu(batch, budget_bytes=nmin, input_grads_bf16=1, keep_scores=keep)
    assert_parity(small, ref, "bf16", "bf16 d_enc/d_pred, smallest workspace")
    assert_padding_zero(small, batch)


# ------------------------------------------------------------------ weighted sum of the samples' losses
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sample_weights_against_the_checker(dtype):
    if dtype == "f32":
        wl = synth.custom_workload("wf32", B=4, T_max=17, U_max=6, H=32, V=24, dtype="f32", index=121,
                                   t_rule="uniform", t_lo=3, u_rule="uniform", u_lo=0)
    else:
        wl = synth.custom_workload("wbf16", B=4, T_max=37, U_max=19, H=128, V=256, dtype="bf16", index=122,
                                   t_rule="uniform", t_lo=9, u_rule="uniform", u_lo=2)
    batch = synth.make_batch(wl)
    w = np.array([0.5, 0.0, 2.0, 1.0 / 3.0], dtype=np.float32)
    _say("weights", dtype, batch.T_len, batch.U_len, w)
    got, ref = run_gpu(batch, sample_weight=w), run_oracle(batch, sample_weight=w.astype(np.float64))
    e, errs = assert_parity(got, ref, dtype, f"weighted {dtype}")
    _say("weighted errs", e, errs)
    assert_padding_zero(got, batch)
    assert np.all(got["d_enc"][1] == 0.0) and np.all(got["d_pred"][1] == 0.0)       # weight 0: left out
    plain, ones = run_gpu(batch), run_gpu(batch, sample_weight=np.ones(4, dtype=np.float32))
    np.testing.assert_array_equal(plain["loss"], got["loss"])
    for k in GRADS:
        assert rel_grad_err(ones[k], plain[k].astype(np.float64)) < 1e-5, k


def test_autograd_front_end_returns_the_library_gradients():
    import torch
    from paper_2211_16270_amd.autograd import rnnt_joint_loss
    wl = synth.custom_workload("ag", B=3, T_max=21, U_max=7, H=128, V=256, dtype="bf16", index=123,
                               t_rule="uniform", t_lo=5, u_rule="uniform", u_lo=1)
    batch = synth.make_batch(wl, pad="zero")
    dev = Bd.to_device(batch)
    leaves = [dev[k].clone().requires_grad_(True) for k in ("enc", "pred", "W_out", "b_out")]

    def grads_of(reduce, sample_weight=None):
        for x in leaves:
            x.grad = None
        loss = rnnt_joint_loss(*leaves, dev["labels"], batch.T_len, batch.U_len, 0, sample_weight=sample_weight)
        reduce(loss).backward()
        torch.cuda.synchronize()
        return loss.detach().float().cpu().numpy(), [x.grad.float().cpu().numpy() for x in leaves]

    direct = run_gpu(batch)
    loss, g_sum = grads_of(lambda l: l.sum())
    np.testing.assert_array_equal(loss, direct["loss"])
    for got, k in zip(g_sum, GRADS):
        want = torch.from_numpy(direct[k]).to(torch.bfloat16 if k != "db_out" else torch.float32).float().numpy()
        assert rel_grad_err(got, want.astype(np.float64)) < 1e-3, k
    # a mean and a mask: the incoming gradient differs from the weights of the first call, which is repeated
    w = np.array([1.0 / 3, 0.0, 1.0 / 3], dtype=np.float32)
    ref = run_oracle(batch, sample_weight=w.astype(np.float64))
    _, g_w = grads_of(lambda l: (l * torch.tensor(w, device=l.device)).sum())
    _, g_w2 = grads_of(lambda l: (l * torch.tensor(w, device=l.device)).sum(), sample_weight=w)
    for a, b2, k in zip(g_w, g_w2, GRADS):
        assert rel_grad_err(a, ref[k]) <= TOL["bf16"]["grad"], k     # bf16 leaves: gradients rounded to the leaf dtype
        assert rel_grad_err(b2, a.astype(np.float64)) < 1e-3, k
    # the same through the path that keeps the scores
    for x in leaves:
        x.grad = None
    lk = rnnt_joint_loss(*leaves, dev["labels"], batch.T_len, batch.U_len, 0, keep_scores=True)
    (lk * torch.tensor(w, device=lk.device)).sum().backward()
    torch.cuda.synchronize()
    for x, k in zip(leaves, GRADS):
        assert rel_grad_err(x.grad.float().cpu().numpy(), ref[k]) <= TOL["bf16"]["grad"], k


def test_autograd_front_end_with_float32_leaves():
    # fp32 tensors go through the fp32 path (here its MFMA GEMM form): gradients against the checker at the
    # fp32 tolerance, for a plain sum and for a masked mean
    import torch
    from paper_2211_16270_amd.autograd import rnnt_joint_loss
    wl = synth.custom_workload("ag32", B=3, T_max=21, U_max=7, H=128, V=192, dtype="f32", index=124,
                               t_rule="uniform", t_lo=5, u_rule="uniform", u_lo=1)
    batch = synth.make_batch(wl, pad="zero")
    dev = Bd.to_device(batch)
    leaves = [dev[k].clone().requires_grad_(True) for k in ("enc", "pred", "W_out", "b_out")]
    for w in (None, np.array([0.5, 0.0, 0.5], dtype=np.float32)):
        for x in leaves:
            x.grad = None
        loss = rnnt_joint_loss(*leaves, dev["labels"], batch.T_len, batch.U_len, 0)
        (loss.sum() if w is None else (loss * torch.tensor(w, device=loss.device)).sum()).backward()
        torch.cuda.synchronize()
        ref = run_oracle(batch, sample_weight=None if w is None else w.astype(np.float64))
        for x, k in zip(leaves, GRADS):
            assert x.grad.dtype == torch.float32
            assert rel_grad_err(x.grad.cpu().numpy(), ref[k]) <= TOL["f32"]["grad"], (k, w)
        assert rel_loss_err(loss.detach().cpu().numpy().astype(np.float64), run_oracle(batch)["loss"]) <= TOL["f32"]["loss"]


# ------------------------------------------------------------------ the benchmarked workload
def test_bf16_bench_workload_subbatch_parity():
    ids = [0, 17]
    batch = synth.make_batch("C2", sample_ids=ids)
    _say("C2 sub-batch", ids, batch.T_len, batch.U_len)
    got, ref = run_gpu(batch), run_oracle(batch)
    e, errs = assert_parity(got, ref, "bf16", "C2 sub")
    _say("C2 sub errs", e, errs)
    assert_padding_zero(got, batch)


def test_bf16_bench_workload_full_batch_sampled_outputs():
    # the configuration bench.py times: full C2 batch, default workspace; the checker recomputes
    # two samples one by one (loss, d_enc, d_pred are per-sample outputs)
    full = synth.make_batch("C2")
    got = run_gpu(full)
    assert np.all(np.isfinite(got["loss"]))
    assert_padding_zero(got, full)
    tol = TOL["bf16"]
    for b in (3, 29):
        T, U = int(full.T_len[b]), int(full.U_len[b])
        r = O.sample_loss_and_grads(full.enc[b, :T], full.pred[b, :U + 1], full.W_out, full.b_out,
                                    full.labels[b, :U], 0)
        assert abs(got["loss"][b] - r["loss"]) <= tol["loss"] * abs(r["loss"])
        assert rel_grad_err(got["d_enc"][b, :T], r["d_enc"]) <= tol["grad"]
        assert rel_grad_err(got["d_pred"][b, :U + 1], r["d_pred"]) <= tol["grad"]
    # softmax shift invariance: the bias gradient sums to zero (up to bf16 rounding of dh)
    assert abs(float(got["db_out"].astype(np.float64).sum())) < 1e-2 * float(np.abs(got["db_out"]).sum())


def test_bf16_bench_workload_permutation_and_split_invariance():
    # properties that hold at any size: the order of the samples only permutes the per-sample outputs, and
    # the parameter gradients of a batch are the sum of those of its parts (different packing into launches)
    n = 32
    full = run_gpu(synth.make_batch("C2"))
    perm = list(reversed(range(n)))
    rev = run_gpu(synth.make_batch("C2", sample_ids=perm))
    assert np.max(np.abs(rev["loss"] - full["loss"][perm]) / np.abs(full["loss"][perm])) < 1e-5
    for k in ("d_enc", "d_pred"):
        for i, b in enumerate(perm):
            assert rel_grad_err(rev[k][i], full[k][b].astype(np.float64)) < 1e-3, (k, b)
    for k in ("dW_out", "db_out"):
        assert rel_grad_err(rev[k], full[k].astype(np.float64)) < 2e-3, k
    lo = run_gpu(synth.make_batch("C2", sample_ids=list(range(0, 12))))
    hi = run_gpu(synth.make_batch("C2", sample_ids=list(range(12, n))))
    for k in ("dW_out", "db_out"):
        both = lo[k].astype(np.float64) + hi[k].astype(np.float64)
        assert rel_grad_err(full[k], both) < 2e-3, k
    assert np.max(np.abs(np.concatenate([lo["loss"], hi["loss"]]) - full["loss"]) / np.abs(full["loss"])) < 1e-5


def test_bf16_memory_headline_workload_sampled():
    # 12 samples of the B=1024, T<=1000, U<=200 workload: long lattices (multi-wave lattice kernel),
    # several backward chunks; the checker recomputes the sample with the fewest lattice nodes
    ids = list(range(12))
    batch = synth.make_batch("C4", sample_ids=ids)
    got = run_gpu(batch)
    assert np.all(np.isfinite(got["loss"]))
    assert_padding_zero(got, batch)
    rows = batch.T_len.astype(np.int64) * (batch.U_len + 1)
    b = int(np.argmin(rows))
    T, U = int(batch.T_len[b]), int(batch.U_len[b])
    _say("C4 sample", b, T, U)
    r = O.sample_loss_and_grads(batch.enc[b, :T], batch.pred[b, :U + 1], batch.W_out, batch.b_out,
                                batch.labels[b, :U], 0)
    tol = TOL["bf16"]
    el = abs(got["loss"][b] - r["loss"]) / abs(r["loss"])
    ee = rel_grad_err(got["d_enc"][b, :T], r["d_enc"])
    ep = rel_grad_err(got["d_pred"][b, :U + 1], r["d_pred"])
    _say("C4 sample errs", el, ee, ep)
    assert el <= tol["loss"] and ee <= tol["grad"] and ep <= tol["grad"]
    assert abs(float(got["db_out"].astype(np.float64).sum())) < 1e-2 * float(np.abs(got["db_out"]).sum())


def test_bf16_paper_shaped_workload_sampled_default_and_kept_scores():
    # the paper's benchmark shape (Section 5.1: 500 x 100, joint size 1024, 4096 word pieces), four samples:
    # unfused backward (H > 640), and the same with the scores kept and bfloat16 input gradients; the checker
    # recomputes the sample with the fewest lattice nodes
    wl = synth.custom_workload("P4", B=4, T_max=500, U_max=100, H=1024, V=4096, dtype="bf16", index=5,
                               t_rule="uniform", t_lo=454, u_rule="uniform", u_lo=54)
    batch = synth.make_batch(wl)
    rows = batch.T_len.astype(np.int64) * (batch.U_len + 1)
    b = int(np.argmin(rows))
    T, U = int(batch.T_len[b]), int(batch.U_len[b])
    _say("paper-shaped sample", b, T, U)
    r = O.sample_loss_and_grads(batch.enc[b, :T], batch.pred[b, :U + 1], batch.W_out, batch.b_out,
                                batch.labels[b, :U], 0)
    tol = TOL["bf16"]
    plain = run_gpu(batch)
    kept = run_gpu(batch, keep_scores=1, input_grads_bf16=1)
    for name, got in (("default", plain), ("kept scores, bf16 input gradients", kept)):
        assert np.all(np.isfinite(got["loss"])), name
        assert_padding_zero(got, batch)
        el = abs(got["loss"][b] - r["loss"]) / abs(r["loss"])
        ee = rel_grad_err(got["d_enc"][b, :T], r["d_enc"])
        ep = rel_grad_err(got["d_pred"][b, :U + 1], r["d_pred"])
        _say(name, "errs", el, ee, ep)
        assert el <= tol["loss"] and ee <= tol["grad"] and ep <= tol["grad"], name
        assert abs(float(got["db_out"].astype(np.float64).sum())) < 1e-2 * float(np.abs(got["db_out"]).sum())
    np.testing.assert_array_equal(kept["loss"], plain["loss"])
    for k in ("dW_out", "db_out"):
        assert rel_grad_err(kept[k], plain[k]) <= tol["grad"], k


def test_f32_paper_shaped_bench_workload_sampled():
    # the workload of `bench.py --config P16F32` (16 samples up to 500 x 100, joint size 1024, 4096 word pieces, fp32)
    # in the default plan that the benchmark times; the checker recomputes the sample with the fewest lattice nodes
    wl = synth.custom_workload("P16F32", B=16, T_max=500, U_max=100, H=1024, V=4096, dtype="f32", index=5,
                               t_rule="uniform", t_lo=454, u_rule="uniform", u_lo=54)
    batch = synth.make_batch(wl)
    rows = batch.T_len.astype(np.int64) * (batch.U_len + 1)
    b = int(np.argmin(rows))
    T, U = int(batch.T_len[b]), int(batch.U_len[b])
    _say("paper-shaped fp32 sample", b, T, U)
    r = O.sample_loss_and_grads(batch.enc[b, :T], batch.pred[b, :U + 1], batch.W_out, batch.b_out,
                                batch.labels[b, :U], 0)
    got = run_gpu(batch)
    st, info, _ = Bd.rnnt_joint_loss_plan(got["desc"], batch.T_len, batch.U_len, 0)
    assert st == 0 and 128 <= info["chunk_rows"] < info["rows_total"]       # several chunks of lattice nodes
    assert np.all(np.isfinite(got["loss"]))
    assert_padding_zero(got, batch)
    tol = TOL["f32"]
    el = abs(got["loss"][b] - r["loss"]) / abs(r["loss"])
    ee = rel_grad_err(got["d_enc"][b, :T], r["d_enc"])
    ep = rel_grad_err(got["d_pred"][b, :U + 1], r["d_pred"])
    _say("paper-shaped fp32 errs", el, ee, ep)
    assert el <= tol["loss"] and ee <= tol["grad"] and ep <= tol["grad"]
    assert abs(float(got["db_out"].astype(np.float64).sum())) < 1e-4 * float(np.abs(got["db_out"]).sum())


@pytest.mark.parametrize("opts", [{}, dict(keep_scores=1)])
def test_bf16_vocabulary_padded_to_the_tile_with_a_large_negative_bias(opts):
    # a vocabulary that is not a multiple of 256 (here 300) is padded by the caller: zero columns in W_out and a
    # bias of -1e4 there, so that the padding has probability exp(-1e4) = 0; the checker sees the 300 real entries
    import dataclasses
    V_real, V_pad = 300, 512
    wl = synth.custom_workload("vpad", B=3, T_max=29, U_max=9, H=128, V=V_pad, dtype="bf16", index=140,
                               t_rule="uniform", t_lo=8, u_rule="uniform", u_lo=1)
    batch = synth.make_batch(wl)
    labels = np.where(batch.labels >= 0, batch.labels % (V_real - 1) + 1, batch.labels).astype(np.int32)
    W = batch.W_out.copy(); W[:, V_real:] = 0.0
    b = np.zeros(V_pad, dtype=np.float32); b[V_real:] = -1e4
    padded = dataclasses.replace(batch, W_out=W, b_out=b, labels=labels)
    got = run_gpu(padded, **opts)
    real = dataclasses.replace(padded, wl=dataclasses.replace(wl, V=V_real), W_out=W[:, :V_real].copy(),
                               b_out=b[:V_real].copy())
    ref = run_oracle(real)
    assert np.all(got["dW_out"][:, V_real:] == 0.0) and np.all(got["db_out"][V_real:] == 0.0)
    cut = dict(got, dW_out=got["dW_out"][:, :V_real], db_out=got["db_out"][:V_real])
    assert_parity(cut, ref, "bf16", f"padded vocabulary {opts}")
    assert_padding_zero(got, padded)


@pytest.mark.parametrize("seed", range(12))
def test_random_small_shapes_against_the_checker(seed):
    # seeded random shapes, lengths and blank positions, both precisions; labels may equal the blank
    rng = np.random.default_rng(9000 + seed)
    bf16 = bool(seed % 3)
    if bf16:
        H = int(rng.choice([128, 256, 384, 512, 640, 768, 1024]))
        V = int(rng.choice([256, 512, 768, 1024]))
    else:
        H = int(rng.integers(1, 70))
        V = int(rng.integers(2, 90))
    B = int(rng.integers(1, 6))
    T_max = int(rng.integers(1, 41))
    U_max = int(rng.integers(0, 21))
    blank = int(rng.integers(0, V))
    wl = synth.custom_workload(f"rnd{seed}", B=B, T_max=T_max, U_max=U_max, H=H, V=V, dtype="bf16" if bf16 else "f32",
                               index=300 + seed)
    batch = synth.make_batch(wl)
    T_len = rng.integers(1, T_max + 1, size=B)
    U_len = rng.integers(0, U_max + 1, size=B)
    batch = synth.with_lengths(batch, T_len, U_len)
    labels = rng.integers(0, V, size=batch.labels.shape).astype(np.int32)        # blank included on purpose
    for b in range(B):
        labels[b, U_len[b]:] = -1
    import dataclasses
    batch = dataclasses.replace(batch, labels=labels)
    # the descriptor's options (bf16 path) and the smallest workspace, drawn last so that the shapes stay what they were
    opts = dict(keep_scores=int(rng.integers(0, 2)), input_grads_bf16=int(rng.integers(0, 2))) if bf16 else {}
    smallest = bool(rng.integers(0, 2))
    _say("random shape", seed, "bf16" if bf16 else "f32", dict(B=B, T_max=T_max, U_max=U_max, H=H, V=V, blank=blank),
         T_len.tolist(), U_len.tolist(), opts, "smallest workspace" if smallest else "")
    budget = 0
    if smallest:
        dt = Bd.RNNT_BF16 if bf16 else Bd.RNNT_F32
        budget = Bd.rnnt_joint_loss_workspace_bytes(Bd.make_desc(B, T_max, U_max, H, V, blank, dt, 0, **opts), T_len, U_len, 1)
    got = run_gpu(batch, blank=blank, budget_bytes=budget, **opts)
    ref = run_oracle(batch, blank=blank)
    assert_parity(got, ref, wl.dtype, f"random shape {seed}")
    assert_padding_zero(got, batch)
