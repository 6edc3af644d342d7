"""The entry point that allocates nothing (rnnt_joint_loss_fwd_bwd_static: its workspace is a static array in
the library's device code) against rnnt_joint_loss_fwd_bwd with a caller's workspace of the same size, through
the C ABI: two calls in a row on the shared array, the second with a smaller input, then an fp32 call."""
import numpy as np
import pytest

from paper_2211_16270_amd import binding as Bd
from paper_2211_16270_amd import synth
from tests.gpu_util import GRADS, TOL, rel_grad_err, rel_loss_err, run_gpu


def _run_static(batch):
    import torch
    wl = batch.wl
    dev = Bd.to_device(batch)
    dt = Bd.RNNT_BF16 if wl.dtype == "bf16" else Bd.RNNT_F32
    desc = Bd.make_desc(batch.B, wl.T_max, wl.U_max, wl.H, wl.V, wl.blank, dt)
    f32 = dict(dtype=torch.float32, device="cuda:0")
    out = dict(loss=torch.empty(batch.B, **f32), d_enc=torch.empty(batch.B, wl.T_max, wl.H, **f32),
               d_pred=torch.empty(batch.B, wl.U_max + 1, wl.H, **f32), dW_out=torch.empty(wl.H, wl.V, **f32),
               db_out=torch.empty(wl.V, **f32))
    for v in out.values():
        v.fill_(float("nan"))          # every output element must be written by the call
    before = torch.cuda.memory_allocated()
    st = Bd.rnnt_joint_loss_fwd_bwd_static(desc, dev["enc"], dev["pred"], dev["W_out"], dev["b_out"], dev["labels"],
                                           dev["T_len"], dev["U_len"], out["loss"], out["d_enc"], out["d_pred"],
                                           out["dW_out"], out["db_out"])
    assert st == 0, Bd.STATUS_NAMES[st]
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return {k: v.cpu().numpy() for k, v in out.items()}


def _compare(batch, what):
    print("static scratch:", what, batch.T_len.tolist(), batch.U_len.tolist(), flush=True)
    got = _run_static(batch)
    # the existing entry point with a workspace of the array's size follows the same schedule
    same = run_gpu(batch, workspace=Bd.Workspace(Bd.RNNT_STATIC_SCRATCH_BYTES))
    dflt = run_gpu(batch)
    tol = TOL[batch.wl.dtype]
    for k in ("loss",) + GRADS:
        assert np.all(np.isfinite(got[k])), (what, k)
    np.testing.assert_array_equal(got["loss"], same["loss"])
    if batch.wl.dtype == "bf16":
        np.testing.assert_array_equal(got["dW_out"], same["dW_out"])      # summed in a fixed order
    for k in GRADS:
        e = rel_grad_err(got[k], same[k].astype(np.float64))              # atomic sums: order of the additions only
        assert e <= 1e-5, (what, k, e)
        e = rel_grad_err(got[k], dflt[k].astype(np.float64))              # another schedule (default workspace)
        assert e <= tol["grad"], (what, k, e)
    assert rel_loss_err(got["loss"].astype(np.float64), dflt["loss"].astype(np.float64)) <= tol["loss"]
    for b in range(batch.B):
        assert np.all(got["d_enc"][b, batch.T_len[b]:] == 0.0)
        assert np.all(got["d_pred"][b, batch.U_len[b] + 1:] == 0.0)


@pytest.mark.gpu
def test_static_scratch_entry_point_two_calls_in_a_row_then_fp32():
    big = synth.make_batch("C2")                                          # 224 010 lattice nodes, 14 backward chunks
    _compare(big, "C2 full batch")
    small = synth.make_batch(synth.custom_workload("ns", B=4, T_max=37, U_max=19, H=128, V=256, dtype="bf16",
                                                   index=150, t_rule="uniform", t_lo=3, u_rule="uniform", u_lo=0))
    _compare(small, "smaller input on the same array")
    _compare(synth.make_batch("C1"), "fp32, plain kernels")
    _compare(big, "C2 again")


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    wl = synth.WORKLOADS["C5"]                                            # V = 8192: 144 MiB of packed weights and partial sums
    T, U, _ = synth.draw_lengths_labels(wl)
    desc = Bd.make_desc(2, wl.T_max, wl.U_max, wl.H, wl.V, 0, Bd.RNNT_BF16)
    import ctypes
    # rejected on the host before any GPU call: the data pointers are never touched
    st = Bd.lib().rnnt_joint_loss_fwd_bwd_static(ctypes.byref(desc), 256, 256, 256, 256, 256, Bd._ip(Bd._i32(T[:2])),
                                                 Bd._ip(Bd._i32(U[:2])), 256, 256, 256, 256, 256, None)
    assert Bd.STATUS_NAMES[st] == "RNNT_ERR_WORKSPACE"
