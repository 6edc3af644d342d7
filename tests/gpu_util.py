"""Helpers of the GPU parity tests: run a synthetic batch through the C-ABI library and through
the float64 checker, and compare with the tolerances the build is held to."""
import numpy as np

from oracle import rnnt_oracle as O
from paper_2211_16270_amd import binding as Bd

# relative tolerances: loss = max_b |d loss_b| / |loss_b|; gradients = max|dg| / max|g| per tensor
TOL = {"f32": dict(loss=1e-5, grad=1e-4), "bf16": dict(loss=2e-3, grad=1e-2)}
GRADS = ("d_enc", "d_pred", "dW_out", "db_out")


def run_gpu(batch, budget_bytes=0, blank=None, workspace=None, accumulate_into=None, sample_weight=None,
            keep_scores=0, input_grads_bf16=0, skip_below_log2=0):
    import torch
    wl = batch.wl
    dev = Bd.to_device(batch)
    dt = Bd.RNNT_BF16 if wl.dtype == "bf16" else Bd.RNNT_F32
    out = Bd.run_fwd_bwd(dev, batch.B, wl.T_max, wl.U_max, wl.H, wl.V, wl.blank if blank is None else blank, dt,
                         workspace=workspace, budget_bytes=budget_bytes, accumulate_into=accumulate_into,
                         sample_weight=sample_weight, keep_scores=keep_scores, input_grads_bf16=input_grads_bf16,
                         skip_below_log2=skip_below_log2)
    torch.cuda.synchronize()
    res = {k: out[k].float().cpu().numpy() for k in ("loss",) + GRADS}
    res["workspace"] = out["workspace"]
    res["desc"] = out["desc"]
    res["dev"] = dev
    return res


def run_oracle(batch, blank=None, sample_weight=None):
    wl = batch.wl
    return O.rnnt_joint_loss(batch.enc.astype(np.float64), batch.pred.astype(np.float64),
                             batch.W_out.astype(np.float64), batch.b_out.astype(np.float64),
                             batch.labels, batch.T_len, batch.U_len, wl.blank if blank is None else blank,
                             sample_weight=sample_weight)


def rel_loss_err(got, ref):
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-30)))


def rel_grad_err(got, ref):
    return float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


def assert_parity(got, ref, dtype, what=""):
    tol = TOL[dtype]
    assert np.all(np.isfinite(got["loss"])), what
    e = rel_loss_err(got["loss"].astype(np.float64), ref["loss"])
    assert e <= tol["loss"], f"{what} loss rel err {e:.3e} > {tol['loss']}"
    errs = {}
    for k in GRADS:
        assert np.all(np.isfinite(got[k])), f"{what} {k} not finite"
        errs[k] = rel_grad_err(got[k].astype(np.float64), ref[k])
        assert errs[k] <= tol["grad"], f"{what} {k} rel err {errs[k]:.3e} > {tol['grad']}"
    return e, errs


def assert_padding_zero(got, batch):
    for b in range(batch.B):
        assert np.all(got["d_enc"][b, batch.T_len[b]:] == 0.0)
        assert np.all(got["d_pred"][b, batch.U_len[b] + 1:] == 0.0)
