"""GPU parity of the path with the joint network's input projections inside (Eq. 4 complete,
Algorithm 1 line 9), through the C ABI, against the float64 checker."""
import numpy as np
import pytest

from oracle import rnnt_oracle as O
from paper_2211_16270_amd import binding as Bd
from paper_2211_16270_amd import synth
from tests.gpu_util import TOL, rel_grad_err, rel_loss_err

pytestmark = pytest.mark.gpu

PGRADS = ("d_hA", "d_hL", "dW_A", "db_Z", "dW_L", "dW_out", "db_out")


def _say(*a):
    print(*a, flush=True)


def run_gpu_proj(batch, proj, budget_bytes=0, accumulate_into=None, keep_scores=0):
    import torch
    wl = batch.wl
    dev = Bd.to_device(batch)
    devp = Bd.proj_to_device(proj, wl.dtype)
    dt = Bd.RNNT_BF16 if wl.dtype == "bf16" else Bd.RNNT_F32
    out = Bd.run_proj_fwd_bwd(dev, devp, batch.B, wl.T_max, wl.U_max, wl.H, wl.V, wl.blank, dt,
                              budget_bytes=budget_bytes, accumulate_into=accumulate_into, keep_scores=keep_scores)
    torch.cuda.synchronize()
    return {k: out[k].float().cpu().numpy() for k in ("loss",) + PGRADS}


def run_oracle_proj(batch, proj):
    f = lambda x: np.asarray(x, dtype=np.float64)
    return O.rnnt_joint_proj_loss(f(proj.hA), f(proj.hL), f(proj.W_A), f(proj.b_Z), f(proj.W_L), f(batch.W_out),
                                  f(batch.b_out), batch.labels, batch.T_len, batch.U_len, batch.wl.blank)


def check(got, ref, dtype, batch, what):
    tol = TOL[dtype]
    el = rel_loss_err(got["loss"].astype(np.float64), ref["loss"])
    errs = {k: rel_grad_err(got[k].astype(np.float64), ref[k]) for k in PGRADS}
    _say(what, "loss", el, {k: float("%.2e" % v) for k, v in errs.items()})
    assert np.all(np.isfinite(got["loss"])) and el <= tol["loss"], (what, el)
    for k in PGRADS:
        assert np.all(np.isfinite(got[k])), (what, k)
        assert errs[k] <= tol["grad"], (what, k, errs[k])
    for b in range(batch.B):
        assert np.all(got["d_hA"][b, batch.T_len[b]:] == 0.0)
        assert np.all(got["d_hL"][b, batch.U_len[b] + 1:] == 0.0)


def test_f32_projected_path_ragged_lengths():
    wl = synth.custom_workload("pf32", B=3, T_max=9, U_max=4, H=24, V=11, dtype="f32", index=131,
                               t_rule="uniform", t_lo=1, u_rule="uniform", u_lo=0)
    batch = synth.make_batch(wl)
    proj = synth.make_proj_inputs(batch, H_A=20, H_L=12)
    check(run_gpu_proj(batch, proj), run_oracle_proj(batch, proj), "f32", batch, "f32 ragged")


@pytest.mark.parametrize("H,V,H_A,H_L", [(256, 128, 132, 200), (24, 11, 10, 7), (128, 256, 516, 4)])
def test_f32_projected_path_tile_gemms_with_edges_and_the_fallback(H, V, H_A, H_L):
    # widths that are multiples of 4 run the projections as fp32 MFMA tile GEMMs (ragged tiles, masked padded rows),
    # others as one thread per output element; (256, 128) and (128, 256) also take the GEMM form of the joint path
    wl = synth.custom_workload("pf32b", B=4, T_max=37, U_max=11, H=H, V=V, dtype="f32", index=133,
                               t_rule="uniform", t_lo=5, u_rule="uniform", u_lo=0)
    batch = synth.make_batch(wl)
    proj = synth.make_proj_inputs(batch, H_A=H_A, H_L=H_L)
    check(run_gpu_proj(batch, proj), run_oracle_proj(batch, proj), "f32", batch, f"f32 {H},{V},{H_A},{H_L}")


def test_f32_identity_projection_equals_the_unprojected_entry_point():
    import torch
    batch = synth.make_batch("C1")
    wl = batch.wl
    fill = lambda x: np.nan_to_num(x, nan=0.0)
    proj = synth.ProjInputs(hA=batch.enc, hL=batch.pred, W_A=np.eye(wl.H, dtype=np.float32),
                            b_Z=np.zeros(wl.H, dtype=np.float32), W_L=np.eye(wl.H, dtype=np.float32))
    got = run_gpu_proj(batch, proj)
    dev = Bd.to_device(batch)
    base = Bd.run_fwd_bwd(dev, batch.B, wl.T_max, wl.U_max, wl.H, wl.V, wl.blank, Bd.RNNT_F32)
    torch.cuda.synchronize()
    np.testing.assert_allclose(got["loss"], base["loss"].cpu().numpy(), rtol=1e-6)
    np.testing.assert_allclose(got["d_hA"], base["d_enc"].cpu().numpy(), atol=1e-6)
    np.testing.assert_allclose(got["d_hL"], base["d_pred"].cpu().numpy(), atol=1e-6)
    np.testing.assert_allclose(got["db_Z"], fill(base["d_enc"].cpu().numpy()).sum(axis=(0, 1)), atol=1e-5)


@pytest.mark.parametrize("H_A,H_L", [(128, 128), (384, 256)])
def test_bf16_projected_path_small(H_A, H_L):
    wl = synth.custom_workload("pbf16", B=4, T_max=37, U_max=11, H=256, V=512, dtype="bf16", index=132,
                               t_rule="uniform", t_lo=5, u_rule="uniform", u_lo=0)
    batch = synth.make_batch(wl)
    proj = synth.make_proj_inputs(batch, H_A=H_A, H_L=H_L)
    ref = run_oracle_proj(batch, proj)
    check(run_gpu_proj(batch, proj), ref, "bf16", batch, f"bf16 small {H_A},{H_L}")
    check(run_gpu_proj(batch, proj, keep_scores=1), ref, "bf16", batch, f"bf16 small {H_A},{H_L}, kept scores")


def test_bf16_projected_path_bench_workload_subbatch_and_accumulate():
    import torch
    ids = [0, 7, 19]
    batch = synth.make_batch("C2", sample_ids=ids)
    proj = synth.make_proj_inputs(batch, H_A=512, H_L=512)
    ref = run_oracle_proj(batch, proj)
    got = run_gpu_proj(batch, proj)
    check(got, ref, "bf16", batch, "C2 sub-batch")
    # accumulate_params: a second call adds to all five parameter gradients
    wl = batch.wl
    acc = {k: torch.from_numpy(got[k].copy()).cuda() for k in ("dW_A", "db_Z", "dW_L", "dW_out", "db_out")}
    got2 = run_gpu_proj(batch, proj, accumulate_into=acc)
    for k in ("dW_A", "db_Z", "dW_L", "dW_out", "db_out"):
        e = rel_grad_err(got2[k].astype(np.float64), 2.0 * ref[k])
        assert e <= TOL["bf16"]["grad"], (k, e)
