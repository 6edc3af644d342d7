"""Seeded synthetic transducer batches (inputs only, no transducer arithmetic).

The benchmarks of the paper (Section 5.1) feed the joint network with randomly
initialised, fixed-seed encodings; no dataset is involved.  This module draws
such batches for the five workloads this build is measured on.  It is the one
module that both the float64 checker and the GPU path's tests/bench use; it
holds nothing but random draws, length/label distributions and the
float32 <-> bfloat16 bit conversion of the *inputs*.

Recipe (per workload index ``i``; all streams are numpy PCG64):

* ``SeedSequence([2211, i, 0])``  -> ``T_len`` then ``U_len`` then ``labels``
* ``SeedSequence([2211, i, 1])``  -> ``W_out``  (N(0, 1/H), float32)
* ``SeedSequence([2211, i, 2, b])`` -> sample ``b``: ``enc[b, :T_b]`` then
  ``pred[b, :U_b+1]`` (N(0,1), float32)

so a sub-batch picked by sample indices carries exactly the values those
samples have in the full batch.  ``b_out`` is zero.  For the bf16 workloads the
float32 draws are rounded once (round-to-nearest-even) and every consumer sees
the rounded values.  Entries beyond a sample's own lengths are filler: NaN
(labels: -1) when ``pad="nan"``, zeros when ``pad="zero"``.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Sequence

import numpy as np

BASE_SEED = 2211


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    B: int
    T_max: int
    U_max: int
    H: int
    V: int
    dtype: str            # "f32" or "bf16": storage type of enc, pred, W_out
    blank: int = 0
    t_rule: str = "full"  # full | uniform | loguniform
    t_lo: int = 0
    u_rule: str = "full"  # full | uniform | ratio
    u_lo: int = 0
    u_ratio: float = 0.0
    label_rule: str = "uniform"  # uniform | zipf
    zipf_s: float = 1.1


WORKLOADS = {
    "C1": Workload("C1", 0, B=2, T_max=20, U_max=5, H=32, V=16, dtype="f32"),
    "C2": Workload("C2", 1, B=32, T_max=250, U_max=50, H=512, V=1024, dtype="bf16",
                   t_rule="uniform", t_lo=150, u_rule="uniform", u_lo=20),
    "C3": Workload("C3", 2, B=128, T_max=500, U_max=100, H=640, V=4096, dtype="bf16",
                   t_rule="uniform", t_lo=250, u_rule="uniform", u_lo=40),
    "C4": Workload("C4", 3, B=1024, T_max=1000, U_max=200, H=512, V=1024, dtype="bf16",
                   t_rule="uniform", t_lo=500, u_rule="uniform", u_lo=80),
    "C5": Workload("C5", 4, B=256, T_max=800, U_max=300, H=512, V=8192, dtype="bf16",
                   t_rule="loguniform", t_lo=50, u_rule="ratio", u_ratio=0.3,
                   label_rule="zipf", zipf_s=1.1),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns.
    NaN stays NaN (quiet bit forced)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r[nan] = np.uint16(0x7FC0)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Batch:
    """One synthetic batch.  ``enc``/``pred``/``W_out`` are float32 arrays holding the
    values every consumer must use (already bf16-representable when ``dtype=="bf16"``)."""
    wl: Workload
    sample_ids: np.ndarray   # [B] indices into the full workload batch
    enc: np.ndarray          # [B, T_max, H] float32
    pred: np.ndarray         # [B, U_max+1, H] float32
    W_out: np.ndarray        # [H, V] float32
    b_out: np.ndarray        # [V] float32
    labels: np.ndarray       # [B, U_max] int32
    T_len: np.ndarray        # [B] int32
    U_len: np.ndarray        # [B] int32

    @property
    def B(self) -> int:
        return int(self.T_len.shape[0])

    @property
    def rows(self) -> int:
        return int(np.sum(self.T_len.astype(np.int64) * (self.U_len.astype(np.int64) + 1)))


def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([BASE_SEED, *key])))


def draw_lengths_labels(wl: Workload):
    """Lengths and labels of the full batch of a workload (cheap; no encodings)."""
    g = _rng(wl.index, 0)
    B = wl.B
    if wl.t_rule == "full":
        T_len = np.full(B, wl.T_max, dtype=np.int32)
    elif wl.t_rule == "uniform":
        T_len = g.integers(wl.t_lo, wl.T_max + 1, size=B).astype(np.int32)
    elif wl.t_rule == "loguniform":
        x = np.exp(g.uniform(np.log(wl.t_lo), np.log(wl.T_max), size=B))
        T_len = np.clip(np.floor(x + 0.5), wl.t_lo, wl.T_max).astype(np.int32)
    else:
        raise ValueError(wl.t_rule)
    if wl.u_rule == "full":
        U_len = np.full(B, wl.U_max, dtype=np.int32)
    elif wl.u_rule == "uniform":
        U_len = g.integers(wl.u_lo, wl.U_max + 1, size=B).astype(np.int32)
    elif wl.u_rule == "ratio":
        U_len = np.minimum(np.floor(wl.u_ratio * T_len + 0.5), wl.U_max).astype(np.int32)
    else:
        raise ValueError(wl.u_rule)
    # labels never equal the blank (index 0) in the five workloads
    if wl.label_rule == "uniform":
        labels = g.integers(1, wl.V, size=(B, wl.U_max)).astype(np.int32)
    elif wl.label_rule == "zipf":
        k = np.arange(1, wl.V, dtype=np.float64)
        cdf = np.cumsum(k ** (-wl.zipf_s))
        cdf /= cdf[-1]
        u = g.random(size=(B, wl.U_max))
        labels = (np.searchsorted(cdf, u, side="left") + 1).astype(np.int32)
        labels = np.minimum(labels, wl.V - 1)
    else:
        raise ValueError(wl.label_rule)
    return T_len, U_len, labels


def make_batch(wl: Workload | str, sample_ids: Optional[Sequence[int]] = None,
               pad: str = "nan") -> Batch:
    """Draw the batch (or the sub-batch ``sample_ids``) of a workload."""
    if isinstance(wl, str):
        wl = WORKLOADS[wl]
    T_all, U_all, lab_all = draw_lengths_labels(wl)
    ids = np.arange(wl.B) if sample_ids is None else np.asarray(sample_ids, dtype=np.int64)
    Bs = len(ids)
    fill = np.nan if pad == "nan" else 0.0
    enc = np.full((Bs, wl.T_max, wl.H), fill, dtype=np.float32)
    pred = np.full((Bs, wl.U_max + 1, wl.H), fill, dtype=np.float32)
    labels = np.full((Bs, wl.U_max), -1 if pad == "nan" else 0, dtype=np.int32)
    T_len = T_all[ids].copy()
    U_len = U_all[ids].copy()
    for j, b in enumerate(ids):
        g = _rng(wl.index, 2, int(b))
        Tb, Ub = int(T_len[j]), int(U_len[j])
        enc[j, :Tb] = g.standard_normal((Tb, wl.H), dtype=np.float32)
        pred[j, :Ub + 1] = g.standard_normal((Ub + 1, wl.H), dtype=np.float32)
        labels[j, :Ub] = lab_all[b, :Ub]
    gw = _rng(wl.index, 1)
    W_out = (gw.standard_normal((wl.H, wl.V), dtype=np.float32)
             * np.float32(1.0 / np.sqrt(wl.H))).astype(np.float32)
    b_out = np.zeros(wl.V, dtype=np.float32)
    if wl.dtype == "bf16":
        enc = bf16_bits_to_f32(f32_to_bf16_bits(enc))
        pred = bf16_bits_to_f32(f32_to_bf16_bits(pred))
        W_out = bf16_bits_to_f32(f32_to_bf16_bits(W_out))
    return Batch(wl, ids, enc, pred, W_out, b_out, labels, T_len, U_len)


def custom_workload(name: str, B: int, T_max: int, U_max: int, H: int, V: int, dtype: str,
                    index: int = 100, **kw) -> Workload:
    """A workload outside the five named ones (used by edge-case tests)."""
    return Workload(name, index, B=B, T_max=T_max, U_max=U_max, H=H, V=V, dtype=dtype, **kw)


def with_lengths(batch: Batch, T_len, U_len, pad: str = "nan") -> Batch:
    """Same draws, other lengths (must not exceed the drawn ones); filler re-applied."""
    T_len = np.asarray(T_len, dtype=np.int32)
    U_len = np.asarray(U_len, dtype=np.int32)
    assert np.all(T_len <= batch.T_len) and np.all(U_len <= batch.U_len)
    fill = np.nan if pad == "nan" else 0.0
    enc, pred, labels = batch.enc.copy(), batch.pred.copy(), batch.labels.copy()
    for j in range(batch.B):
        enc[j, T_len[j]:] = fill
        pred[j, U_len[j] + 1:] = fill
        labels[j, U_len[j]:] = -1 if pad == "nan" else 0
    return replace(batch, enc=enc, pred=pred, labels=labels, T_len=T_len, U_len=U_len)


@dataclass
class ProjInputs:
    """Inputs of the two linear maps inside the tanh of the joint network (float32 arrays holding
    the values every consumer must use, bf16-representable for bf16 workloads)."""
    hA: np.ndarray     # [B, T_max, H_A]
    hL: np.ndarray     # [B, U_max+1, H_L]
    W_A: np.ndarray    # [H_A, H]
    b_Z: np.ndarray    # [H] float32
    W_L: np.ndarray    # [H_L, H]


def make_proj_inputs(batch: Batch, H_A: int, H_L: int, pad: str = "nan") -> ProjInputs:
    """Acoustic / label encodings and projection weights for the samples of `batch`: hA, hL ~ N(0,1),
    W_A ~ N(0, 1/H_A), W_L ~ N(0, 1/H_L) (so that the projected encodings are ~ N(0,1) like the
    workloads' enc, pred), b_Z ~ 0.1 N(0,1).  Per-sample streams as in make_batch."""
    wl = batch.wl
    fill = np.nan if pad == "nan" else 0.0
    Bs = batch.B
    hA = np.full((Bs, wl.T_max, H_A), fill, dtype=np.float32)
    hL = np.full((Bs, wl.U_max + 1, H_L), fill, dtype=np.float32)
    for j, b in enumerate(batch.sample_ids):
        g = _rng(wl.index, 3, int(b), H_A, H_L)
        Tb, Ub = int(batch.T_len[j]), int(batch.U_len[j])
        hA[j, :Tb] = g.standard_normal((Tb, H_A), dtype=np.float32)
        hL[j, :Ub + 1] = g.standard_normal((Ub + 1, H_L), dtype=np.float32)
    gw = _rng(wl.index, 4, H_A, H_L)
    W_A = gw.standard_normal((H_A, wl.H), dtype=np.float32) * np.float32(1.0 / np.sqrt(H_A))
    W_L = gw.standard_normal((H_L, wl.H), dtype=np.float32) * np.float32(1.0 / np.sqrt(H_L))
    b_Z = (gw.standard_normal(wl.H, dtype=np.float32) * np.float32(0.1)).astype(np.float32)
    if wl.dtype == "bf16":
        hA, hL, W_A, W_L = (bf16_bits_to_f32(f32_to_bf16_bits(x)) for x in (hA, hL, W_A, W_L))
    return ProjInputs(hA, hL, W_A.astype(np.float32), b_Z, W_L.astype(np.float32))
