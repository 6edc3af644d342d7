"""Float64 CPU checker for the transducer joint -> output layer -> loss -> gradient path.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU
library is compared against.  It is imported by the tests, by the smoke check and
by the benchmark's CPU-baseline leg, never by the product path, and it shares no
code with the HIP kernels.

What it computes (per sample b, on the unpadded slice T = T_len[b], U = U_len[b];
"Section/Eq." refer to the paper, arxiv 2211.16270):

  1. joint            z[t,u,:] = tanh(enc[b,t,:] + pred[b,u,:])          Eq. (4), with the
                      input projections W^A h^A + b^Z and W^L h^L already applied
                      by the caller (enc and pred are the projected encodings)
  2. output layer     h[t,u,:] = z[t,u,:] @ W_out + b_out                 Eq. (6)
  3. f^W_1            lse[t,u] = ln sum_v exp h[t,u,v]                     Eq. (7), Section 2
                      (the log of the softmax denominator P_D), lp = h - lse
  4. emissions        lpb = lp[..., blank],  lpy[t,u] = lp[t,u,y_u]  (u < U)
  5. f^W_2 forward    alpha[0,0] = 0
                      alpha[t,u] = LSE(alpha[t-1,u] + lpb[t-1,u], alpha[t,u-1] + lpy[t,u-1])
  6. f^W_2 backward   beta[T-1,U] = lpb[T-1,U]
                      beta[t,u]  = LSE(beta[t+1,u] + lpb[t,u],  beta[t,u+1] + lpy[t,u])
  7. f^W_3            lnP = alpha[T-1,U] + lpb[T-1,U];  loss[b] = -lnP      Eq. (9), Section 2
  8. f^W_4            dh = gamma * softmax - [v=blank] Bk - [v=y_u] Yk      Eq. (10)
                      gamma = exp(alpha + beta - lnP)
                      Bk[t,u] = exp(alpha[t,u] + lpb[t,u] + beta[t+1,u] - lnP)  (t < T-1)
                      Bk[T-1,U] = exp(alpha[T-1,U] + lpb[T-1,U] - lnP) = 1, Bk[T-1,u<U] = 0
                      Yk[t,u] = exp(alpha[t,u] + lpy[t,u] + beta[t,u+1] - lnP)  (u < U)
  9. Algorithm 1,     db_out += sum_{t,u} dh;  dW_out += z^T dh;  dz = dh W_out^T
     lines 8, 10, 11  dx = dz * (1 - z^2);  d_enc[b,t] = sum_u dx;  d_pred[b,u] = sum_t dx

The paper does not print the lattice recursion (Section 3.1 points to the
transducer literature); steps 5-8 are the standard transducer forward/backward
variables of Graves (2012), cited there, and step 8 is the chain rule through
steps 3-7.  The total loss is the sum over the batch (Section 2), gradients are
those of the sum, and Algorithm 1 states that accumulating per sample gives the
batched result; `rnnt_joint_loss_batched_padded` is that batched form.

`rnnt_joint_proj_loss` puts the two input projections of Eq. (4) (W^A h^A + b^Z, W^L h^L) in
front and chains the gradients back through them (Algorithm 1 line 9); it is pinned by finite
differences of the whole chain, by its reduction to `rnnt_joint_loss` for identity projections
and by sum_t d_enc = sum_u d_pred (both are the gradient of b^Z).

Pins (tests/test_oracle_*.py): exhaustive alignment enumeration, the closed forms
for T=1, U=0 and uniform scores, sum_v dh = 0, occupation identities of the
lattice, central finite differences through the whole chain (also of the weighted
sum of the samples' losses), per-sample == batched-padded, batch permutation, and
the worked values of Eq. (11).
"""
from __future__ import annotations

import math

import numpy as np

NEG_INF = -np.inf


def _lse2(a: float, b: float) -> float:
    """ln(e^a + e^b) for scalars, either of which may be -inf."""
    if a == NEG_INF:
        return b
    if b == NEG_INF:
        return a
    m = a if a > b else b
    return m + math.log1p(math.exp(-abs(a - b)))


def joint(enc_b: np.ndarray, pred_b: np.ndarray) -> np.ndarray:
    """Step 1.  enc_b [T,H], pred_b [U+1,H] -> z [T,U+1,H]."""
    return np.tanh(enc_b[:, None, :] + pred_b[None, :, :])


def output_layer(z: np.ndarray, W_out: np.ndarray, b_out: np.ndarray) -> np.ndarray:
    """Step 2.  z [T,U+1,H] -> h [T,U+1,V]."""
    return z @ W_out + b_out


def log_softmax(h: np.ndarray):
    """Step 3.  Returns (lse [T,U+1], lp [T,U+1,V])."""
    m = np.max(h, axis=-1, keepdims=True)
    lse = m[..., 0] + np.log(np.sum(np.exp(h - m), axis=-1))
    return lse, h - lse[..., None]


def emissions(lp: np.ndarray, y: np.ndarray, blank: int):
    """Step 4.  lp [T,U+1,V], y [U] -> lpb [T,U+1], lpy [T,U] (column u is label y_u)."""
    U = lp.shape[1] - 1
    lpb = lp[:, :, blank]
    lpy = np.empty((lp.shape[0], U), dtype=lp.dtype)
    for u in range(U):
        lpy[:, u] = lp[:, u, y[u]]
    return lpb, lpy


def forward_variables(lpb: np.ndarray, lpy: np.ndarray) -> np.ndarray:
    """Step 5.  alpha [T,U+1]."""
    T, U1 = lpb.shape
    alpha = np.full((T, U1), NEG_INF, dtype=np.float64)
    alpha[0, 0] = 0.0
    for t in range(T):
        for u in range(U1):
            if t == 0 and u == 0:
                continue
            a = alpha[t - 1, u] + lpb[t - 1, u] if t > 0 else NEG_INF
            b = alpha[t, u - 1] + lpy[t, u - 1] if u > 0 else NEG_INF
            alpha[t, u] = _lse2(a, b)
    return alpha


def backward_variables(lpb: np.ndarray, lpy: np.ndarray) -> np.ndarray:
    """Step 6.  beta [T,U+1]."""
    T, U1 = lpb.shape
    U = U1 - 1
    beta = np.full((T, U1), NEG_INF, dtype=np.float64)
    beta[T - 1, U] = lpb[T - 1, U]
    for t in range(T - 1, -1, -1):
        for u in range(U, -1, -1):
            if t == T - 1 and u == U:
                continue
            a = beta[t + 1, u] + lpb[t, u] if t < T - 1 else NEG_INF
            b = beta[t, u + 1] + lpy[t, u] if u < U else NEG_INF
            beta[t, u] = _lse2(a, b)
    return beta


def occupations(alpha, beta, lpb, lpy, lnP):
    """Posterior weights of step 8: gamma [T,U+1], Bk [T,U+1], Yk [T,U]."""
    T, U1 = lpb.shape
    U = U1 - 1
    gamma = np.exp(alpha + beta - lnP)
    Bk = np.zeros((T, U1), dtype=np.float64)
    if T > 1:
        Bk[:T - 1, :] = np.exp(alpha[:T - 1, :] + lpb[:T - 1, :] + beta[1:, :] - lnP)
    Bk[T - 1, U] = math.exp(alpha[T - 1, U] + lpb[T - 1, U] - lnP)
    Yk = np.exp(alpha[:, :U] + lpy + beta[:, 1:] - lnP) if U > 0 else np.zeros((T, 0))
    return gamma, Bk, Yk


def dlogits(lp, alpha, beta, lpb, lpy, lnP, y, blank) -> np.ndarray:
    """Step 8.  dh [T,U+1,V] = d(-lnP)/dh."""
    U = lp.shape[1] - 1
    gamma, Bk, Yk = occupations(alpha, beta, lpb, lpy, lnP)
    dh = gamma[:, :, None] * np.exp(lp)
    dh[:, :, blank] -= Bk
    for u in range(U):
        dh[:, u, y[u]] -= Yk[:, u]
    return dh


def sample_loss_and_grads(enc_b, pred_b, W_out, b_out, y, blank, want_intermediates=False):
    """Steps 1-9 for one unpadded sample.  enc_b [T,H], pred_b [U+1,H], y [U]."""
    enc_b = np.asarray(enc_b, dtype=np.float64)
    pred_b = np.asarray(pred_b, dtype=np.float64)
    W_out = np.asarray(W_out, dtype=np.float64)
    b_out = np.asarray(b_out, dtype=np.float64)
    T, H = enc_b.shape
    U = pred_b.shape[0] - 1
    assert len(y) == U and T >= 1
    z = joint(enc_b, pred_b)
    h = output_layer(z, W_out, b_out)
    lse, lp = log_softmax(h)
    lpb, lpy = emissions(lp, y, blank)
    alpha = forward_variables(lpb, lpy)
    beta = backward_variables(lpb, lpy)
    lnP = alpha[T - 1, U] + lpb[T - 1, U]
    dh = dlogits(lp, alpha, beta, lpb, lpy, lnP, y, blank)
    dh2 = dh.reshape(T * (U + 1), -1)
    z2 = z.reshape(T * (U + 1), H)
    db = dh2.sum(axis=0)
    dW = z2.T @ dh2
    dz = (dh2 @ W_out.T).reshape(T, U + 1, H)
    dx = dz * (1.0 - z * z)
    out = dict(loss=-lnP, d_enc=dx.sum(axis=1), d_pred=dx.sum(axis=0), dW_out=dW, db_out=db)
    if want_intermediates:
        out.update(z=z, h=h, lse=lse, lp=lp, lpb=lpb, lpy=lpy, alpha=alpha, beta=beta,
                   lnP=lnP, dh=dh, beta00=beta[0, 0])
    return out


def rnnt_joint_loss(enc, pred, W_out, b_out, labels, T_len, U_len, blank, sample_weight=None):
    """Algorithm 1, lines 3-12, in float64: loop over samples, slice to the true lengths,
    accumulate the output-layer gradients, assign the encoding gradients.

    enc [B,T_max,H], pred [B,U_max+1,H], W_out [H,V], b_out [V], labels [B,U_max],
    T_len/U_len [B].  Entries outside a sample's lengths are never read.
    Returns loss [B], d_enc [B,T_max,H], d_pred [B,U_max+1,H], dW_out [H,V], db_out [V]
    (gradients of sum_b loss[b]; zeros in the padded rows of d_enc/d_pred).
    With sample_weight [B] the gradients are those of sum_b sample_weight[b] * loss[b] (the
    criterion of Section 2 is a sum over the samples, so each sample's gradients are scaled by
    its weight before they are accumulated or assigned); loss[b] itself stays -ln P(y_b|x_b).
    """
    enc = np.asarray(enc)
    pred = np.asarray(pred)
    B, T_max, H = enc.shape
    V = np.asarray(W_out).shape[1]
    loss = np.zeros(B, dtype=np.float64)
    d_enc = np.zeros((B, T_max, H), dtype=np.float64)
    d_pred = np.zeros((B, pred.shape[1], H), dtype=np.float64)
    dW = np.zeros((H, V), dtype=np.float64)
    db = np.zeros(V, dtype=np.float64)
    for b in range(B):
        T, U = int(T_len[b]), int(U_len[b])
        r = sample_loss_and_grads(enc[b, :T], pred[b, :U + 1], W_out, b_out,
                                  np.asarray(labels[b, :U]), blank)
        w = 1.0 if sample_weight is None else float(sample_weight[b])
        loss[b] = r["loss"]
        d_enc[b, :T] = w * r["d_enc"]
        d_pred[b, :U + 1] = w * r["d_pred"]
        dW += w * r["dW_out"]
        db += w * r["db_out"]
    return dict(loss=loss, d_enc=d_enc, d_pred=d_pred, dW_out=dW, db_out=db)


def rnnt_joint_loss_batched_padded(enc, pred, W_out, b_out, labels, T_len, U_len, blank):
    """The "batched" form that Algorithm 1 is stated to equal: the whole [B,T_max,U_max+1,V]
    score tensor at once, lattices masked by the lengths.  Filler in the padding must be
    finite here (the 4-D tensor is really formed); tiny shapes only."""
    enc = np.asarray(enc, dtype=np.float64)
    pred = np.asarray(pred, dtype=np.float64)
    W_out = np.asarray(W_out, dtype=np.float64)
    b_out = np.asarray(b_out, dtype=np.float64)
    B, T_max, H = enc.shape
    U1_max = pred.shape[1]
    z = np.tanh(enc[:, :, None, :] + pred[:, None, :, :])           # [B,T,U+1,H]
    h = z @ W_out + b_out                                            # [B,T,U+1,V]
    m = h.max(axis=-1, keepdims=True)
    lp = h - (m + np.log(np.exp(h - m).sum(axis=-1, keepdims=True)))
    dh = np.zeros_like(h)
    loss = np.zeros(B)
    for b in range(B):
        T, U = int(T_len[b]), int(U_len[b])
        y = np.asarray(labels[b, :U])
        lpb, lpy = emissions(lp[b, :T, :U + 1], y, blank)
        alpha = forward_variables(lpb, lpy)
        beta = backward_variables(lpb, lpy)
        lnP = alpha[T - 1, U] + lpb[T - 1, U]
        loss[b] = -lnP
        dh[b, :T, :U + 1] = dlogits(lp[b, :T, :U + 1], alpha, beta, lpb, lpy, lnP, y, blank)
    dh2 = dh.reshape(-1, dh.shape[-1])
    dW = z.reshape(-1, H).T @ dh2
    db = dh2.sum(axis=0)
    dx = (dh @ W_out.T) * (1.0 - z * z)
    return dict(loss=loss, d_enc=dx.sum(axis=2), d_pred=dx.sum(axis=1), dW_out=dW, db_out=db)


def input_projections(hA_b, hL_b, W_A, b_Z, W_L):
    """The two linear maps inside the tanh of Eq. (4) for one unpadded sample:
    enc[t,:] = hA[t,:] @ W_A + b_Z,  pred[u,:] = hL[u,:] @ W_L.
    hA_b [T,H_A], hL_b [U+1,H_L], W_A [H_A,H], b_Z [H], W_L [H_L,H] (the paper writes the
    matrices as H x H_A and H x H_L; here the joint dimension H is the contiguous one)."""
    hA_b = np.asarray(hA_b, dtype=np.float64)
    hL_b = np.asarray(hL_b, dtype=np.float64)
    W_A = np.asarray(W_A, dtype=np.float64)
    W_L = np.asarray(W_L, dtype=np.float64)
    b_Z = np.asarray(b_Z, dtype=np.float64)
    return hA_b @ W_A + b_Z, hL_b @ W_L


def sample_proj_loss_and_grads(hA_b, hL_b, W_A, b_Z, W_L, W_out, b_out, y, blank):
    """Eq. (4) in full (projections inside the tanh) followed by steps 1-9, and the chain rule
    back through the projections (Algorithm 1 line 9 for theta^J, lines 10-11 for the encodings)."""
    enc_b, pred_b = input_projections(hA_b, hL_b, W_A, b_Z, W_L)
    r = sample_loss_and_grads(enc_b, pred_b, W_out, b_out, y, blank)
    hA_b = np.asarray(hA_b, dtype=np.float64)
    hL_b = np.asarray(hL_b, dtype=np.float64)
    W_A = np.asarray(W_A, dtype=np.float64)
    W_L = np.asarray(W_L, dtype=np.float64)
    return dict(loss=r["loss"], dW_out=r["dW_out"], db_out=r["db_out"],
                d_hA=r["d_enc"] @ W_A.T, d_hL=r["d_pred"] @ W_L.T,
                dW_A=hA_b.T @ r["d_enc"], dW_L=hL_b.T @ r["d_pred"], db_Z=r["d_enc"].sum(axis=0),
                d_enc=r["d_enc"], d_pred=r["d_pred"])


def rnnt_joint_proj_loss(hA, hL, W_A, b_Z, W_L, W_out, b_out, labels, T_len, U_len, blank):
    """Algorithm 1, lines 3-12, with the joint network of Eq. (4) complete: loop over samples,
    slice to the true lengths, accumulate all parameter gradients, assign the encoding gradients.
    hA [B,T_max,H_A], hL [B,U_max+1,H_L]; returns loss [B], d_hA, d_hL (zeros in the padding),
    dW_A, db_Z, dW_L, dW_out, db_out (gradients of sum_b loss[b])."""
    hA = np.asarray(hA)
    hL = np.asarray(hL)
    B = hA.shape[0]
    out = dict(loss=np.zeros(B), d_hA=np.zeros(hA.shape), d_hL=np.zeros(hL.shape),
               dW_A=np.zeros(np.asarray(W_A).shape), db_Z=np.zeros(np.asarray(b_Z).shape),
               dW_L=np.zeros(np.asarray(W_L).shape), dW_out=np.zeros(np.asarray(W_out).shape),
               db_out=np.zeros(np.asarray(b_out).shape))
    for b in range(B):
        T, U = int(T_len[b]), int(U_len[b])
        r = sample_proj_loss_and_grads(hA[b, :T], hL[b, :U + 1], W_A, b_Z, W_L, W_out, b_out,
                                       np.asarray(labels[b, :U]), blank)
        out["loss"][b] = r["loss"]
        out["d_hA"][b, :T] = r["d_hA"]
        out["d_hL"][b, :U + 1] = r["d_hL"]
        for k in ("dW_A", "db_Z", "dW_L", "dW_out", "db_out"):
            out[k] += r[k]
    return out


def parallel_iterations(T: int, U: int, V: int) -> int:
    """Eq. (11): number of sample iterations run concurrently under the paper's dynamic
    parallelism, PI = 2^max(0, min(4, floor(log2(1e9 / (4 T U V)))))."""
    return 2 ** max(0, min(4, math.floor(math.log(1e9 / (4.0 * T * U * V)) / math.log(2.0))))
