"""Pins of the float64 checker against things that do not depend on it: exhaustive
enumeration of alignments, closed forms, identities of the transducer lattice, finite
differences, the batched form of Algorithm 1, and the worked values of Eq. (11)."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import rnnt_oracle as O

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rand_problem(rng, B, T_max, U_max, H, V, full=False, blank=0, scale=1.0):
    enc = rng.standard_normal((B, T_max, H))
    pred = rng.standard_normal((B, U_max + 1, H))
    W = rng.standard_normal((H, V)) * scale / math.sqrt(H)
    b = rng.standard_normal(V) * 0.3
    labels = rng.integers(0, V, size=(B, U_max))
    if full:
        T_len = np.full(B, T_max)
        U_len = np.full(B, U_max)
    else:
        T_len = rng.integers(1, T_max + 1, size=B)
        U_len = rng.integers(0, U_max + 1, size=B)
    return enc, pred, W, b, labels, T_len, U_len, blank


def brute_force_neg_log_likelihood(P, y, blank):
    """-ln of the total probability of all alignments, in the linear domain.
    P [T,U+1,V] are probabilities.  An alignment is a monotone walk from (0,0) to (T-1,U):
    a blank moves t -> t+1, label y_u moves u -> u+1; it ends with one blank at (T-1,U)."""
    T, U1, _ = P.shape
    U = U1 - 1
    total = 0.0
    n_moves = T - 1 + U
    for label_slots in itertools.combinations(range(n_moves), U):
        slots = set(label_slots)
        t = u = 0
        p = 1.0
        for s in range(n_moves):
            if s in slots:
                p *= P[t, u, y[u]]
                u += 1
            else:
                p *= P[t, u, blank]
                t += 1
        assert (t, u) == (T - 1, U)
        total += p * P[T - 1, U, blank]
    return -math.log(total)


def _loss_from_scores(h, y, blank):
    lse, lp = O.log_softmax(h)
    lpb, lpy = O.emissions(lp, y, blank)
    alpha = O.forward_variables(lpb, lpy)
    return -(alpha[-1, -1] + lpb[-1, -1])


# ---------------------------------------------------------------- loss: enumeration
@pytest.mark.parametrize("T,U,V,blank", [
    (1, 0, 3, 0), (1, 3, 4, 0), (3, 0, 4, 1), (4, 3, 5, 0), (5, 2, 4, 2), (2, 5, 3, 1),
    (6, 6, 4, 3), (6, 1, 7, 0), (3, 4, 2, 0),
])
def test_loss_equals_enumeration_of_all_alignments(T, U, V, blank):
    rng = np.random.default_rng(1000 + 17 * T + 5 * U + V)
    h = rng.standard_normal((T, U + 1, V)) * 1.7
    y = rng.integers(0, V, size=U)
    if U >= 2:
        y[1] = blank          # a label equal to the blank index is legal
    P = np.exp(h) / np.exp(h).sum(-1, keepdims=True)
    ref = brute_force_neg_log_likelihood(P, y, blank)
    got = _loss_from_scores(h, y, blank)
    assert abs(got - ref) < 1e-12 * max(1.0, abs(ref))
    # the backward variables give the same likelihood
    lse, lp = O.log_softmax(h)
    lpb, lpy = O.emissions(lp, y, blank)
    beta = O.backward_variables(lpb, lpy)
    assert abs(-beta[0, 0] - ref) < 1e-12 * max(1.0, abs(ref))


def test_full_pipeline_loss_equals_enumeration_on_smallest_workload_shape():
    # the shape of the smallest workload (T=20, U=5, H=32, V=16): 42 504 alignments
    rng = np.random.default_rng(7)
    T, U, H, V = 20, 5, 32, 16
    enc = rng.standard_normal((T, H))
    pred = rng.standard_normal((U + 1, H))
    W = rng.standard_normal((H, V)) / math.sqrt(H)
    b = np.zeros(V)
    y = rng.integers(1, V, size=U)
    r = O.sample_loss_and_grads(enc, pred, W, b, y, 0, want_intermediates=True)
    # scores written out independently of the checker's helpers
    h = np.empty((T, U + 1, V))
    for t in range(T):
        for u in range(U + 1):
            h[t, u] = np.tanh(enc[t] + pred[u]) @ W + b
    P = np.exp(h) / np.exp(h).sum(-1, keepdims=True)
    ref = brute_force_neg_log_likelihood(P, y, 0)
    assert abs(r["loss"] - ref) < 1e-11 * abs(ref)
    assert abs(-r["beta00"] - ref) < 1e-11 * abs(ref)


# ---------------------------------------------------------------- loss: closed forms
def test_single_cell_lattice_is_minus_log_p_blank():
    rng = np.random.default_rng(3)
    H, V, blank = 5, 7, 2
    enc = rng.standard_normal((1, H))
    pred = rng.standard_normal((1, H))
    W = rng.standard_normal((H, V))
    b = rng.standard_normal(V)
    r = O.sample_loss_and_grads(enc, pred, W, b, np.zeros(0, dtype=int), blank)
    h = np.tanh(enc[0] + pred[0]) @ W + b
    p = np.exp(h) / np.exp(h).sum()
    assert abs(r["loss"] + math.log(p[blank])) < 1e-13


def test_no_labels_is_sum_of_blank_log_probs():
    rng = np.random.default_rng(4)
    T, V, blank = 9, 6, 0
    h = rng.standard_normal((T, 1, V))
    P = np.exp(h) / np.exp(h).sum(-1, keepdims=True)
    ref = -sum(math.log(P[t, 0, blank]) for t in range(T))
    assert abs(_loss_from_scores(h, np.zeros(0, dtype=int), blank) - ref) < 1e-12


def test_single_frame_is_labels_then_blank():
    rng = np.random.default_rng(5)
    U, V, blank = 6, 5, 4
    h = rng.standard_normal((1, U + 1, V))
    y = rng.integers(0, V, size=U)
    P = np.exp(h) / np.exp(h).sum(-1, keepdims=True)
    ref = -sum(math.log(P[0, u, y[u]]) for u in range(U)) - math.log(P[0, U, blank])
    assert abs(_loss_from_scores(h, y, blank) - ref) < 1e-12


def _closed_form_rows():
    rows = []
    with open(os.path.join(GOLD, "uniform_scores_closed_form.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            T, U, V, val = line.split()
            rows.append((int(T), int(U), int(V), float(val)))
    return rows


@pytest.mark.parametrize("T,U,V,val", _closed_form_rows())
def test_uniform_scores_closed_form(T, U, V, val):
    # all scores equal -> loss = (T+U) ln V - ln C(T+U-1, U); checks the recursion at full size
    lpb = np.full((T, U + 1), -math.log(V))
    lpy = np.full((T, U), -math.log(V))
    alpha = O.forward_variables(lpb, lpy)
    beta = O.backward_variables(lpb, lpy)
    assert abs(-(alpha[-1, -1] + lpb[-1, -1]) - val) < 1e-10 * val
    assert abs(-beta[0, 0] - val) < 1e-10 * val


def test_uniform_scores_through_the_whole_pipeline():
    T, U, H, V = 20, 5, 32, 16
    rng = np.random.default_rng(6)
    r = O.sample_loss_and_grads(rng.standard_normal((T, H)), rng.standard_normal((U + 1, H)),
                                np.zeros((H, V)), np.zeros(V), rng.integers(1, V, size=U), 0)
    assert abs(r["loss"] - 58.657364587863752) < 1e-11
    assert np.abs(r["d_enc"]).max() == 0.0 and np.abs(r["d_pred"]).max() == 0.0  # W_out = 0


# ---------------------------------------------------------------- lattice identities
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_occupation_identities(seed):
    rng = np.random.default_rng(20 + seed)
    T, U, V, blank = 7 + seed, 4 + seed, 6, 1
    h = rng.standard_normal((T, U + 1, V)) * 2.0
    y = rng.integers(0, V, size=U)
    lse, lp = O.log_softmax(h)
    lpb, lpy = O.emissions(lp, y, blank)
    alpha = O.forward_variables(lpb, lpy)
    beta = O.backward_variables(lpb, lpy)
    lnP = alpha[-1, -1] + lpb[-1, -1]
    assert abs(lnP - beta[0, 0]) < 1e-12
    gamma, Bk, Yk = O.occupations(alpha, beta, lpb, lpy, lnP)
    # every alignment emits exactly one blank per frame and every label exactly once
    np.testing.assert_allclose(Bk.sum(axis=1), np.ones(T), atol=1e-12)
    np.testing.assert_allclose(Yk.sum(axis=0), np.ones(U), atol=1e-12)
    # a visited node is left by exactly one emission
    np.testing.assert_allclose(gamma[:, :U], Bk[:, :U] + Yk, atol=1e-12)
    np.testing.assert_allclose(gamma[:, U], Bk[:, U], atol=1e-12)
    assert abs(gamma.sum() - (T + U)) < 1e-11
    assert abs(gamma[0, 0] - 1.0) < 1e-12 and abs(gamma[-1, -1] - 1.0) < 1e-12
    dh = O.dlogits(lp, alpha, beta, lpb, lpy, lnP, y, blank)
    assert np.abs(dh.sum(axis=-1)).max() < 1e-12        # softmax shift invariance at every (t,u)


# ---------------------------------------------------------------- gradients: finite differences
def test_dlogits_matches_finite_differences_of_the_loss():
    rng = np.random.default_rng(31)
    T, U, V, blank = 4, 3, 5, 2
    h = rng.standard_normal((T, U + 1, V))
    y = np.array([1, blank, 4])
    lse, lp = O.log_softmax(h)
    lpb, lpy = O.emissions(lp, y, blank)
    alpha = O.forward_variables(lpb, lpy)
    beta = O.backward_variables(lpb, lpy)
    lnP = alpha[-1, -1] + lpb[-1, -1]
    dh = O.dlogits(lp, alpha, beta, lpb, lpy, lnP, y, blank)
    eps = 1e-6
    for idx in np.ndindex(*h.shape):
        hp = h.copy(); hp[idx] += eps
        hm = h.copy(); hm[idx] -= eps
        fd = (_loss_from_scores(hp, y, blank) - _loss_from_scores(hm, y, blank)) / (2 * eps)
        assert abs(fd - dh[idx]) < 2e-8, (idx, fd, dh[idx])


def _total_loss(enc, pred, W, b, labels, T_len, U_len, blank):
    return O.rnnt_joint_loss(enc, pred, W, b, labels, T_len, U_len, blank)["loss"].sum()


def test_all_gradients_match_finite_differences_through_the_whole_chain():
    rng = np.random.default_rng(32)
    args = list(_rand_problem(rng, B=3, T_max=5, U_max=3, H=4, V=5, blank=1))
    args[5][:] = [5, 3, 1]
    args[6][:] = [3, 0, 2]
    g = O.rnnt_joint_loss(*args)
    eps = 1e-6
    for name, pos in (("d_enc", 0), ("d_pred", 1), ("dW_out", 2), ("db_out", 3)):
        x = args[pos]
        fd = np.zeros_like(x)
        for idx in np.ndindex(*x.shape):
            old = x[idx]
            x[idx] = old + eps
            lp_ = _total_loss(*args)
            x[idx] = old - eps
            lm_ = _total_loss(*args)
            x[idx] = old
            fd[idx] = (lp_ - lm_) / (2 * eps)
        np.testing.assert_allclose(g[name], fd, atol=5e-8, err_msg=name)
    assert abs(g["db_out"].sum()) < 1e-12


def test_padding_is_never_read_and_gets_zero_gradient():
    rng = np.random.default_rng(33)
    enc, pred, W, b, labels, T_len, U_len, blank = _rand_problem(rng, 3, 6, 4, 5, 6)
    T_len[:] = [6, 2, 4]; U_len[:] = [1, 4, 0]
    ref = O.rnnt_joint_loss(enc, pred, W, b, labels, T_len, U_len, blank)
    enc2, pred2, lab2 = enc.copy(), pred.copy(), labels.copy()
    for i in range(3):
        enc2[i, T_len[i]:] = np.nan
        pred2[i, U_len[i] + 1:] = np.nan
        lab2[i, U_len[i]:] = -7
    got = O.rnnt_joint_loss(enc2, pred2, W, b, lab2, T_len, U_len, blank)
    for k in ref:
        np.testing.assert_array_equal(ref[k], got[k])
    for i in range(3):
        assert np.all(got["d_enc"][i, T_len[i]:] == 0) and np.all(got["d_pred"][i, U_len[i] + 1:] == 0)


# ---------------------------------------------------------------- Algorithm 1 == batched
def test_sample_wise_accumulation_equals_batched_padded():
    rng = np.random.default_rng(41)
    args = _rand_problem(rng, B=4, T_max=6, U_max=4, H=5, V=7, blank=0)
    a = O.rnnt_joint_loss(*args)
    b = O.rnnt_joint_loss_batched_padded(*args)
    for k in a:
        np.testing.assert_allclose(a[k], b[k], rtol=0, atol=1e-12, err_msg=k)


def test_batch_permutation_and_additivity():
    rng = np.random.default_rng(42)
    enc, pred, W, b, labels, T_len, U_len, blank = _rand_problem(rng, 4, 6, 4, 5, 7)
    full = O.rnnt_joint_loss(enc, pred, W, b, labels, T_len, U_len, blank)
    perm = np.array([2, 0, 3, 1])
    p = O.rnnt_joint_loss(enc[perm], pred[perm], W, b, labels[perm], T_len[perm], U_len[perm], blank)
    np.testing.assert_allclose(p["loss"], full["loss"][perm], atol=1e-13)
    np.testing.assert_allclose(p["d_enc"], full["d_enc"][perm], atol=1e-13)
    np.testing.assert_allclose(p["dW_out"], full["dW_out"], atol=1e-12)
    dW = np.zeros_like(W)
    for i in range(4):
        s = slice(i, i + 1)
        dW += O.rnnt_joint_loss(enc[s], pred[s], W, b, labels[s], T_len[s], U_len[s], blank)["dW_out"]
    np.testing.assert_allclose(dW, full["dW_out"], atol=1e-12)


def test_weighted_gradients_match_finite_differences_of_the_weighted_sum():
    # gradients of sum_b w_b loss_b (Section 2: the criterion is a sum over the samples); a weight of
    # zero removes a sample, unit weights give the unweighted call, the losses themselves do not change
    rng = np.random.default_rng(43)
    args = list(_rand_problem(rng, B=3, T_max=5, U_max=3, H=4, V=5, blank=1))
    args[5][:] = [5, 2, 4]
    args[6][:] = [3, 1, 0]
    w = np.array([0.25, 0.0, 1.75])
    g = O.rnnt_joint_loss(*args, sample_weight=w)
    plain = O.rnnt_joint_loss(*args)
    np.testing.assert_array_equal(g["loss"], plain["loss"])
    ones = O.rnnt_joint_loss(*args, sample_weight=np.ones(3))
    for k in plain:
        np.testing.assert_array_equal(ones[k], plain[k])
    assert np.all(g["d_enc"][1] == 0) and np.all(g["d_pred"][1] == 0)
    eps = 1e-6

    def weighted_total():
        return float(np.dot(w, O.rnnt_joint_loss(*args)["loss"]))

    for name, pos in (("d_enc", 0), ("d_pred", 1), ("dW_out", 2), ("db_out", 3)):
        x = args[pos]
        fd = np.zeros_like(x)
        for idx in np.ndindex(*x.shape):
            old = x[idx]
            x[idx] = old + eps
            lp_ = weighted_total()
            x[idx] = old - eps
            lm_ = weighted_total()
            x[idx] = old
            fd[idx] = (lp_ - lm_) / (2 * eps)
        np.testing.assert_allclose(g[name], fd, atol=5e-8, err_msg=name)


# ---------------------------------------------------------------- Eq. (11)
def test_parallel_iterations_worked_values():
    with open(os.path.join(GOLD, "eq11_parallel_iterations.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for T, U, V, fl, pi in rows:
        assert O.parallel_iterations(int(T), int(U), int(V)) == int(pi)
        assert int(pi) == 2 ** max(0, min(4, int(fl)))
    # range 1..16 as stated with the formula
    assert O.parallel_iterations(10, 2, 4096) == 16 and O.parallel_iterations(2000, 400, 4096) == 1


# ---------------------------------------------------------------- the pins do bite
@pytest.mark.parametrize("mistake", ["label_index", "blank_term_sign", "beta_uses_wrong_emission",
                                     "transposed_W", "alpha_moves_swapped"])
def test_planted_mistakes_are_caught(monkeypatch, mistake):
    """Each plausible slip, planted into a copy of the checker's step, must break a pin."""
    rng = np.random.default_rng(50)
    if mistake == "label_index":
        def bad(lp, y, blank):
            lpb, lpy = orig(lp, y, blank)
            return lpb, lpy[:, ::-1]
        orig = O.emissions
        monkeypatch.setattr(O, "emissions", bad)
        h = rng.standard_normal((4, 4, 5)); y = np.array([1, 2, 3])
        P = np.exp(h) / np.exp(h).sum(-1, keepdims=True)
        assert abs(_loss_from_scores(h, y, 0) - brute_force_neg_log_likelihood(P, y, 0)) > 1e-3
    elif mistake == "blank_term_sign":
        orig = O.occupations
        monkeypatch.setattr(O, "occupations", lambda *a: tuple(x * s for x, s in zip(orig(*a), (1, -1, 1))))
        h = rng.standard_normal((4, 4, 5)); y = np.array([1, 2, 3])
        lse, lp = O.log_softmax(h); lpb, lpy = O.emissions(lp, y, 0)
        al, be = O.forward_variables(lpb, lpy), O.backward_variables(lpb, lpy)
        dh = O.dlogits(lp, al, be, lpb, lpy, al[-1, -1] + lpb[-1, -1], y, 0)
        assert np.abs(dh.sum(-1)).max() > 1e-3
    elif mistake == "beta_uses_wrong_emission":
        orig = O.backward_variables
        monkeypatch.setattr(O, "backward_variables", lambda lpb, lpy: orig(np.roll(lpb, 1, axis=0), lpy))
        h = rng.standard_normal((5, 3, 4)); y = np.array([1, 2])
        lse, lp = O.log_softmax(h); lpb, lpy = O.emissions(lp, y, 0)
        al, be = O.forward_variables(lpb, lpy), O.backward_variables(lpb, lpy)
        assert abs(al[-1, -1] + lpb[-1, -1] - be[0, 0]) > 1e-3
    elif mistake == "transposed_W":
        monkeypatch.setattr(O, "output_layer", lambda z, W, b: z @ W.T + b)
        H = V = 4
        enc = rng.standard_normal((2, H)); pred = rng.standard_normal((2, H))
        W = rng.standard_normal((H, V)); b = np.zeros(V); y = np.array([1])
        r = O.sample_loss_and_grads(enc, pred, W, b, y, 0)
        h = np.tanh(enc[:, None] + pred[None]) @ W
        P = np.exp(h) / np.exp(h).sum(-1, keepdims=True)
        assert abs(r["loss"] - brute_force_neg_log_likelihood(P, y, 0)) > 1e-3
    else:
        orig = O.forward_variables
        # forward variables that charge the blank move with the label emission and vice versa
        monkeypatch.setattr(O, "forward_variables",
                            lambda lpb, lpy: orig(np.pad(lpy, ((0, 0), (0, 1))), lpb[:, :-1]))
        h = rng.standard_normal((4, 3, 5)); y = np.array([1, 2])
        P = np.exp(h) / np.exp(h).sum(-1, keepdims=True)
        assert abs(_loss_from_scores(h, y, 0) - brute_force_neg_log_likelihood(P, y, 0)) > 1e-3


# ---------------------------------------------------------------- Eq. 4 with its projections
def _rand_proj_problem(rng, B, T_max, U_max, DA, DL, H, V, blank=0):
    hA = rng.standard_normal((B, T_max, DA))
    hL = rng.standard_normal((B, U_max + 1, DL))
    W_A = rng.standard_normal((DA, H)) / math.sqrt(DA)
    b_Z = rng.standard_normal(H) * 0.2
    W_L = rng.standard_normal((DL, H)) / math.sqrt(DL)
    W = rng.standard_normal((H, V)) / math.sqrt(H)
    b = rng.standard_normal(V) * 0.3
    labels = rng.integers(0, V, size=(B, U_max))
    T_len = rng.integers(1, T_max + 1, size=B)
    U_len = rng.integers(0, U_max + 1, size=B)
    return [hA, hL, W_A, b_Z, W_L, W, b, labels, T_len, U_len, blank]


def test_projected_chain_matches_finite_differences():
    rng = np.random.default_rng(71)
    args = _rand_proj_problem(rng, B=3, T_max=4, U_max=3, DA=3, DL=2, H=4, V=5, blank=2)
    args[8][:] = [4, 2, 1]
    args[9][:] = [3, 0, 2]
    g = O.rnnt_joint_proj_loss(*args)
    eps = 1e-6
    for name, pos in (("d_hA", 0), ("d_hL", 1), ("dW_A", 2), ("db_Z", 3), ("dW_L", 4), ("dW_out", 5), ("db_out", 6)):
        x = args[pos]
        fd = np.zeros_like(x)
        for idx in np.ndindex(*x.shape):
            old = x[idx]
            x[idx] = old + eps
            lp_ = O.rnnt_joint_proj_loss(*args)["loss"].sum()
            x[idx] = old - eps
            lm_ = O.rnnt_joint_proj_loss(*args)["loss"].sum()
            x[idx] = old
            fd[idx] = (lp_ - lm_) / (2 * eps)
        np.testing.assert_allclose(g[name], fd, atol=1e-7, err_msg=name)
    # padded rows of the encodings get exactly zero
    for i in range(3):
        assert np.all(g["d_hA"][i, args[8][i]:] == 0) and np.all(g["d_hL"][i, args[9][i] + 1:] == 0)


def test_identity_projections_reduce_to_the_unprojected_path():
    rng = np.random.default_rng(72)
    enc, pred, W, b, labels, T_len, U_len, blank = _rand_problem(rng, 3, 5, 4, 6, 7)
    eye = np.eye(6)
    ref = O.rnnt_joint_loss(enc, pred, W, b, labels, T_len, U_len, blank)
    got = O.rnnt_joint_proj_loss(enc, pred, eye, np.zeros(6), eye, W, b, labels, T_len, U_len, blank)
    np.testing.assert_allclose(got["loss"], ref["loss"], rtol=1e-14)
    np.testing.assert_allclose(got["d_hA"], ref["d_enc"], atol=1e-15)
    np.testing.assert_allclose(got["d_hL"], ref["d_pred"], atol=1e-15)
    np.testing.assert_allclose(got["dW_out"], ref["dW_out"], atol=1e-14)
    # with identity maps dW_A = sum_b enc_b^T d_enc_b and the bias gradient is the sum of the rows
    dWA = sum(enc[i, :T_len[i]].T @ ref["d_enc"][i, :T_len[i]] for i in range(3))
    np.testing.assert_allclose(got["dW_A"], dWA, atol=1e-13)
    np.testing.assert_allclose(got["db_Z"], ref["d_enc"].sum(axis=(0, 1)), atol=1e-13)


def test_bias_gradient_is_the_same_from_either_encoding():
    # b^Z enters every lattice node once: its gradient is sum_{t,u} dx = sum_t d_enc[t] = sum_u d_pred[u]
    rng = np.random.default_rng(73)
    enc, pred, W, b, labels, T_len, U_len, blank = _rand_problem(rng, 4, 6, 5, 5, 6)
    r = O.rnnt_joint_loss(enc, pred, W, b, labels, T_len, U_len, blank)
    np.testing.assert_allclose(r["d_enc"].sum(axis=1), r["d_pred"].sum(axis=1), atol=1e-13)


@pytest.mark.parametrize("mistake", ["bias_on_both", "transposed_grad", "dropped_bias"])
def test_planted_projection_mistakes_are_caught(monkeypatch, mistake):
    rng = np.random.default_rng(74)
    args = _rand_proj_problem(rng, B=2, T_max=3, U_max=2, DA=3, DL=3, H=3, V=4)
    args[8][:] = [3, 2]
    args[9][:] = [2, 1]
    good = O.rnnt_joint_proj_loss(*args)
    orig = O.input_projections
    if mistake == "bias_on_both":
        monkeypatch.setattr(O, "input_projections", lambda a, l, WA, bZ, WL: (orig(a, l, WA, bZ, WL)[0], orig(a, l, WA, bZ, WL)[1] + bZ))
    elif mistake == "dropped_bias":
        monkeypatch.setattr(O, "input_projections", lambda a, l, WA, bZ, WL: orig(a, l, WA, 0 * np.asarray(bZ), WL))
    else:
        monkeypatch.setattr(O, "input_projections", lambda a, l, WA, bZ, WL: orig(a, l, np.asarray(WA).T.copy() if np.asarray(WA).shape[0] == np.asarray(WA).shape[1] else WA, bZ, WL))
    bad = O.rnnt_joint_proj_loss(*args)
    # the pins above would fail: the loss moves, or the analytic gradient no longer matches the function
    eps = 1e-6
    x = args[3]
    fd = np.zeros_like(x)
    for i in range(x.size):
        old = x[i]
        x[i] = old + eps
        lp_ = O.rnnt_joint_proj_loss(*args)["loss"].sum()
        x[i] = old - eps
        lm_ = O.rnnt_joint_proj_loss(*args)["loss"].sum()
        x[i] = old
        fd[i] = (lp_ - lm_) / (2 * eps)
    moved = not np.allclose(bad["loss"], good["loss"], rtol=1e-9)
    broken_grad = not np.allclose(bad["db_Z"], fd, atol=1e-6)
    assert moved or broken_grad
