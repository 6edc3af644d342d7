"""CPU-only tests of the C-ABI library: it loads, exports what the header declares, rejects bad
arguments before touching a GPU, and its scheduler packs samples as promised."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2211_16270_amd import binding as Bd
from paper_2211_16270_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "rnnt_joint_loss.h")
HEADERS = [HEADER, os.path.join(ROOT, "include", "rnnt_joint_loss_debug.h")]
GOLD = os.path.join(ROOT, "tests", "golden")


def test_library_exports_every_declared_symbol():
    text = "".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(rnnt_[a-z_0-9]+)\s*\(", text))
    assert declared == set(Bd.EXPORTS), declared ^ set(Bd.EXPORTS)
    L = Bd.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert L.rnnt_status_string(0) == b"ok"
    for code in range(1, 8):
        assert len(L.rnnt_status_string(code)) > 3


def test_no_hip_error_is_reported_before_one_happened():
    assert Bd.lib().rnnt_last_hip_error() == b""
    assert Bd.lib().rnnt_debug_mfma_loop(None, None, 1, 1, None) == 1   # null pointers are refused on the host
    assert Bd.lib().rnnt_debug_mfma_loop(ctypes.c_void_p(256), ctypes.c_void_p(256), 0, 1, None) == 2
    assert Bd.lib().rnnt_debug_mfma_loop(ctypes.c_void_p(256), ctypes.c_void_p(256), 1, 2000000, None) == 2
    assert Bd.lib().rnnt_debug_mfma_loop_fp8(None, None, 1, 1, None) == 1
    assert Bd.lib().rnnt_debug_mfma_loop_fp8(ctypes.c_void_p(256), ctypes.c_void_p(256), 1, 0, None) == 2


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(Bd.RnntDesc) == 44
    assert ctypes.sizeof(Bd.RnntPlanInfo) == 8 * 3 + 4 * 2 + 8 * 2 + 8 * 3


def _tiles(T, U):
    """64-row lattice tiles per sample: 8 frames x 8 label positions, or 16 x 4 where that needs 3 % fewer."""
    T, U = np.asarray(T, dtype=np.int64), np.asarray(U, dtype=np.int64)
    a, b = ((T + 7) // 8) * ((U + 8) // 8), ((T + 15) // 16) * ((U + 4) // 4)
    return np.where(b * 33 < a * 32, b, a)


def _lens(name):
    wl = synth.WORKLOADS[name]
    T, U, _ = synth.draw_lengths_labels(wl)
    dt = Bd.RNNT_BF16 if wl.dtype == "bf16" else Bd.RNNT_F32
    return wl, Bd.make_desc(wl.B, wl.T_max, wl.U_max, wl.H, wl.V, 0, dt), T, U


def test_argument_checks_happen_on_the_host():
    wl, desc, T, U = _lens("C2")
    L = Bd.lib()
    dummy = ctypes.c_void_p(0x1000)

    def call(d, Tl, Ul, ws=dummy, ws_bytes=1 << 30, enc=dummy):
        Tl = np.ascontiguousarray(Tl, dtype=np.int32)
        Ul = np.ascontiguousarray(Ul, dtype=np.int32)
        return L.rnnt_joint_loss_fwd_bwd(ctypes.byref(d), enc, dummy, dummy, dummy, dummy, Bd._ip(Tl), Bd._ip(Ul),
                                         dummy, dummy, dummy, dummy, dummy, ws, ws_bytes, None)

    assert call(desc, T, U, enc=None) == 1                       # RNNT_ERR_NULL
    bad = Bd.make_desc(wl.B, wl.T_max, wl.U_max, wl.H, wl.V, wl.V, Bd.RNNT_BF16)
    assert call(bad, T, U) == 2                                  # blank out of range
    T2 = T.copy(); T2[3] = wl.T_max + 1
    assert call(desc, T2, U) == 3
    T2[3] = 0
    assert call(desc, T2, U) == 3
    U2 = U.copy(); U2[0] = -1
    assert call(desc, T, U2) == 3
    assert call(desc, T, U, ws=None) == 5
    assert call(desc, T, U, ws=ctypes.c_void_p(0x1010)) == 5     # misaligned
    assert call(desc, T, U, ws_bytes=4096) == 5                  # too small
    odd = Bd.make_desc(wl.B, wl.T_max, wl.U_max, 500, wl.V, 0, Bd.RNNT_BF16)
    assert call(odd, T, U) == 6                                  # H not supported by the MFMA path
    assert call(desc, T, U, enc=ctypes.c_void_p(0x1004)) == 6    # the kernels need 16-byte aligned arrays
    assert Bd.rnnt_joint_loss_workspace_bytes(bad, T, U) == 0


def test_sample_weights_are_checked_on_the_host():
    wl, desc, T, U = _lens("C2")
    L = Bd.lib()
    dummy = ctypes.c_void_p(0x1000)

    def call(w, ws=dummy):
        w = None if w is None else np.ascontiguousarray(w, dtype=np.float32)
        wp = None if w is None else w.ctypes.data_as(ctypes.POINTER(ctypes.c_float))
        return L.rnnt_joint_loss_fwd_bwd_weighted(ctypes.byref(desc), dummy, dummy, dummy, dummy, dummy, Bd._ip(T),
                                                  Bd._ip(U), wp, dummy, dummy, dummy, dummy, dummy, ws, 1 << 30, None)

    w = np.ones(wl.B, dtype=np.float32)
    for bad in (-0.5, np.nan, np.inf):
        w2 = w.copy(); w2[7] = bad
        assert call(w2) == 8                                     # RNNT_ERR_WEIGHT, before the workspace is looked at
    assert call(w, ws=None) == 5                                 # valid weights: the next check (workspace) fails
    assert call(None, ws=None) == 5                              # no weights = the unweighted call
    assert Bd.lib().rnnt_status_string(8).decode().startswith("a sample weight")


def test_label_validation():
    wl, desc, T, U = _lens("C2")
    _, _, lab = synth.draw_lengths_labels(wl)
    assert Bd.rnnt_validate_labels_host(desc, lab, U) == 0
    lab2 = lab.copy(); lab2[5, U[5] - 1] = wl.V
    assert Bd.rnnt_validate_labels_host(desc, lab2, U) == 4
    lab2[5, U[5] - 1] = 3; lab2[5, wl.U_max - 1] = -9 if U[5] < wl.U_max else 3   # beyond U_len: ignored
    assert Bd.rnnt_validate_labels_host(desc, lab2, U) == 0


def test_parallel_iterations_rule_matches_the_worked_values():
    with open(os.path.join(GOLD, "eq11_parallel_iterations.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    for T, U, V, _, pi in rows:
        assert Bd.rnnt_parallel_iterations(int(T), int(U), int(V)) == int(pi)
    assert Bd.rnnt_parallel_iterations(0, 1, 1) == 0


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_default_plan_properties(name):
    wl, desc, T, U = _lens(name)
    n = Bd.rnnt_joint_loss_workspace_bytes(desc, T, U, 0)
    # 256 MiB lattice state + 832 MiB chunk buffers + tables, packed weights and the dW partial sums
    assert 0 < n <= (1088 << 20) + (160 << 20)
    st, info, groups = Bd.rnnt_joint_loss_plan(desc, T, U, n)
    assert st == 0
    rows = T.astype(np.int64) * (U.astype(np.int64) + 1)
    assert info["rows_total"] == rows.sum()
    assert info["rows_padded"] == wl.B * wl.T_max * (wl.U_max + 1)
    tiles = _tiles(T, U)
    assert info["tiles_total"] == tiles.sum()
    assert info["workspace_bytes"] <= n
    # every sample in exactly one group, groups are consecutive, each fits the lattice capacity
    assert groups.min() == 0 and groups.max() == info["n_groups"] - 1
    assert np.all(np.diff(groups) >= 0)
    for g in range(info["n_groups"]):
        assert rows[groups == g].sum() <= info["group_rows_cap"]
    assert info["lattice_bytes"] >= 20 * info["group_rows_cap"]
    if wl.dtype == "bf16":
        assert info["chunk_rows"] % 128 == 0 and info["chunk_rows"] >= 128
        assert info["chunk_bytes"] >= info["chunk_rows"] * (2 * wl.V + 2 * wl.H)


def test_backward_chunks_are_whole_rounds_of_256_tiles_when_a_group_needs_several():
    # one workgroup per tile and 256 compute units: a chunk of a multiple of 256 tiles has no partly filled last round
    for name in ("C3", "C4"):
        wl, desc, T, U = _lens(name)
        st, info, groups = Bd.rnnt_joint_loss_plan(desc, T, U, 0)
        assert st == 0
        cap = info["chunk_rows"] // 64
        assert cap >= 1024
        per = cap // 256 * 256
        tiles = _tiles(T, U)
        want = 0
        for g in range(info["n_groups"]):
            n = int(tiles[groups == g].sum())
            want += -(-n // per) if n > cap else 1
        assert info["n_chunks"] == want, name


def test_fp32_shapes_with_gemm_tiles_get_chunk_buffers():
    T = np.array([30, 17, 25], dtype=np.int32); U = np.array([7, 0, 11], dtype=np.int32)
    rows = int((T.astype(np.int64) * (U + 1)).sum())
    for H, V, gemm in [(128, 256, True), (256, 128, True), (96, 200, True), (128, 202, False), (60, 256, False)]:
        desc = Bd.make_desc(3, 30, 11, H, V, 0, Bd.RNNT_F32)
        st, info, _ = Bd.rnnt_joint_loss_plan(desc, T, U, 0)
        assert st == 0
        if gemm:
            # S [rows, V], Z and dZ [rows, H] in fp32, rows = the call's lattice nodes rounded up to 128
            assert info["chunk_rows"] == -(-rows // 128) * 128
            assert info["chunk_bytes"] >= info["chunk_rows"] * (4 * V + 8 * H)
            nmin = Bd.rnnt_joint_loss_workspace_bytes(desc, T, U, 1)
            st, small, groups = Bd.rnnt_joint_loss_plan(desc, T, U, nmin)
            assert st == 0 and small["chunk_rows"] == 128 and small["n_groups"] == 2
            # chunks are ranges of 128 lattice nodes of a group
            per_sample = T.astype(np.int64) * (U + 1)
            assert small["n_chunks"] == sum(-(-int(per_sample[groups == g].sum()) // 128) for g in range(2))
            assert info["n_chunks"] == info["n_groups"] == 1
        else:
            assert info["chunk_rows"] == 0 and info["chunk_bytes"] == 0


def test_workspace_does_not_grow_with_batch_size_once_capped():
    # memory "almost independent of batch size" (Section 5.2): doubling B leaves the default plan's size
    wl = synth.WORKLOADS["C4"]
    T, U, _ = synth.draw_lengths_labels(wl)
    d1 = Bd.make_desc(512, wl.T_max, wl.U_max, wl.H, wl.V, 0, Bd.RNNT_BF16)
    d2 = Bd.make_desc(1024, wl.T_max, wl.U_max, wl.H, wl.V, 0, Bd.RNNT_BF16)
    n1 = Bd.rnnt_joint_loss_workspace_bytes(d1, T[:512], U[:512], 0)
    n2 = Bd.rnnt_joint_loss_workspace_bytes(d2, T, U, 0)
    assert abs(n2 - n1) <= 8 * 1024 * 1024      # only the per-sample and per-tile index tables grow


def test_budgets_shrink_the_plan_and_a_too_small_budget_is_reported():
    wl, desc, T, U = _lens("C4")
    big = Bd.rnnt_joint_loss_workspace_bytes(desc, T, U, 0)
    small_budget = 96 << 20
    n = Bd.rnnt_joint_loss_workspace_bytes(desc, T, U, small_budget)
    assert 0 < n <= small_budget < big
    st, info, groups = Bd.rnnt_joint_loss_plan(desc, T, U, n)
    st0, info0, _ = Bd.rnnt_joint_loss_plan(desc, T, U, big)
    assert st == 0 and st0 == 0
    assert info["n_groups"] > info0["n_groups"] and info["n_chunks"] > info0["n_chunks"]
    rows = T.astype(np.int64) * (U.astype(np.int64) + 1)
    for g in range(info["n_groups"]):
        assert rows[groups == g].sum() <= info["group_rows_cap"]
    # the largest sample still fits: it is processed alone, the backward walks it in row chunks
    assert info["group_rows_cap"] >= rows.max()
    tiny = Bd.rnnt_joint_loss_workspace_bytes(desc, T, U, 1 << 20)
    assert tiny > (1 << 20)
    st, _, _ = Bd.rnnt_joint_loss_plan(desc, T, U, 1 << 20)
    assert st == 5
    st, info_min, _ = Bd.rnnt_joint_loss_plan(desc, T, U, tiny)
    assert st == 0 and info_min["chunk_rows"] == 128 and info_min["group_rows_cap"] == rows.max()


def test_keep_scores_plan_has_one_backward_chunk_per_group_of_whole_samples():
    wl, desc, T, U = _lens("C2")
    keep = Bd.make_desc(wl.B, wl.T_max, wl.U_max, wl.H, wl.V, 0, Bd.RNNT_BF16, keep_scores=1)
    st, info, groups = Bd.rnnt_joint_loss_plan(keep, T, U, 0)
    assert st == 0 and info["n_chunks"] == info["n_groups"] == 1 and (groups == 0).all()
    # the chunk buffers hold every tile row of the call: dH, Z and the running maxima
    per_row = 2 * (wl.V + 64) + 2 * (wl.H + 64) + 4 * (wl.V // 64)
    slack = 128 * 2 * (wl.V + 64) + 3 * 256          # dH ends on a multiple of 256 rows; alignment of the three
    assert info["chunk_rows"] * per_row <= info["chunk_bytes"] < info["chunk_rows"] * per_row + slack
    assert info["chunk_rows"] >= info["tiles_total"] * 64
    # smallest plan: the chunk buffers still hold the largest sample, one sample or more per group
    nmin = Bd.rnnt_joint_loss_workspace_bytes(keep, T, U, 1)
    st, small, groups = Bd.rnnt_joint_loss_plan(keep, T, U, nmin)
    assert st == 0 and small["n_chunks"] == small["n_groups"] > 1
    tiles = _tiles(T, U)
    assert small["chunk_rows"] >= int(tiles.max()) * 64
    for g in range(small["n_groups"]):
        assert int(tiles[groups == g].sum()) * 64 <= small["chunk_rows"]
    assert np.all(np.diff(groups) >= 0)
    st, _, _ = Bd.rnnt_joint_loss_plan(keep, T, U, nmin - 256)
    assert st == 5
    # a budget in between gives groups in between
    st, mid, _ = Bd.rnnt_joint_loss_plan(keep, T, U, (nmin + info["workspace_bytes"]) // 2)
    assert st == 0 and 1 <= mid["n_groups"] < small["n_groups"] and mid["workspace_bytes"] <= (nmin + info["workspace_bytes"]) // 2
    # only the bf16 path has the mode, and the flag is 0 or 1
    assert Bd.rnnt_joint_loss_workspace_bytes(Bd.make_desc(2, 8, 3, 16, 8, 0, Bd.RNNT_F32, keep_scores=1), [8, 8], [3, 3]) == 0
    assert Bd.rnnt_joint_loss_workspace_bytes(
        Bd.make_desc(wl.B, wl.T_max, wl.U_max, wl.H, wl.V, 0, Bd.RNNT_BF16, keep_scores=2), T, U) == 0


def test_bf16_input_gradients_add_a_bounded_staging_area_and_cap_the_group_size():
    wl, desc, T, U = _lens("C4")
    half = Bd.make_desc(wl.B, wl.T_max, wl.U_max, wl.H, wl.V, 0, Bd.RNNT_BF16, input_grads_bf16=1)
    n0 = Bd.rnnt_joint_loss_workspace_bytes(desc, T, U, 0)
    n1 = Bd.rnnt_joint_loss_workspace_bytes(half, T, U, 0)
    per_sample = (wl.T_max + wl.U_max + 1) * wl.H * 4
    cap = (256 << 20) // per_sample
    assert 0 < n1 - n0 <= (256 << 20) + 512 and n1 - n0 >= cap * per_sample
    st, info, groups = Bd.rnnt_joint_loss_plan(half, T, U, n1)
    assert st == 0 and np.bincount(groups).max() <= cap
    # the outputs shrink by more than the workspace grows
    assert (n1 - n0) < wl.B * per_sample // 2
    # smallest plan: one sample per group
    nmin = Bd.rnnt_joint_loss_workspace_bytes(half, T[:8], U[:8], 1)
    h8 = Bd.make_desc(8, wl.T_max, wl.U_max, wl.H, wl.V, 0, Bd.RNNT_BF16, input_grads_bf16=1)
    nmin = Bd.rnnt_joint_loss_workspace_bytes(h8, T[:8], U[:8], 1)
    st, info, groups = Bd.rnnt_joint_loss_plan(h8, T[:8], U[:8], nmin)
    assert st == 0 and info["n_groups"] == 8
    # bf16 only; not for the projected entry point, whose d_enc / d_pred are internal
    assert Bd.rnnt_joint_loss_workspace_bytes(Bd.make_desc(2, 8, 3, 16, 8, 0, Bd.RNNT_F32, input_grads_bf16=1), [8, 8], [3, 3]) == 0
    assert Bd.rnnt_joint_proj_workspace_bytes(half, 512, 512, T, U, 0) == 0


def test_random_plans_keep_their_promises():
    # seeded random shapes, lengths, options and budgets: every sample is in exactly one group, groups are runs of
    # consecutive samples, a plan never exceeds the workspace it was made for, the size the library asks for is
    # accepted, and the options' extra limits hold (kept scores: a group's tile rows fit the chunk buffers;
    # bfloat16 input gradients: groups no larger than the staging area was sized for)
    rng = np.random.default_rng(20240)
    for case in range(150):
        bf16 = bool(rng.integers(0, 4))
        B = int(rng.integers(1, 40))
        T_max, U_max = int(rng.integers(1, 300)), int(rng.integers(0, 120))
        if bf16:
            H, V = int(rng.choice([128, 256, 512, 640, 768, 1024])), int(rng.choice([256, 512, 1024, 4096]))
            opts = dict(keep_scores=int(rng.integers(0, 2)), input_grads_bf16=int(rng.integers(0, 2)))
        else:
            H, V, opts = int(rng.integers(1, 200)), int(rng.integers(2, 300)), {}
        T = rng.integers(1, T_max + 1, size=B).astype(np.int32)
        U = rng.integers(0, U_max + 1, size=B).astype(np.int32)
        desc = Bd.make_desc(B, T_max, U_max, H, V, 0, Bd.RNNT_BF16 if bf16 else Bd.RNNT_F32, **opts)
        n_default = Bd.rnnt_joint_loss_workspace_bytes(desc, T, U, 0)
        n_min = Bd.rnnt_joint_loss_workspace_bytes(desc, T, U, 1)
        assert 0 < n_min <= n_default, (case, n_min, n_default)
        tiles = _tiles(T, U)
        rows = T.astype(np.int64) * (U + 1)
        for budget in (n_default, n_min, int(rng.integers(n_min, n_default + 1)), n_default + int(rng.integers(1, 1 << 24))):
            st, info, groups = Bd.rnnt_joint_loss_plan(desc, T, U, budget)
            what = (case, opts, budget, info)
            assert st == 0, what
            assert info["workspace_bytes"] <= budget, what
            assert groups.min() == 0 and np.all(np.diff(groups) >= 0) and np.all(np.diff(groups) <= 1), what
            assert groups.max() + 1 == info["n_groups"] and info["n_chunks"] >= info["n_groups"], what
            assert info["rows_total"] == rows.sum() and info["tiles_total"] == tiles.sum(), what
            for g in range(info["n_groups"]):
                m = groups == g
                assert rows[m].sum() <= info["group_rows_cap"] or m.sum() == 1, what
                if opts.get("keep_scores"):
                    assert tiles[m].sum() * 64 <= info["chunk_rows"], what
            if opts.get("keep_scores"):
                assert info["n_chunks"] == info["n_groups"], what
            if bf16:
                assert info["chunk_rows"] % 128 == 0 and info["chunk_rows"] >= 128, what
        assert Bd.rnnt_joint_loss_plan(desc, T, U, n_min - 256)[0] == 5, case


def test_tile_shape_per_sample():
    # 8 x 8 tiles, or 16 x 4 where that covers the lattice with at least 3 % fewer tiles
    desc = Bd.make_desc(5, 40, 20, 128, 256, 0, Bd.RNNT_BF16)
    T = np.array([16, 8, 32, 40, 33], dtype=np.int32)
    U = np.array([3, 7, 11, 20, 8], dtype=np.int32)
    st, info, _ = Bd.rnnt_joint_loss_plan(desc, T, U, 0)
    # 16 x 4: 1 (against 2); 8 x 8: 1; 16 x 4: 2 * 3 = 6 (against 4 * 2 = 8); 8 x 8: 5 * 3 = 15 (16 x 4: 3 * 6 = 18);
    # 33 x 9: 8 x 8 gives 5 * 2 = 10, 16 x 4 gives 3 * 3 = 9
    assert st == 0 and info["tiles_total"] == 1 + 1 + 6 + 15 + 9
    assert info["tiles_total"] == int(_tiles(T, U).sum())


def test_projected_entry_point_checks_and_workspace():
    wl, desc, T, U = _lens("C2")
    L = Bd.lib()
    dummy = ctypes.c_void_p(0x1000)
    Tl, Ul = np.ascontiguousarray(T, dtype=np.int32), np.ascontiguousarray(U, dtype=np.int32)

    def call(H_A, H_L, hA=dummy, ws_bytes=1 << 32, d=desc):
        return L.rnnt_joint_proj_loss_fwd_bwd(ctypes.byref(d), H_A, H_L, hA, dummy, dummy, dummy, dummy, dummy, dummy,
                                              dummy, Bd._ip(Tl), Bd._ip(Ul), *([dummy] * 8), dummy, ws_bytes, None)

    assert call(512, 512, hA=None) == 1                # RNNT_ERR_NULL
    assert call(0, 512) == 2                           # RNNT_ERR_SHAPE
    assert call(200, 512) == 6                         # bf16 needs multiples of 128
    assert call(8192, 512) == 6
    inner = Bd.rnnt_joint_loss_workspace_bytes(desc, T, U, 0)
    n = Bd.rnnt_joint_proj_workspace_bytes(desc, 512, 256, T, U, 0)
    # in front of the inner workspace: enc, pred in the input dtype and d_enc, d_pred in fp32
    rows_a, rows_l = wl.B * wl.T_max, wl.B * (wl.U_max + 1)
    extra = (rows_a + rows_l) * wl.H * (2 + 4)
    assert inner + extra <= n <= inner + extra + 4 * 256
    assert call(512, 256, ws_bytes=extra) == 5         # RNNT_ERR_WORKSPACE: nothing left for the inner path
    assert call(512, 256, ws_bytes=extra + 4096) == 5  # less than the smallest inner plan
    assert Bd.rnnt_joint_proj_workspace_bytes(desc, 100, 256, T, U, 0) == 0


def test_group_of_samples_never_exceeds_32_bit_lattice_indices():
    # 4096 samples of 1000 x 1024 nodes are 4.2e9 lattice nodes; with a workspace that could hold them all the
    # planner still cuts groups below 2^31 nodes (the kernels index a group's lattice state with 32-bit integers)
    B = 4096
    desc = Bd.make_desc(B, 1000, 1023, 512, 1024, 0, Bd.RNNT_BF16)
    T, U = np.full(B, 1000, dtype=np.int32), np.full(B, 1023, dtype=np.int32)
    st, info, groups = Bd.rnnt_joint_loss_plan(desc, T, U, 200 << 30)
    assert st == 0 and info["rows_total"] == B * 1000 * 1024 > 2 ** 31
    assert info["group_rows_cap"] <= 2 ** 31 - 1 and info["n_groups"] >= 2
    counts = np.bincount(groups)
    assert counts.max() * 1000 * 1024 <= 2 ** 31 - 1


def test_plan_handle_holds_the_schedule_of_the_plan_query():
    # no GPU needed: the handle falls back to ordinary host memory for its tables
    wl = synth.WORKLOADS["C4"]
    T, U, _ = synth.draw_lengths_labels(wl)
    desc = Bd.make_desc(wl.B, wl.T_max, wl.U_max, wl.H, wl.V, 0, Bd.RNNT_BF16)
    st, info, _ = Bd.rnnt_joint_loss_plan(desc, T, U, 0)
    assert st == 0
    h = Bd.PlanHandle(desc, T, U)
    assert h.workspace_bytes == info["workspace_bytes"] == Bd.rnnt_joint_loss_workspace_bytes(desc, T, U, 0)
    assert h.describe() == info
    h.close()
    # room for the lattice state of two groups: each group at most half as large, same lattice bytes
    h2 = Bd.PlanHandle(desc, T, U, overlap_lattice=True)
    d2 = h2.describe()
    assert d2["lattice_bytes"] <= info["lattice_bytes"] + 4096
    assert d2["group_rows_cap"] * 2 <= info["group_rows_cap"] + 2
    assert d2["n_groups"] >= 2 * info["n_groups"] - 1 and d2["rows_total"] == info["rows_total"]
    h2.close()
    # bad arguments are refused when the handle is made
    bad = Bd.make_desc(wl.B, wl.T_max, wl.U_max, 500, wl.V, 0, Bd.RNNT_BF16)
    with pytest.raises(Bd.RnntError):
        Bd.PlanHandle(bad, T, U)
    with pytest.raises(Bd.RnntError):
        Bd.PlanHandle(desc, T + 1000, U)
    assert Bd.lib().rnnt_plan_workspace_bytes(None) == 0
    Bd.lib().rnnt_plan_destroy(None)
