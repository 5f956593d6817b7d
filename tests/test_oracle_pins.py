"""Pins of the CPU oracle against things other than itself (CPU only).

Brute force on tiny inputs, a dense one-hot formulation of the reduce, hand-computed
Adagrad steps (tests/golden/adagrad_hand_example.txt), a library optimizer on the special
case where row-wise and element-wise Adagrad coincide, a closed form over T steps, library
bf16 conversion, and the invariants of the collision partition (Section 3.2 of the paper:
strict write-read ordering is only needed on collision rows, so every schedule of the two
update passes must give the same table).
"""
import math
import os
import subprocess
import ctypes

import numpy as np
import pytest
import torch

import oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- brute force
def brute_unique(ids):
    ids = [int(x) for x in ids]
    uniq = []
    for v in ids:                       # O(n^2) membership
        if v not in uniq:
            uniq.append(v)
    # selection-sort ascending
    out = []
    while uniq:
        m = min(uniq)
        out.append(m)
        uniq.remove(m)
    inverse = [out.index(v) for v in ids]
    perm = []
    seg = [0]
    for k, u in enumerate(out):
        occ = [j for j, v in enumerate(ids) if v == u]      # ascending j
        perm.extend(occ)
        seg.append(len(perm))
    return out, seg, perm, inverse


def brute_split(u_t, u_t1):
    u_t, u_t1 = [int(x) for x in u_t], [int(x) for x in u_t1]
    co = [(v, i) for i, v in enumerate(u_t) if any(v == w for w in u_t1)]
    ex = [(v, i) for i, v in enumerate(u_t) if not any(v == w for w in u_t1)]
    exn = [(w, j) for j, w in enumerate(u_t1) if not any(w == v for v in u_t)]
    return co, ex, exn


@pytest.mark.parametrize("seed", range(12))
def test_unique_and_split_match_brute_force(seed):
    rng = np.random.default_rng(seed)
    n_rows = int(rng.integers(1, 17))
    n0, n1 = int(rng.integers(0, 65)), int(rng.integers(0, 65))
    a = rng.integers(0, n_rows, size=n0)
    b = rng.integers(0, n_rows, size=n1)
    for ids in (a, b):
        r = O.unique_ids(ids, n_rows)
        u, seg, perm, inv = brute_unique(ids)
        assert r["unique"].tolist() == u
        assert r["seg_offsets"].tolist() == seg
        assert r["perm"].tolist() == perm
        assert r["inverse"].tolist() == inv
        assert r["n_unique"] == len(u)
    ua, ub = O.unique_ids(a, n_rows)["unique"], O.unique_ids(b, n_rows)["unique"]
    sp = O.collision_split(ua, ub)
    co, ex, exn = brute_split(ua, ub)
    assert list(zip(sp["co"].tolist(), sp["co_slot"].tolist())) == co
    assert list(zip(sp["ex"].tolist(), sp["ex_slot"].tolist())) == ex
    assert list(zip(sp["ex_next"].tolist(), sp["ex_next_slot"].tolist())) == exn


def test_unique_full_64bit_keys():
    ids = np.array([2**62, 5, 2**40 + 3, 5, 2**62, 0], dtype=np.int64)
    r = O.unique_ids(ids, 0)
    assert r["unique"].tolist() == [0, 5, 2**40 + 3, 2**62]
    assert r["perm"].tolist() == [5, 1, 3, 2, 0, 4]
    assert r["inverse"].tolist() == [3, 1, 2, 1, 3, 0]


def test_unique_and_split_at_the_top_of_the_id_range():
    """IDs up to 2^63 - 1 are legal when the table size is not given: brute force on both operations."""
    top = 2**63 - 1
    a = np.array([top, 7, top - 1, top, top - 3, 7], dtype=np.int64)
    b = np.array([top - 1, top - 2, top, 3], dtype=np.int64)
    ra, rb = O.unique_ids(a, 0), O.unique_ids(b, 0)
    ua, sa, pa, ia = brute_unique(a)
    assert ra["unique"].tolist() == ua == [7, top - 3, top - 1, top]
    assert ra["seg_offsets"].tolist() == sa and ra["perm"].tolist() == pa and ra["inverse"].tolist() == ia
    sp = O.collision_split(ra["unique"], rb["unique"])
    co, ex, exn = brute_split(ra["unique"], rb["unique"])
    assert list(zip(sp["co"].tolist(), sp["co_slot"].tolist())) == co == [(top - 1, 2), (top, 3)]
    assert list(zip(sp["ex"].tolist(), sp["ex_slot"].tolist())) == ex
    assert list(zip(sp["ex_next"].tolist(), sp["ex_next_slot"].tolist())) == exn == [(3, 0), (top - 2, 1)]


def test_unique_rejects_out_of_range():
    with pytest.raises(O.OracleError) as e:
        O.unique_ids(np.array([1, 7, 3]), 7)
    assert e.value.code == O.ERANGE
    with pytest.raises(O.OracleError):
        O.unique_ids(np.array([1, -1]), 0)


def test_split_rejects_unsorted():
    with pytest.raises(O.OracleError):
        O.collision_split(np.array([3, 2]), np.array([1]))
    with pytest.raises(O.OracleError):
        O.collision_split(np.array([1]), np.array([2, 2]))


# ----------------------------------------------------------------------------- gather
def test_gather_matches_library_indexing():
    rng = np.random.default_rng(3)
    table = rng.standard_normal((50, 12)).astype(np.float32)
    lens = rng.integers(0, 6, size=9)          # includes empty sequences
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    values = rng.integers(0, 50, size=int(offsets[-1]))
    out = O.gather_jagged(table, values, offsets)
    assert out.tobytes() == table[values].tobytes()
    tb = (rng.integers(0, 2**16, size=(50, 8))).astype(np.uint16)
    outb = O.gather_jagged(tb, values, offsets)
    assert np.array_equal(outb, tb[values])


def test_gather_errors():
    table = np.zeros((4, 4), dtype=np.float32)
    with pytest.raises(O.OracleError) as e:
        O.gather_jagged(table, np.array([0, 4]), np.array([0, 2]))
    assert e.value.code == O.ERANGE
    with pytest.raises(O.OracleError):
        O.gather_jagged(table, np.array([0, 1]), np.array([0, 1]))      # offsets[-1] != n
    with pytest.raises(O.OracleError):
        O.gather_jagged(table, np.array([0, 1]), np.array([0, 3, 2]))   # non-monotone
    assert O.gather_jagged(table, np.empty(0, np.int64), np.array([0, 0, 0])).shape == (0, 4)


# ----------------------------------------------------------------------------- reduce
@pytest.mark.parametrize("seed", range(4))
def test_reduce_matches_dense_one_hot(seed):
    rng = np.random.default_rng(100 + seed)
    n_rows, n, dim = 11, 57, 5
    ids = rng.integers(0, n_rows, size=n)
    grads = rng.standard_normal((n, dim)).astype(np.float32)
    lay = O.unique_ids(ids, n_rows)
    g = O.segment_reduce_grads(grads, lay["perm"], lay["seg_offsets"])
    onehot = (ids.reshape(-1, 1) == lay["unique"].reshape(1, -1)).astype(np.float64)   # [n, U]
    dense = onehot.T @ grads.astype(np.float64)
    # fp64 sums rounded once to fp32: equal up to the fp64 summation order (<< 1 fp32 ulp)
    assert np.array_equal(g, dense.astype(np.float32)) or np.allclose(g, dense, rtol=2e-7, atol=0)
    assert np.allclose(g.astype(np.float64).sum(0), grads.astype(np.float64).sum(0), atol=1e-5)


def test_reduce_is_fp64_accumulated():
    # 1 + 2^-30 + ... would be lost in fp32 accumulation; the cancelling big terms must not
    # destroy the small one.
    grads = np.array([[1e8], [1.0], [-1e8]], dtype=np.float32)
    lay = O.unique_ids(np.array([4, 4, 4]), 10)
    g = O.segment_reduce_grads(grads, lay["perm"], lay["seg_offsets"])
    assert g.tolist() == [[1.0]]


# ----------------------------------------------------------------------------- adagrad
def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "adagrad_hand_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([float(x) for x in line.split()])
    return rows


def test_adagrad_hand_example():
    table = np.zeros((3, 2), dtype=np.float32)
    table[1] = [1.0, 2.0]
    before_other = table[[0, 2]].copy()
    state = np.zeros(3, dtype=np.float32)
    g = np.array([[3.0, -4.0]], dtype=np.float32)
    for _step, s, w0, w1 in _golden_rows():
        O.rowwise_adagrad_update(table, state, np.array([1]), np.array([0]), g, 0.01, 1e-8)
        assert state[1] == pytest.approx(s, rel=1e-6)
        assert table[1, 0] == pytest.approx(w0, abs=5e-7)
        assert table[1, 1] == pytest.approx(w1, abs=5e-7)
    assert np.array_equal(table[[0, 2]], before_other)
    assert state[0] == 0 and state[2] == 0


def test_adagrad_duplicates_sum_then_one_step():
    # the same row three times with grads summing to [3,-4] == one occurrence of [3,-4]
    ids = np.array([1, 1, 1])
    grads = np.array([[1, -1], [1, -2], [1, -1]], dtype=np.float32)
    lay = O.unique_ids(ids, 3)
    g = O.segment_reduce_grads(grads, lay["perm"], lay["seg_offsets"])
    assert g.tolist() == [[3.0, -4.0]]
    t1 = np.zeros((3, 2), np.float32); t1[1] = [1, 2]; s1 = np.zeros(3, np.float32)
    O.rowwise_adagrad_update(t1, s1, lay["unique"], np.array([0]), g, 0.01, 1e-8)
    _step, s, w0, w1 = _golden_rows()[0]
    assert s1[1] == pytest.approx(s) and t1[1, 0] == pytest.approx(w0, abs=5e-7) and t1[1, 1] == pytest.approx(w1, abs=5e-7)


@pytest.mark.parametrize("dim", [1, 4])
def test_adagrad_equals_elementwise_library_adagrad_when_columns_have_equal_magnitude(dim):
    # If |g_d| is the same for every column of a row, mean_d g^2 == g_d^2 and row-wise Adagrad is
    # element-wise Adagrad: compare with torch.optim.Adagrad (eps outside the sqrt, state 0).
    rng = np.random.default_rng(7)
    n_rows, steps, lr, eps = 6, 5, 0.05, 1e-8
    w0 = rng.standard_normal((n_rows, dim)).astype(np.float32)
    table, state = w0.copy(), np.zeros(n_rows, np.float32)
    p = torch.nn.Parameter(torch.from_numpy(w0.copy()))
    opt = torch.optim.Adagrad([p], lr=lr, lr_decay=0.0, weight_decay=0.0, initial_accumulator_value=0.0, eps=eps)
    for _ in range(steps):
        touched = np.sort(rng.choice(n_rows, size=3, replace=False))
        mag = rng.uniform(0.1, 2.0, size=(3, 1)).astype(np.float32)
        sign = rng.choice([-1.0, 1.0], size=(3, dim)).astype(np.float32)
        g = mag * sign
        O.rowwise_adagrad_update(table, state, touched, np.arange(3, dtype=np.int32), g, lr, eps)
        dense = torch.zeros(n_rows, dim)
        dense[torch.from_numpy(touched)] = torch.from_numpy(g)
        p.grad = dense
        opt.step()
    assert np.allclose(table, p.detach().numpy(), rtol=1e-6, atol=1e-7)
    acc = opt.state[p]["sum"].numpy()
    assert np.allclose(state, acc[:, 0], rtol=1e-6)


def test_adagrad_closed_form_constant_gradient():
    # |g_d| = c for T steps: S_T = T c^2, w_T = w_0 - lr*sign(g)*sum_{tau<=T} tau^-1/2
    dim, c, T, lr = 8, 0.5, 20, 0.01
    sign = np.array([1, -1] * (dim // 2), dtype=np.float32)
    g = (c * sign).reshape(1, dim)
    table = np.ones((2, dim), np.float32); state = np.zeros(2, np.float32)
    for _ in range(T):
        O.rowwise_adagrad_update(table, state, np.array([1]), np.array([0]), g, lr, 1e-12)
    assert state[1] == pytest.approx(T * c * c, rel=1e-6)
    expect = 1.0 - lr * sign * sum(tau ** -0.5 for tau in range(1, T + 1))
    assert np.allclose(table[1], expect, atol=1e-6)
    assert np.all(table[0] == 1.0)


def test_adagrad_lr_zero_keeps_weights_but_grows_state():
    table = np.full((2, 4), 0.25, np.float32); state = np.zeros(2, np.float32)
    g = np.array([[1, 2, 3, 4]], np.float32)
    O.rowwise_adagrad_update(table, state, np.array([0]), np.array([0]), g, 0.0, 1e-8)
    assert np.all(table == 0.25) and state[0] == pytest.approx(7.5) and state[1] == 0


def test_mean_not_sum_is_detected_by_the_hand_example(tmp_path):
    # Plant the plausible mistake (sum over columns instead of mean) in a private build of the
    # oracle and check that the hand example rejects it.
    lib = tmp_path / "libfs_oracle_sum.so"
    subprocess.run(["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-DFSO_ADAGRAD_MEAN=0",
                    "-o", str(lib), os.path.join(os.path.dirname(O.__file__), "freescale_oracle.c"), "-lm"], check=True)
    bad = ctypes.CDLL(str(lib))
    table = np.array([[1.0, 2.0]], np.float32); state = np.zeros(1, np.float32)
    g = np.array([[3.0, -4.0]], np.float32)
    rows = np.array([0], np.int64); slots = np.array([0], np.int32)
    vp = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    rc = bad.fso_rowwise_adagrad_update(vp(table), 0, vp(state), ctypes.c_int64(1), ctypes.c_int32(2), vp(rows),
                                        vp(slots), ctypes.c_int64(1), vp(g), ctypes.c_float(0.01), ctypes.c_float(1e-8))
    assert rc == 0
    assert abs(state[0] - 12.5) > 1.0


# ----------------------------------------------------------------------------- bf16
def test_bf16_conversion_matches_library_rne():
    rng = np.random.default_rng(11)
    x = np.concatenate([
        rng.standard_normal(2000).astype(np.float32),
        (rng.standard_normal(500) * 1e-30).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 1.0 + 2**-8, 1.0 + 3 * 2**-8, 3.3895314e38,
                  np.inf, -np.inf, 65504.0, 1e-45], dtype=np.float32),       # ties both ways, overflow to inf
    ])
    got = O.f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    assert np.array_equal(O.bf16_bits_to_f32(got), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_bf16_update_widens_updates_rounds():
    w = np.array([[0.5, -0.25, 0.0078125, 1.0]], dtype=np.float32)
    table = O.f32_to_bf16_bits(w)
    state = np.zeros(1, np.float32)
    g = np.array([[1.0, -1.0, 1.0, -1.0]], np.float32)
    O.rowwise_adagrad_update(table, state, np.array([0]), np.array([0]), g, 0.01, 1e-8)
    # S=1, c=0.01/(1+1e-8) -> fp32 0.01
    c = np.float32(0.01) / (np.float32(1.0) + np.float32(1e-8))
    expect = torch.from_numpy((w - c * g).astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(table, expect)


# ----------------------------------------------------------------------------- invariants
def _random_case(rng, n_rows, b, max_len, dim):
    lens = rng.integers(0, max_len + 1, size=b)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    ranks = np.minimum(rng.zipf(1.3, size=int(offsets[-1])), n_rows) - 1
    values = (ranks * 7 + 3) % n_rows
    grads = rng.standard_normal((values.shape[0], dim)).astype(np.float32)
    return values.astype(np.int64), offsets, grads


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("tdtype", ["f32", "bf16"])
def test_partition_invariants_and_schedule_independence(seed, tdtype):
    rng = np.random.default_rng(1000 + seed)
    n_rows, dim = 97, 8
    v0, o0, g0 = _random_case(rng, n_rows, 6, 20, dim)
    v1, o1, _ = _random_case(rng, n_rows, 6, 20, dim)
    w = (rng.standard_normal((n_rows, dim)) * 0.1).astype(np.float32)
    table0 = w if tdtype == "f32" else O.f32_to_bf16_bits(w)
    lay0 = O.unique_ids(v0, n_rows)
    u0 = lay0["unique"]
    assert np.all(np.diff(u0) > 0)
    assert np.array_equal(u0[lay0["inverse"]], v0)
    assert sorted(lay0["perm"].tolist()) == list(range(len(v0)))
    assert np.all(np.diff(v0[lay0["perm"]]) >= 0)
    assert lay0["seg_offsets"][-1] == len(v0)

    results = {}
    for sched in O.SCHEDULES:
        table, state = table0.copy(), np.zeros(n_rows, np.float32)
        r = O.step(table, state, lay0, g0, v1, o1, 0.01, 1e-8, schedule=sched)
        results[sched] = (table, state, r)
    t_ref, s_ref, r_ref = results["co_then_ex"]
    sp = r_ref["split"]
    u1 = r_ref["layout_next"]["unique"]
    assert len(sp["co"]) + len(sp["ex"]) == len(u0)
    assert set(sp["co"]).isdisjoint(sp["ex"])
    assert set(sp["co"]) | set(sp["ex"]) == set(u0.tolist())
    assert set(sp["co"]) <= set(u1.tolist())
    assert set(sp["ex"]).isdisjoint(u1.tolist())
    assert set(sp["ex_next"]) | set(sp["co"]) == set(u1.tolist())
    assert np.array_equal(u0[sp["co_slot"]], sp["co"]) and np.array_equal(u0[sp["ex_slot"]], sp["ex"])
    assert np.array_equal(u1[sp["ex_next_slot"]], sp["ex_next"])
    # rows outside U_t untouched; state non-decreasing
    untouched = np.setdiff1d(np.arange(n_rows), u0)
    assert np.array_equal(t_ref[untouched], table0[untouched])
    assert np.all(s_ref >= 0) and np.all(s_ref[untouched] == 0)
    # the lookahead gather sees the post-update table (also when issued between the passes)
    assert np.array_equal(r_ref["emb_next"], t_ref[v1])
    for sched in O.SCHEDULES[1:]:
        t, s, r = results[sched]
        assert t.tobytes() == t_ref.tobytes(), sched
        assert s.tobytes() == s_ref.tobytes(), sched
        assert r["emb_next"].tobytes() == r_ref["emb_next"].tobytes(), sched


def test_degenerate_splits():
    ids = np.array([5, 9, 5, 1])
    lay = O.unique_ids(ids, 10)
    same = O.collision_split(lay["unique"], lay["unique"])
    assert same["co"].tolist() == [1, 5, 9] and len(same["ex"]) == 0 and len(same["ex_next"]) == 0
    disj = O.collision_split(np.array([1, 3]), np.array([0, 2, 4]))
    assert len(disj["co"]) == 0 and disj["ex"].tolist() == [1, 3] and disj["ex_next"].tolist() == [0, 2, 4]
    empty = O.collision_split(np.array([1, 3]), np.empty(0, np.int64))
    assert empty["ex"].tolist() == [1, 3] and len(empty["co"]) == 0
    empty2 = O.collision_split(np.empty(0, np.int64), np.array([2]))
    assert empty2["ex_next"].tolist() == [2]
    one = O.unique_ids(np.full(9, 4), 10)
    assert one["unique"].tolist() == [4] and one["seg_offsets"].tolist() == [0, 9]
    grads = np.arange(18, dtype=np.float32).reshape(9, 2)
    g = O.segment_reduce_grads(grads, one["perm"], one["seg_offsets"])
    assert g.tolist() == [grads.sum(0).tolist()]
    none = O.unique_ids(np.empty(0, np.int64), 10)
    assert none["n_unique"] == 0 and none["seg_offsets"].tolist() == [0]


def test_last_iteration_flushes_everything_in_one_pass():
    rng = np.random.default_rng(5)
    v0, o0, g0 = _random_case(rng, 31, 4, 10, 4)
    table = rng.standard_normal((31, 4)).astype(np.float32); state = np.zeros(31, np.float32)
    lay = O.unique_ids(v0, 31)
    r = O.step(table, state, lay, g0, None, None, 0.01, 1e-8)
    assert len(r["split"]["co"]) == 0 and np.array_equal(r["split"]["ex"], lay["unique"])
    assert r["emb_next"] is None


# ------------------------------------------------------------------ two-part lookup and merge
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_class_lookup_matches_brute_force(seed):
    rng = np.random.default_rng(400 + seed)
    rows, dim, n = 50, 4, 200
    table = rng.standard_normal((rows, dim)).astype(np.float32)
    values = rng.integers(0, rows, size=n).astype(np.int64)
    u_t = np.unique(rng.integers(0, rows, size=20)).astype(np.int64)
    members = [int(x) for x in u_t]
    for which in (0, 1):
        out = np.full((n, dim), -7.0, dtype=np.float32)
        O.gather_jagged_class(table, values, u_t, which, out)
        for j in range(n):
            r = int(values[j])
            if (r in members) == bool(which):
                assert np.array_equal(out[j], table[r])
            else:
                assert np.all(out[j] == -7.0)
    # both kinds into one buffer, in either order, is the whole lookup
    for order in ((0, 1), (1, 0)):
        out = np.full((n, dim), -7.0, dtype=np.float32)
        for which in order:
            O.gather_jagged_class(table, values, u_t, which, out)
        assert np.array_equal(out, table[values])
    with pytest.raises(O.OracleError):
        O.gather_jagged_class(table, values, u_t[::-1].copy(), 0, np.zeros((n, dim), np.float32))
    with pytest.raises(O.OracleError):
        O.gather_jagged_class(table, np.array([rows], dtype=np.int64), u_t, 0, np.zeros((1, dim), np.float32))


def _synchronous_baseline(table, state, values_seq, grads_seq, lr, eps):
    """Fig. 1 of the paper on one shard: every update of iteration i lands, then iteration i+1 looks up."""
    out = []
    for i, g in enumerate(grads_seq):
        lay = O.unique_ids(values_seq[i], table.shape[0])
        red = O.segment_reduce_grads(g, lay["perm"], lay["seg_offsets"])
        O.rowwise_adagrad_update(table, state, lay["unique"], np.arange(lay["unique"].shape[0], dtype=np.int32),
                                 red, lr, eps)
        if i + 1 < len(values_seq):
            out.append(table[values_seq[i + 1]].copy())
    return out


@pytest.mark.parametrize("seed,tdtype", [(0, "f32"), (1, "f32"), (2, "bf16")])
def test_two_part_lookup_keeps_parity_with_the_synchronous_baseline(seed, tdtype):
    # Section 3.2: ordering only the collision rows keeps numerical parity with the synchronous run
    rng = np.random.default_rng(500 + seed)
    rows, dim, T = 40, 8, 6
    w0 = (rng.standard_normal((rows, dim)) * 0.1).astype(np.float32)
    if tdtype == "bf16":
        w0 = O.f32_to_bf16_bits(w0)
    values_seq = [rng.integers(0, rows, size=int(rng.integers(5, 60))).astype(np.int64) for _ in range(T + 1)]
    grads_seq = [rng.standard_normal((values_seq[i].shape[0], dim)).astype(np.float32) for i in range(T)]
    wa, sa = w0.copy(), np.zeros(rows, np.float32)
    wb, sb = w0.copy(), np.zeros(rows, np.float32)
    merged = O.run_two_phase(wa, sa, values_seq, grads_seq, 0.05, 1e-8)
    want = _synchronous_baseline(wb, sb, values_seq, grads_seq, 0.05, 1e-8)
    assert len(merged) == len(want) == T
    for a, b in zip(merged, want):
        assert np.array_equal(a, b)
    assert np.array_equal(wa, wb) and np.array_equal(sa, sb)
    # without a lookahead for the last iteration: one batch fewer comes back, same table
    wc, sc = w0.copy(), np.zeros(rows, np.float32)
    merged_c = O.run_two_phase(wc, sc, values_seq[:T], grads_seq, 0.05, 1e-8)
    assert len(merged_c) == T - 1 and np.array_equal(wc, wb)


def test_fetching_exclusive_rows_before_the_deferred_update_is_detected():
    # row 3 is exclusive at iteration 0 (absent from batch 1) and looked up again by batch 2: its deferred
    # update must land before Forward fetches the exclusive rows of batch 2
    rows, dim = 6, 4
    w0 = np.ones((rows, dim), np.float32)
    values_seq = [np.array([3, 1], np.int64), np.array([1, 2], np.int64), np.array([3, 2], np.int64)]
    grads_seq = [np.full((2, dim), 0.5, np.float32), np.full((2, dim), 0.25, np.float32)]
    wa, sa = w0.copy(), np.zeros(rows, np.float32)
    good = O.run_two_phase(wa, sa, values_seq, grads_seq, 0.1, 1e-8)
    wb, sb = w0.copy(), np.zeros(rows, np.float32)
    want = _synchronous_baseline(wb, sb, values_seq, grads_seq, 0.1, 1e-8)
    assert all(np.array_equal(a, b) for a, b in zip(good, want))
    wc, sc = w0.copy(), np.zeros(rows, np.float32)
    bad = O.run_two_phase(wc, sc, values_seq, grads_seq, 0.1, 1e-8, prefetch_before_deferred=True)
    assert not np.array_equal(bad[1], want[1])          # stale row 3 in the batch of iteration 2
    assert np.array_equal(bad[1][1], want[1][1])        # row 2 (a collision row) is still fresh


# ----------------------------------------------------------- FBS partitioner, indexed permute
@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_split_grads_matches_list_filtering_and_keeps_the_row_sums(seed):
    """split() of Algorithm 2's Backward against plain list filtering, and against what it is for: the summed
    gradient of every row, taken from the part its row went to, equals the sum taken over the whole batch bit for
    bit (each part keeps batch order, so the additions are the same ones)."""
    rng = np.random.default_rng(100 + seed)
    rows, n, dim = 40, int(rng.integers(1, 300)), 4 * int(rng.integers(1, 5))
    values = rng.integers(0, rows, size=n).astype(np.int64)
    nxt = np.unique(rng.integers(0, rows, size=int(rng.integers(0, 60)))).astype(np.int64)
    grads = rng.standard_normal((n, dim)).astype(np.float32)
    r = O.split_grads(grads, values, nxt)
    members = set(int(x) for x in nxt)
    co = [j for j in range(n) if int(values[j]) in members]
    ex = [j for j in range(n) if int(values[j]) not in members]
    assert r["co_index"].tolist() == co and r["ex_index"].tolist() == ex
    assert r["g_co"].tobytes() == grads[co].tobytes() if co else r["g_co"].shape[0] == 0
    assert r["g_ex"].tobytes() == grads[ex].tobytes() if ex else r["g_ex"].shape[0] == 0
    # reduce(co part) and reduce(ex part) together are reduce(all)
    lay = O.unique_ids(values, rows)
    whole = O.segment_reduce_grads(grads, lay["perm"], lay["seg_offsets"])
    seen = 0
    for idx, g in ((r["co_index"], r["g_co"]), (r["ex_index"], r["g_ex"])):
        if len(idx) == 0:
            continue
        lay_p = O.unique_ids(values[idx], rows)
        red_p = O.segment_reduce_grads(g, lay_p["perm"], lay_p["seg_offsets"])
        slot = np.searchsorted(lay["unique"], lay_p["unique"])
        assert np.array_equal(lay["unique"][slot], lay_p["unique"])
        assert red_p.tobytes() == whole[slot].tobytes()
        seen += len(lay_p["unique"])
    assert seen == lay["n_unique"]                       # every row is in exactly one part


def test_split_grads_degenerate_cases():
    grads = np.arange(12, dtype=np.float32).reshape(3, 4)
    values = np.array([5, 2, 5], dtype=np.int64)
    r = O.split_grads(grads, values, np.empty(0, np.int64))           # no lookahead batch: everything exclusive
    assert r["co_index"].tolist() == [] and r["ex_index"].tolist() == [0, 1, 2] and r["g_ex"].tobytes() == grads.tobytes()
    r = O.split_grads(grads, values, np.array([2, 5, 9], dtype=np.int64))   # everything collides
    assert r["co_index"].tolist() == [0, 1, 2] and r["ex_index"].tolist() == [] and r["g_co"].tobytes() == grads.tobytes()
    r = O.split_grads(grads, values, np.array([5], dtype=np.int64))
    assert r["co_index"].tolist() == [0, 2] and r["ex_index"].tolist() == [1]
    with pytest.raises(O.OracleError):
        O.split_grads(grads, values, np.array([5, 2], dtype=np.int64))      # membership list not ascending


def test_fbs_zigzag_matches_the_printed_pattern():
    want = {}
    with open(os.path.join(GOLDEN, "fbs_zigzag_pattern.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            cols = [int(x) for x in line.split()]
            want[cols[0]] = cols[1:]
    lengths = np.arange(18, dtype=np.int64) * 3 + 5          # already sorted: sample index == sorted position
    sample_of, rank_offsets = O.partition_fbs(lengths, 4)
    for rank, positions in want.items():
        assert sample_of[rank_offsets[rank]:rank_offsets[rank + 1]].tolist() == positions


def _fbs_by_rounds(lengths, n):
    """The same partition told by rounds: cut the sorted list into blocks of n, reverse every second block,
    and give the c-th entry of a block to rank c (a short last block, reversed, ends at rank n-1)."""
    order = sorted(range(len(lengths)), key=lambda b: (int(lengths[b]), b))
    ranks = [[] for _ in range(n)]
    for r in range(0, (len(order) + n - 1) // n):
        block = order[r * n:(r + 1) * n]
        if r % 2 == 0:
            for c, smp in enumerate(block):
                ranks[c].append(smp)
        else:
            for c, smp in enumerate(block):
                ranks[n - 1 - c].append(smp)
    return ranks


@pytest.mark.parametrize("B,n", [(16, 4), (64, 8), (37, 5), (3, 8), (0, 4), (1, 1), (100, 1), (257, 16)])
def test_fbs_partition_is_a_balanced_bijection(B, n):
    rng = np.random.default_rng(B * 31 + n)
    lengths = rng.integers(0, 50, size=B).astype(np.int64)            # many ties
    sample_of, rank_offsets = O.partition_fbs(lengths, n)
    assert sorted(sample_of.tolist()) == list(range(B))
    assert rank_offsets[0] == 0 and rank_offsets[n] == B
    ranks = [sample_of[rank_offsets[i]:rank_offsets[i + 1]].tolist() for i in range(n)]
    assert ranks == _fbs_by_rounds(lengths, n)
    sizes = [len(r) for r in ranks]
    assert max(sizes) - min(sizes) <= 1
    if B % n == 0 and B > 0:
        # equal sample counts, and the summed lengths of two ranks differ by at most the spread of the
        # lengths (the ranges of the double rounds telescope)
        assert len(set(sizes)) == 1
        totals = [int(lengths[r].sum()) for r in ranks]
        assert max(totals) - min(totals) <= int(lengths.max() - lengths.min())
    with pytest.raises(O.OracleError):
        O.partition_fbs(np.array([3, -1], dtype=np.int64), 2)


def test_fbs_beats_contiguous_blocks_on_skewed_lengths():
    # what the zig-zag is for: sorted blocks would put all long samples on the last rank
    rng = np.random.default_rng(9)
    lengths = np.sort((rng.pareto(1.5, size=256) * 16 + 16).astype(np.int64).clip(16, 4096))
    sample_of, ro = O.partition_fbs(lengths, 8)
    totals = [int(lengths[sample_of[ro[i]:ro[i + 1]]].sum()) for i in range(8)]
    blocks = [int(lengths[i * 32:(i + 1) * 32].sum()) for i in range(8)]
    assert max(totals) - min(totals) <= int(lengths.max() - lengths.min())
    assert max(blocks) - min(blocks) > 3 * (max(totals) - min(totals))


@pytest.mark.parametrize("seed", [0, 1])
def test_indexed_permute_matches_list_concatenation(seed):
    rng = np.random.default_rng(700 + seed)
    B = 23
    lens = rng.integers(0, 9, size=B)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    values = rng.integers(0, 10**12, size=int(offsets[-1])).astype(np.int64)
    for sample_of in (rng.permutation(B).astype(np.int32), np.array([5, 5, 0], dtype=np.int32), np.empty(0, np.int32)):
        out, out_offsets = O.jagged_indexed_permute(values, offsets, sample_of)
        pieces = [values[offsets[p]:offsets[p + 1]].tolist() for p in sample_of]
        assert out.tolist() == [x for piece in pieces for x in piece]
        assert out_offsets.tolist() == [0] + list(np.cumsum([len(p) for p in pieces]))
    # rows instead of scalars
    rows = rng.standard_normal((int(offsets[-1]), 3)).astype(np.float32)
    perm = rng.permutation(B).astype(np.int32)
    out, _ = O.jagged_indexed_permute(rows, offsets, perm)
    assert np.array_equal(out, np.concatenate([rows[offsets[p]:offsets[p + 1]] for p in perm]))
    with pytest.raises(O.OracleError):
        O.jagged_indexed_permute(values, offsets, np.array([B], dtype=np.int32))


# ------------------------------------------- keyed transpose, ranged dispatch, ranged combine
def _kjt(rng, F, B, width=0):
    lens = rng.integers(0, 6, size=F * B)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    n = int(offsets[-1])
    values = rng.integers(0, 10**9, size=(n,) if width == 0 else (n, width)).astype(np.int64)
    segs = [[values[offsets[f * B + b]:offsets[f * B + b + 1]] for b in range(B)] for f in range(F)]   # [f][b]
    return values, offsets, segs


def _cat(pieces, like):
    pieces = list(pieces)
    return np.concatenate(pieces) if pieces else like[:0]


@pytest.mark.parametrize("F,B,width", [(3, 5, 0), (1, 7, 0), (4, 1, 2), (2, 0, 0), (6, 9, 3)])
def test_keyed_transpose_matches_nested_lists(F, B, width):
    rng = np.random.default_rng(F * 10 + B)
    values, offsets, segs = _kjt(rng, F, B, width)
    out, out_off = O.jagged_keyed_transpose(values, offsets, F, B)
    want = [segs[f][b] for b in range(B) for f in range(F)]
    assert np.array_equal(out, _cat(want, values))
    assert out_off.tolist() == [0] + list(np.cumsum([len(x) for x in want]))
    # transposing back (the roles of keys and samples swapped) gives the input
    back, back_off = O.jagged_keyed_transpose(out, out_off, B, F)
    assert np.array_equal(back, values) and back_off.tolist() == offsets.tolist()


@pytest.mark.parametrize("F,B,cuts", [(3, 10, [0, 4, 4, 7, 10]), (1, 6, [0, 2, 6]), (2, 5, [0, 5]), (4, 8, [0, 1, 2, 3, 8])])
def test_ranged_dispatch_and_combine_match_nested_lists_and_undo_each_other(F, B, cuts):
    rng = np.random.default_rng(F * 100 + B)
    values, offsets, segs = _kjt(rng, F, B, 0)
    ro = np.array(cuts, dtype=np.int64)
    out, out_off, splits = O.jagged_ranged_dispatch(values, offsets, F, B, ro)
    per_rank = [[segs[f][b] for f in range(F) for b in range(cuts[r], cuts[r + 1])] for r in range(len(cuts) - 1)]
    want = [x for rank in per_rank for x in rank]
    assert np.array_equal(out, _cat(want, values))
    assert out_off.tolist() == [0] + list(np.cumsum([len(x) for x in want]))
    assert splits.tolist() == [sum(len(x) for x in rank) for rank in per_rank]
    back, back_off = O.jagged_ranged_combine(out, out_off, F, B, ro)
    assert np.array_equal(back, values) and back_off.tolist() == offsets.tolist()
    if F == 1:
        # one key: what every rank is sent already lies in rank order
        assert np.array_equal(out, values) and out_off.tolist() == offsets.tolist()
    with pytest.raises(O.OracleError):
        O.jagged_ranged_dispatch(values, offsets, F, B, np.array([0, B + 1], dtype=np.int64))
    with pytest.raises(O.OracleError):
        O.jagged_ranged_combine(values, offsets, F, B, np.array([0, 3, 2, B], dtype=np.int64))


# ----------------------------------------------------------------------- VBS partitioner
def _vbs_brute(lengths, weights, n):
    order = sorted(range(len(lengths)), key=lambda b: (int(lengths[b]), b))
    total = sum(int(weights[lengths[b]]) for b in order)
    ranks, before = [[] for _ in range(n)], 0
    for b in order:
        r = min(n - 1, n * before // total) if total > 0 else 0          # Python integers: exact
        ranks[r].append(b)
        before += int(weights[lengths[b]])
    return order, ranks


@pytest.mark.parametrize("B,n,alpha", [(40, 4, 1.0), (257, 8, 1.7), (5, 8, 2.0), (0, 3, 1.0), (100, 1, 1.3), (64, 64, 0.5)])
def test_vbs_partition_matches_exact_integer_brute_force(B, n, alpha):
    rng = np.random.default_rng(B * 13 + n)
    max_len = 300
    lengths = rng.integers(0, max_len + 1, size=B).astype(np.int64)
    weights = np.round(np.arange(max_len + 1, dtype=np.float64) ** alpha * 1024).astype(np.int64)
    sample_of, ro = O.partition_vbs(lengths, weights, n)
    order, ranks = _vbs_brute(lengths, weights, n)
    assert sample_of.tolist() == order
    assert [sample_of[ro[r]:ro[r + 1]].tolist() for r in range(n)] == ranks
    assert ro[0] == 0 and ro[n] == B and np.all(np.diff(ro) >= 0)
    if B:
        # every rank within one sample's weight of its share of the total
        w = weights[lengths]
        share = w.sum() / n
        for r in range(n):
            assert w[sample_of[ro[r]:ro[r + 1]]].sum() <= share + w.max() + 1


def test_vbs_special_cases():
    lengths = np.array([9, 3, 3, 7, 1, 5, 5, 2], dtype=np.int64)
    # equal weights: the sorted order cut into equal runs
    ones = np.ones(10, dtype=np.int64)
    sample_of, ro = O.partition_vbs(lengths, ones, 4)
    assert sample_of.tolist() == [4, 7, 1, 2, 5, 6, 3, 0] and ro.tolist() == [0, 2, 4, 6, 8]
    # weight = length (alpha = 1): total 35 over 2 ranks, the cut falls where the running weight reaches 17.5
    ident = np.arange(10, dtype=np.int64)
    sample_of, ro = O.partition_vbs(lengths, ident, 2)
    run = np.cumsum(lengths[sample_of]) - lengths[sample_of]
    assert ro.tolist() == [0, int(np.searchsorted(run * 2, 35, side="left")), 8] == [0, 6, 8]
    # all weights zero: one rank takes everything; heavier long samples: fewer of them per rank
    _, ro = O.partition_vbs(lengths, np.zeros(10, dtype=np.int64), 3)
    assert ro.tolist() == [0, 8, 8, 8]
    sq = ident ** 2
    _, ro = O.partition_vbs(lengths, sq, 2)
    assert ro[1] - ro[0] > ro[2] - ro[1]
    with pytest.raises(O.OracleError):
        O.partition_vbs(np.array([11], dtype=np.int64), ident, 2)
