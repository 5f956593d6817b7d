"""GPU parity: every C-ABI operation against the CPU oracle, element by element.

Bars: bit-exact for gathers, distinct IDs, segment layout, permutation, inverse map and the
collision partition; |gpu - ref| <= 1e-6 + 1e-5*|ref| for fp32 reduced gradients, Adagrad state
and updated rows; bf16 rows within one bf16 ulp.
"""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_24073_amd as fs
from fs_workloads import CONFIGS, make_iterations
from helpers import (assert_close_f32, assert_rows_close, dev, table_to_dev, table_to_host)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = fs.Context(max_ids=600_000, max_dim=256)
    yield c
    c.close()


def zipf_ids(rng, n, num_rows, a=1.2):
    ranks = np.minimum(rng.zipf(a, size=n), num_rows) - 1
    return ((ranks * 2654435761) % num_rows).astype(np.int64)


def rand_table(rng, rows, dim, dtype):
    """fp32 array, or uint16 array of bf16 bit patterns."""
    w = (rng.standard_normal((rows, dim)) * 0.05).astype(np.float32)
    if dtype == "f32":
        return w
    return torch.from_numpy(w).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


# ------------------------------------------------------------------------------------ gather
@pytest.mark.parametrize("dim,dtype", [(64, "f32"), (128, "f32"), (256, "f32"), (4, "f32"), (20, "f32"),
                                       (128, "bf16"), (8, "bf16"), (256, "bf16"), (72, "bf16")])
@pytest.mark.parametrize("n_users,max_len", [(1, 1), (7, 5), (33, 70), (64, 300)])
def test_gather_bit_exact(ctx, dim, dtype, n_users, max_len):
    rng = np.random.default_rng(dim * 1000 + n_users)
    rows = 5000
    table = rand_table(rng, rows, dim, dtype)
    lens = rng.integers(0, max_len + 1, size=n_users)          # empty sequences included
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    values = zipf_ids(rng, int(offsets[-1]), rows)
    want = O.gather_jagged(table, values, offsets)
    got = fs.fs_gather_jagged(ctx, table_to_dev(table), dev(values), dev(offsets))
    assert fs.fs_check_async(ctx) == fs.FS_OK
    assert table_to_host(got).tobytes() == want.tobytes()


def test_gather_flags_bad_ids_and_offsets_without_faulting(ctx):
    rng = np.random.default_rng(1)
    table = rand_table(rng, 100, 64, "f32")
    values = np.array([5, 100, 7, -1, 99], dtype=np.int64)
    offsets = np.array([0, 2, 5], dtype=np.int64)
    got = table_to_host(fs.fs_gather_jagged(ctx, table_to_dev(table), dev(values), dev(offsets)))
    assert fs.fs_check_async(ctx) == fs.FS_ERANGE
    assert "row id out of range" in ctx.last_error()
    assert np.array_equal(got[[0, 2, 4]], table[[5, 7, 99]])
    assert np.all(got[[1, 3]] == 0)
    assert fs.fs_check_async(ctx) == fs.FS_OK                          # flags were cleared
    bad_offsets = np.array([0, 3, 2, 5], dtype=np.int64)
    fs.fs_gather_jagged(ctx, table_to_dev(table), dev(np.array([1, 2, 3, 4, 5], dtype=np.int64)), dev(bad_offsets))
    assert fs.fs_check_async(ctx) == fs.FS_ERANGE
    assert "malformed offsets" in ctx.last_error()


def test_host_visible_errors(ctx):
    t = torch.zeros((10, 64), device="cuda")
    v = torch.zeros(4, dtype=torch.int64, device="cuda")
    with pytest.raises(fs.FreeScaleError) as e:
        fs.fs_gather_jagged(ctx, torch.zeros((10, 6), device="cuda"), v, None)       # dim % 4
    assert e.value.code == fs.FS_EINVAL
    with pytest.raises(fs.FreeScaleError) as e:
        fs.fs_unique_ids(ctx, torch.zeros(ctx.max_ids + 1, dtype=torch.int64, device="cuda"), 10)
    assert e.value.code == fs.FS_ENOMEM
    lib = ctx.lib
    assert lib.fs_gather_jagged(ctx.handle, None, 10, 64, 0, v.data_ptr(), None, 0, 4, t.data_ptr(), None) == fs.FS_EINVAL
    assert lib.fs_gather_jagged(ctx.handle, t.data_ptr(), 10, 64, 7, v.data_ptr(), None, 0, 4, t.data_ptr(), None) == fs.FS_EINVAL
    assert lib.fs_gather_jagged(ctx.handle, t.data_ptr(), 10, 64, 0, v.data_ptr(), None, 0, -1, t.data_ptr(), None) == fs.FS_EINVAL
    assert lib.fs_gather_jagged(ctx.handle, None, 10, 64, 0, None, None, 0, 0, None, None) == fs.FS_OK   # n == 0 no-op
    assert "gather" in ctx.last_error()


def test_row_read_calibration_kernel_reads_the_rows_it_is_given(ctx):
    """fs_stream_row_read (a measurement aid): the folded word of one wavefront is the xor of every 32-bit word of
    the rows it was pointed at."""
    rng = np.random.default_rng(2)
    rows = rng.integers(0, 2**31, size=(500, 128), dtype=np.int64).astype(np.int32)
    index = rng.integers(0, 500, size=37).astype(np.int64)
    sink = torch.zeros(1024, dtype=torch.int32, device="cuda")
    fs.fs_stream_row_read(ctx, dev(rows), dev(index), sink)
    torch.cuda.synchronize()
    want = np.bitwise_xor.reduce(rows[index].reshape(-1))
    assert int(sink[0].item()) == int(want)


# ------------------------------------------------------------------------------------ unique
def check_unique(ctx, ids, num_rows):
    want = O.unique_ids(ids, num_rows)
    got = fs.fs_unique_ids(ctx, dev(ids), num_rows)
    assert fs.fs_check_async(ctx) == fs.FS_OK
    u = int(got["n_unique"].item())
    n = len(ids)
    assert u == want["n_unique"]
    assert np.array_equal(got["unique"][:u].cpu().numpy(), want["unique"])
    assert np.array_equal(got["seg_offsets"][:u + 1].cpu().numpy(), want["seg_offsets"])
    assert np.array_equal(got["perm"][:n].cpu().numpy(), want["perm"])
    assert np.array_equal(got["inverse"][:n].cpu().numpy(), want["inverse"])
    return got, want


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 2047, 2048, 2049, 5000, 70001])
@pytest.mark.parametrize("num_rows", [1, 100, 10_000, 4_000_000, 64_000_000])
def test_unique_bit_exact(ctx, n, num_rows):
    rng = np.random.default_rng(n * 7 + num_rows % 1000)
    check_unique(ctx, zipf_ids(rng, n, num_rows), num_rows)


@pytest.mark.parametrize("n", [1, 300, 9000])
def test_unique_wide_keys(ctx, n):
    rng = np.random.default_rng(n)
    pool = rng.integers(0, 2**62, size=max(n // 3, 1), dtype=np.int64)
    ids = pool[rng.integers(0, len(pool), size=n)]
    check_unique(ctx, ids, 0)                                   # 63-bit keys
    check_unique(ctx, ids % (2**35), 2**35)                     # 64-bit key path, bounded


def test_unique_degenerate(ctx):
    check_unique(ctx, np.full(5000, 42, dtype=np.int64), 100)            # one distinct row
    check_unique(ctx, np.arange(5000, dtype=np.int64)[::-1].copy(), 5000)  # all distinct, descending
    got = fs.fs_unique_ids(ctx, torch.empty(0, dtype=torch.int64, device="cuda"), 100)
    assert int(got["n_unique"].item()) == 0 and int(got["seg_offsets"][0].item()) == 0


def test_unique_flags_out_of_range_ids(ctx):
    ids = np.array([3, 200, 5], dtype=np.int64)
    fs.fs_unique_ids(ctx, dev(ids), 100)
    assert fs.fs_check_async(ctx) == fs.FS_ERANGE


# ------------------------------------------------------------------------------------ split
def check_split(ctx, u_t, u_t1):
    want = O.collision_split(u_t, u_t1)
    nt, nt1 = len(u_t), len(u_t1)
    d_ut = dev(u_t) if nt else None
    d_ut1 = dev(u_t1) if nt1 else None
    d_nt = dev(np.array([nt], dtype=np.int64)) if nt else None
    d_nt1 = dev(np.array([nt1], dtype=np.int64)) if nt1 else None
    # capacities larger than the counts: the launch is sized by the cap, the data by the device scalar
    pad = lambda t, k: None if t is None else torch.cat([t, torch.full((k,), -7, dtype=t.dtype, device="cuda")])
    got = fs.fs_collision_split(ctx, pad(d_ut, 37), d_nt, pad(d_ut1, 1500), d_nt1, nt + 37 if nt else 0,
                                nt1 + 1500 if nt1 else 0)
    counts = got["counts"].cpu().numpy()
    assert counts.tolist() == [len(want["co"]), len(want["ex"]), len(want["ex_next"])]
    for name, cnt in (("co", counts[0]), ("ex", counts[1]), ("ex_next", counts[2])):
        assert np.array_equal(got[name][:cnt].cpu().numpy(), want[name]), name
        assert np.array_equal(got[name + "_slot"][:cnt].cpu().numpy(), want[name + "_slot"]), name


@pytest.mark.parametrize("n0,n1,rows", [(1, 1, 2), (50, 80, 40), (3000, 2500, 3000), (70000, 90000, 200000),
                                        (1024, 1024, 5000), (1025, 1023, 800)])
def test_split_bit_exact(ctx, n0, n1, rows):
    rng = np.random.default_rng(n0 + n1)
    u_t = np.unique(zipf_ids(rng, n0, rows))
    u_t1 = np.unique(zipf_ids(rng, n1, rows))
    check_split(ctx, u_t, u_t1)


def test_split_degenerate(ctx):
    a = np.array([1, 5, 9, 12], dtype=np.int64)
    check_split(ctx, a, a)                                         # everything collides
    check_split(ctx, a, a + 100)                                   # nothing collides
    check_split(ctx, a, np.empty(0, dtype=np.int64))               # no lookahead batch
    check_split(ctx, np.empty(0, dtype=np.int64), a)               # nothing to update
    check_split(ctx, np.empty(0, dtype=np.int64), np.empty(0, dtype=np.int64))


@pytest.mark.parametrize("n_t", [5, 1024, 1025, 3000])
def test_split_at_the_top_of_the_id_range(ctx, n_t):
    """Table size not given: IDs run up to 2^63 - 1.  The largest IDs are the last elements of the last tile
    of either list (a tile is 1024 rows), where the window search must not step past the largest ID."""
    top = 2**63 - 1
    rng = np.random.default_rng(n_t)
    low = np.unique(rng.integers(0, 2**62, size=n_t, dtype=np.int64))[:max(n_t - 4, 0)]
    u_t = np.concatenate([low, np.array([top - 5, top - 2, top - 1, top], dtype=np.int64)])[-n_t:]
    u_t1 = np.concatenate([low[::2], np.array([top - 4, top - 2, top], dtype=np.int64)])
    check_split(ctx, u_t, u_t1)
    check_split(ctx, u_t1, u_t)
    check_split(ctx, u_t, u_t)
    # and through the dedup: 63-bit keys with the largest values present
    ids = np.concatenate([u_t[-3:], u_t[rng.integers(0, len(u_t), size=4000)], np.array([top, top], dtype=np.int64)])
    check_unique(ctx, ids, 0)


# ------------------------------------------------------------------------------------ reduce
def check_reduce(ctx, ids, grads, num_rows):
    lay = O.unique_ids(ids, num_rows)
    want = O.segment_reduce_grads(grads, lay["perm"], lay["seg_offsets"])
    d_grads, d_perm, d_seg = dev(grads), dev(lay["perm"]), dev(lay["seg_offsets"])
    d_nu = dev(np.array([lay["n_unique"]], dtype=np.int64))
    got = fs.fs_segment_reduce_grads(ctx, d_grads, d_perm, d_seg, d_nu)
    torch.cuda.synchronize()
    assert_close_f32(got[:lay["n_unique"]].cpu().numpy(), want, "reduced gradients")
    # the optional inverse map only changes how a wavefront finds its segments, not a single bit
    got_inv = fs.fs_segment_reduce_grads(ctx, d_grads, d_perm, d_seg, d_nu, inverse=dev(lay["inverse"]))
    torch.cuda.synchronize()
    assert torch.equal(got[:lay["n_unique"]], got_inv[:lay["n_unique"]])
    return got[:lay["n_unique"]]


@pytest.mark.parametrize("dim", [4, 20, 64, 128, 256])
@pytest.mark.parametrize("n", [1, 127, 128, 129, 1000, 20011])
def test_reduce_matches_oracle(ctx, dim, n):
    rng = np.random.default_rng(dim + n)
    rows = 3000
    ids = zipf_ids(rng, n, rows, a=1.15)
    grads = rng.standard_normal((n, dim)).astype(np.float32)
    check_reduce(ctx, ids, grads, rows)


@pytest.mark.parametrize("dim", [64, 128])
def test_reduce_long_segments_and_chunk_aligned_cuts(ctx, dim):
    rng = np.random.default_rng(9)
    # one row with every occurrence (spans dozens of chunks)
    n = 5000
    check_reduce(ctx, np.full(n, 3, dtype=np.int64), rng.standard_normal((n, dim)).astype(np.float32), 10)
    # segments that start exactly on chunk borders: 128 / 256 / 384 occurrences back to back
    ids = np.concatenate([np.full(128, 1), np.full(256, 2), np.full(384, 3), np.full(5, 4), np.full(123, 5),
                          np.full(1, 6), np.full(127, 7), np.full(128, 8)]).astype(np.int64)
    perm = rng.permutation(len(ids))
    check_reduce(ctx, ids[perm], rng.standard_normal((len(ids), dim)).astype(np.float32), 10)
    # all distinct
    ids = rng.permutation(3000).astype(np.int64)
    check_reduce(ctx, ids, rng.standard_normal((3000, dim)).astype(np.float32), 3000)


def test_reduce_cancellation_needs_wide_accumulation(ctx):
    # large cancelling terms around small ones: fp32 accumulation would miss the 1e-6 absolute bar
    rng = np.random.default_rng(4)
    n, dim = 4096, 64
    big = (rng.standard_normal((n // 2, dim)) * 1e4).astype(np.float32)
    grads = np.concatenate([big, -big, rng.standard_normal((100, dim)).astype(np.float32) * 1e-3])
    ids = np.zeros(len(grads), dtype=np.int64)
    check_reduce(ctx, ids, grads[rng.permutation(len(grads))], 5)


def test_reduce_is_reproducible(ctx):
    rng = np.random.default_rng(12)
    n, dim = 30000, 128
    ids = zipf_ids(rng, n, 2000)
    grads = rng.standard_normal((n, dim)).astype(np.float32)
    a = check_reduce(ctx, ids, grads, 2000).clone()
    b = check_reduce(ctx, ids, grads, 2000)
    assert torch.equal(a, b)


# ------------------------------------------------------------------------------------ adagrad
@pytest.mark.parametrize("dim,dtype", [(64, "f32"), (128, "f32"), (256, "f32"), (4, "f32"), (20, "f32"),
                                       (128, "bf16"), (8, "bf16"), (72, "bf16")])
def test_adagrad_matches_oracle(ctx, dim, dtype):
    rng = np.random.default_rng(dim)
    rows, n_upd = 4000, 1777
    table = rand_table(rng, rows, dim, dtype)
    state = (rng.random(rows) * 0.5).astype(np.float32)
    reduced = rng.standard_normal((2500, dim)).astype(np.float32)
    upd_rows = np.sort(rng.choice(rows, size=n_upd, replace=False)).astype(np.int64)
    slots = rng.permutation(2500)[:n_upd].astype(np.int32)
    t_ref, s_ref = table.copy(), state.copy()
    O.rowwise_adagrad_update(t_ref, s_ref, upd_rows, slots, reduced, 0.01, 1e-8)
    d_table, d_state = table_to_dev(table), dev(state)
    # the list is longer than the count: entries past the device count must be ignored
    junk = np.full(50, 3, dtype=np.int64)
    fs.fs_rowwise_adagrad_update(ctx, d_table, d_state, dev(np.concatenate([upd_rows, junk])),
                                 dev(np.concatenate([slots, np.zeros(50, np.int32)])),
                                 dev(np.array([n_upd], dtype=np.int64)), n_upd + 50, dev(reduced), 0.01, 1e-8)
    assert fs.fs_check_async(ctx) == fs.FS_OK
    got_t, got_s = table_to_host(d_table), d_state.cpu().numpy()
    assert_close_f32(got_s, s_ref, "adagrad state")
    assert_rows_close(got_t, t_ref, "updated rows")
    untouched = np.setdiff1d(np.arange(rows), upd_rows)
    assert got_t[untouched].tobytes() == table[untouched].tobytes()
    assert got_s[untouched].tobytes() == state[untouched].tobytes()


def test_adagrad_skips_out_of_range_rows(ctx):
    table = np.ones((10, 64), np.float32); state = np.zeros(10, np.float32)
    d_table, d_state = dev(table), dev(state)
    fs.fs_rowwise_adagrad_update(ctx, d_table, d_state, dev(np.array([2, 10, -3], dtype=np.int64)),
                                 dev(np.array([0, 1, 2], dtype=np.int32)), dev(np.array([3], dtype=np.int64)), 3,
                                 dev(np.ones((3, 64), np.float32)), 0.01, 1e-8)
    assert fs.fs_check_async(ctx) == fs.FS_ERANGE
    got = d_table.cpu().numpy()
    assert np.all(got[2] != 1.0) and np.all(np.delete(got, 2, axis=0) == 1.0)


# ------------------------------------------------------------------------------------ class order, fused pass
def class_order_from_oracle(layout, sp):
    """Class order written out from the oracle's layout and split, rows with more than
    FS_SHORT_SEGMENT occurrences only: collision rows' occurrences first, then the exclusive rows';
    inside a class by ascending row, inside a row in batch order.  cstart is -1 for other rows."""
    seg, perm = layout["seg_offsets"].astype(np.int64), layout["perm"]
    cperm, cslot, cstart = [], [], np.full(len(layout["unique"]), -1, np.int32)
    pos = 0
    n_class0 = 0
    for slots in (sp["co_slot"], sp["ex_slot"]):
        for s in slots:
            if seg[s + 1] - seg[s] <= fs.FS_SHORT_SEGMENT:
                continue
            cstart[s] = pos
            cperm.append(perm[seg[s]:seg[s + 1]])
            cslot.append(np.full(seg[s + 1] - seg[s], s, np.int32))
            pos += seg[s + 1] - seg[s]
        if slots is sp["co_slot"]:
            n_class0 = pos
    cat = lambda xs: np.concatenate(xs) if xs else np.empty(0, np.int32)
    return cat(cperm), cat(cslot), cstart, [n_class0, pos]


def gpu_layout_and_classes(ctx, ids_t, ids_t1, num_rows):
    lay = fs.fs_unique_ids(ctx, dev(ids_t), num_rows)
    if ids_t1 is None:
        sp = fs.fs_collision_split_classes(ctx, lay, None, None, 0)
    else:
        lay1 = fs.fs_unique_ids(ctx, dev(ids_t1), num_rows)
        sp = fs.fs_collision_split_classes(ctx, lay, lay1["unique"], lay1["n_unique"], len(ids_t1))
    return lay, sp


@pytest.mark.parametrize("n0,n1,rows", [(1, 1, 2), (50, 80, 40), (3000, 2500, 3000), (70000, 90000, 200000),
                                        (5000, 0, 1000), (4096, 4096, 100)])
def test_class_order_bit_exact(ctx, n0, n1, rows):
    rng = np.random.default_rng(n0 * 7 + n1)
    ids_t = zipf_ids(rng, n0, rows, a=1.1)
    ids_t1 = zipf_ids(rng, n1, rows, a=1.1) if n1 else None
    lay_o = O.unique_ids(ids_t, rows)
    sp_o = O.collision_split(lay_o["unique"], O.unique_ids(ids_t1, rows)["unique"] if n1 else np.empty(0, np.int64))
    want = class_order_from_oracle(lay_o, sp_o)
    lay, sp = gpu_layout_and_classes(ctx, ids_t, ids_t1, rows)
    assert fs.fs_check_async(ctx) == fs.FS_OK
    assert sp["class_pos"].cpu().numpy().tolist() == want[3]
    n_pos = want[3][1]
    assert np.array_equal(sp["cperm"][:n_pos].cpu().numpy(), want[0])
    assert np.array_equal(sp["cslot"][:n_pos].cpu().numpy(), want[1])
    in_order = want[2] >= 0
    assert np.array_equal(sp["cstart"][:len(want[2])].cpu().numpy()[in_order], want[2][in_order])
    for name in ("co", "ex"):
        cnt = len(sp_o[name])
        assert np.array_equal(sp[name][:cnt].cpu().numpy(), sp_o[name])
    # one record per row, at the row's place in its class list
    rec = sp["short_rec"][:2 * 12 * n0].cpu().numpy().reshape(2, n0, 12)
    seg = lay_o["seg_offsets"].astype(np.int64)
    for cls, name in enumerate(("co", "ex")):
        rows_c, slots_c = sp_o[name], sp_o[name + "_slot"]
        got = rec[cls, :len(rows_c)]
        assert np.array_equal(got[:, 0:2].copy().view(np.int64).ravel(), rows_c)
        assert np.array_equal(got[:, 2], slots_c)
        lens = (seg[slots_c + 1] - seg[slots_c]).astype(np.int32)
        assert np.array_equal(got[:, 3], lens)
        for li in np.nonzero(lens <= fs.FS_SHORT_SEGMENT)[0]:
            s_ = slots_c[li]
            assert np.array_equal(got[li, 4:4 + lens[li]], lay_o["perm"][seg[s_]:seg[s_ + 1]])


def check_fused(ctx, rng, ids_t, ids_t1, rows, dim, dtype, n_passes=1):
    table = rand_table(rng, rows, dim, dtype)
    state = (rng.random(rows) * 0.1).astype(np.float32)
    d_table, d_state = table_to_dev(table), dev(state)
    t_ref, s_ref = table.copy(), state.copy()
    for _ in range(n_passes):
        grads = rng.standard_normal((len(ids_t), dim)).astype(np.float32)
        lay_o = O.unique_ids(ids_t, rows)
        red_o = O.segment_reduce_grads(grads, lay_o["perm"], lay_o["seg_offsets"])
        u = len(lay_o["unique"])
        O.rowwise_adagrad_update(t_ref, s_ref, lay_o["unique"], np.arange(u, dtype=np.int32), red_o, 0.02, 1e-8)
        lay, sp = gpu_layout_and_classes(ctx, ids_t, ids_t1, rows)
        reduced = torch.full((max(len(ids_t), 1), dim), float("nan"), dtype=torch.float32, device="cuda")
        for cls in (1, 0):
            fs.fs_reduce_update_class(ctx, cls, d_table, d_state, 0.02, 1e-8, dev(grads), lay, sp, reduced)
        assert fs.fs_check_async(ctx) == fs.FS_OK
        assert_close_f32(reduced[:u].cpu().numpy(), red_o, "reduced gradients of the fused pass")
    assert_close_f32(d_state.cpu().numpy(), s_ref, "adagrad state after the fused passes")
    assert_rows_close(table_to_host(d_table), t_ref, "rows after the fused passes")


@pytest.mark.parametrize("dim,dtype", [(128, "f32"), (64, "f32"), (256, "f32"), (4, "f32"), (20, "f32"), (32, "f32"),
                                       (128, "bf16"), (8, "bf16"), (256, "bf16"), (72, "bf16")])
@pytest.mark.parametrize("n", [1, 63, 64, 65, 1000, 20011])
def test_fused_pass_matches_oracle(ctx, dim, dtype, n):
    rng = np.random.default_rng(dim * 31 + n)
    rows = 3000
    check_fused(ctx, rng, zipf_ids(rng, n, rows, a=1.15), zipf_ids(rng, n, rows, a=1.15), rows, dim, dtype)


@pytest.mark.parametrize("dim,dtype", [(128, "f32"), (64, "f32"), (128, "bf16")])
def test_fused_pass_long_segments_and_aligned_cuts(ctx, dim, dtype):
    """One row with thousands of occurrences (its pieces are added by whoever arrives last),
    segments that end exactly on a chunk border, a run of singletons; two launches in a row on the
    same context (the piece counters must be back at zero)."""
    rng = np.random.default_rng(9)
    rows = 500
    ids = np.concatenate([np.full(6000, 7), np.full(64, 8), np.full(128, 9), np.arange(100, 300),
                          np.full(63, 10), np.full(1, 11), np.full(2500, 12), np.arange(300, 364)]).astype(np.int64)
    ids = ids[rng.permutation(len(ids))]
    nxt = np.array([7, 9, 12, 150, 151, 152, 320, 499], dtype=np.int64)
    check_fused(ctx, rng, ids, nxt, rows, dim, dtype, n_passes=3)


def exact_sum_grads(rng, n, dim):
    """Gradients whose sums are exact in any order: multiples of 2^-4 in [-4, 4].  A sum over fewer than 2^13
    occurrences has at most 19 significant bits, its square 38, the sum of 256 squares 46: fp64 holds all of
    them exactly and the fp32 sum is exact too, so the order in which a kernel adds cannot show."""
    return (rng.integers(-64, 65, size=(n, dim)) / 16.0).astype(np.float32)


@pytest.mark.parametrize("dim,dtype", [(128, "f32"), (64, "f32"), (20, "f32"), (256, "f32"),
                                       (128, "bf16"), (256, "bf16"), (72, "bf16")])
@pytest.mark.parametrize("shape", ["one_occurrence_per_row", "long_and_cut_segments"])
def test_update_is_bit_exact_where_the_sums_are_exact(ctx, dim, dtype, shape):
    """Where the summed gradient does not depend on the order of addition, kernel and oracle do the same IEEE
    operations (fp64 sum of squares / dim rounded once, fp32 add, correctly rounded sqrt and divide, one
    rounding per product and difference, no contraction, round-to-nearest-even to bf16): table and state must
    agree bit for bit - for the stand-alone operations, for the record path of the fused pass (rows with one
    occurrence) and for its position-cut path (rows with thousands, pieces added by the last arriver)."""
    rng = np.random.default_rng(dim + len(shape))
    rows = 20_000
    if shape == "one_occurrence_per_row":
        ids = rng.permutation(rows)[:6000].astype(np.int64)
        nxt = np.concatenate([ids[::3], rng.permutation(rows)[:500]]).astype(np.int64)
    else:
        ids = np.concatenate([np.full(6000, 7), np.full(64, 8), np.full(128, 9), np.arange(100, 300),
                              np.full(63, 10), np.full(1, 11), np.full(2500, 12), np.arange(300, 364),
                              np.full(9, 13), np.full(8, 14)]).astype(np.int64)
        ids = ids[rng.permutation(len(ids))]
        nxt = np.array([7, 9, 12, 13, 150, 151, 152, 320, 499], dtype=np.int64)
    table = rand_table(rng, rows, dim, dtype)
    state = (rng.random(rows) * 0.1).astype(np.float32)
    d_fused, s_fused = table_to_dev(table), dev(state)       # fs_reduce_update_class, both classes
    d_alone, s_alone = table_to_dev(table), dev(state)       # fs_segment_reduce_grads + fs_rowwise_adagrad_update
    t_ref, s_ref = table.copy(), state.copy()
    lay_o = O.unique_ids(ids, rows)
    u = len(lay_o["unique"])
    lay, sp = gpu_layout_and_classes(ctx, ids, nxt, rows)
    for _ in range(2):                                       # twice: the second step starts from a grown state
        grads = exact_sum_grads(rng, len(ids), dim)
        red_o = O.segment_reduce_grads(grads, lay_o["perm"], lay_o["seg_offsets"])
        O.rowwise_adagrad_update(t_ref, s_ref, lay_o["unique"], np.arange(u, dtype=np.int32), red_o, 0.02, 1e-8)
        d_grads = dev(grads)
        reduced = torch.full((len(ids), dim), float("nan"), dtype=torch.float32, device="cuda")
        for cls in (0, 1):
            fs.fs_reduce_update_class(ctx, cls, d_fused, s_fused, 0.02, 1e-8, d_grads, lay, sp, reduced)
        red_alone = fs.fs_segment_reduce_grads(ctx, d_grads, lay["perm"], lay["seg_offsets"], lay["n_unique"])
        fs.fs_rowwise_adagrad_update(ctx, d_alone, s_alone, lay["unique"], dev(np.arange(u, dtype=np.int32)),
                                     lay["n_unique"], u, red_alone, 0.02, 1e-8)
        assert fs.fs_check_async(ctx) == fs.FS_OK
        assert reduced[:u].cpu().numpy().tobytes() == red_o.tobytes()
        assert red_alone[:u].cpu().numpy().tobytes() == red_o.tobytes()
    for what, d_t, d_s in (("fused pass", d_fused, s_fused), ("stand-alone operations", d_alone, s_alone)):
        assert d_s.cpu().numpy().tobytes() == s_ref.tobytes(), f"{what}: Adagrad state"
        assert table_to_host(d_t).tobytes() == t_ref.tobytes(), f"{what}: rows"


def test_fused_pass_without_lookahead_and_with_full_overlap(ctx):
    rng = np.random.default_rng(10)
    ids = zipf_ids(rng, 5000, 800, a=1.1)
    check_fused(ctx, rng, ids, None, 800, 128, "f32")           # every row exclusive
    check_fused(ctx, rng, ids, ids.copy(), 800, 128, "f32")     # every row a collision row


def test_fused_pass_is_reproducible(ctx):
    rng = np.random.default_rng(11)
    rows, dim, n = 2000, 128, 30000
    ids, ids1 = zipf_ids(rng, n, rows, a=1.05), zipf_ids(rng, n, rows, a=1.05)
    grads = dev(rng.standard_normal((n, dim)).astype(np.float32))
    table = rand_table(rng, rows, dim, "f32")
    results = []
    for _ in range(3):
        d_table, d_state = table_to_dev(table), torch.zeros(rows, device="cuda")
        lay, sp = gpu_layout_and_classes(ctx, ids, ids1, rows)
        for cls in (0, 1):
            fs.fs_reduce_update_class(ctx, cls, d_table, d_state, 0.01, 1e-8, grads, lay, sp)
        assert fs.fs_check_async(ctx) == fs.FS_OK
        results.append((d_table.cpu().numpy().tobytes(), d_state.cpu().numpy().tobytes()))
    assert results[0] == results[1] == results[2]


# ------------------------------------------------------------------------------------ whole step
def run_steps_gpu(ctx, table, state, its, lr, eps, mode="step"):
    """Runs every iteration of `its` (list of fs_workloads.Iteration) on the GPU.

    mode "step": fs_prioritized_step; "fused_calls": its building blocks one after another on one
    stream; "five_ops": the five plain operations (unfused reduce, then the two Adagrad passes).
    Returns the device table/state and, per iteration, the outputs copied to the host."""
    d_table, d_state = table_to_dev(table), dev(state)
    num_rows = table.shape[0]
    d_vals = [dev(it.values) for it in its]
    d_offs = [dev(it.offsets) for it in its]
    d_grads = [dev(it.grads) for it in its]
    layout = fs.fs_unique_ids(ctx, d_vals[0], num_rows)
    emb0 = fs.fs_gather_jagged(ctx, d_table, d_vals[0], d_offs[0])
    outs = [{"emb": table_to_host(emb0)}]
    for t in range(len(its)):
        last = t == len(its) - 1
        n_t = d_vals[t].numel()
        n_t1 = 0 if last else d_vals[t + 1].numel()
        layout_next = None if last else fs.alloc_layout(n_t1, "cuda")
        split = fs.alloc_split(n_t, n_t1, "cuda")
        reduced = torch.empty((max(n_t, 1), table.shape[1]), dtype=torch.float32, device="cuda")
        emb = None if last else torch.empty((n_t1, table.shape[1]), dtype=d_table.dtype, device="cuda")
        if mode == "step":
            args = fs.make_step_args(d_table, d_state, lr, eps, layout, d_grads[t], None if last else d_vals[t + 1],
                                     None if last else d_offs[t + 1], layout_next, split, reduced, emb)
            fs.fs_prioritized_step(ctx, args)
        elif mode == "fused_calls":
            if not last:
                fs.fs_unique_ids(ctx, d_vals[t + 1], num_rows, out=layout_next)
            layout["n"] = n_t
            fs.fs_collision_split_classes(ctx, layout, None if last else layout_next["unique"],
                                          None if last else layout_next["n_unique"], n_t1, out=split)
            for cls in (0, 1):
                fs.fs_reduce_update_class(ctx, cls, d_table, d_state, lr, eps, d_grads[t], layout, split, reduced)
            if not last:
                fs.fs_gather_jagged(ctx, d_table, d_vals[t + 1], d_offs[t + 1], out=emb)
        else:
            if not last:
                fs.fs_unique_ids(ctx, d_vals[t + 1], num_rows, out=layout_next)
            fs.fs_collision_split(ctx, layout["unique"], layout["n_unique"], None if last else layout_next["unique"],
                                  None if last else layout_next["n_unique"], n_t, n_t1, out=split)
            fs.fs_segment_reduce_grads(ctx, d_grads[t], layout["perm"], layout["seg_offsets"], layout["n_unique"], out=reduced)
            fs.fs_rowwise_adagrad_update(ctx, d_table, d_state, split["co"], split["co_slot"], split["counts"][0:1], n_t, reduced, lr, eps)
            fs.fs_rowwise_adagrad_update(ctx, d_table, d_state, split["ex"], split["ex_slot"], split["counts"][1:2], n_t, reduced, lr, eps)
            if not last:
                fs.fs_gather_jagged(ctx, d_table, d_vals[t + 1], d_offs[t + 1], out=emb)
        assert fs.fs_check_async(ctx) == fs.FS_OK
        u = int(layout["n_unique"].item())
        counts = split["counts"].cpu().numpy()
        rec = {"reduced": reduced[:u].cpu().numpy(), "counts": counts}
        for name, cnt in (("co", counts[0]), ("ex", counts[1]), ("ex_next", counts[2])):
            rec[name] = split[name][:cnt].cpu().numpy()
            rec[name + "_slot"] = split[name + "_slot"][:cnt].cpu().numpy()
        if not last:
            u1 = int(layout_next["n_unique"].item())
            rec["layout_next"] = {"unique": layout_next["unique"][:u1].cpu().numpy(),
                                  "seg_offsets": layout_next["seg_offsets"][:u1 + 1].cpu().numpy(),
                                  "perm": layout_next["perm"][:n_t1].cpu().numpy(),
                                  "inverse": layout_next["inverse"][:n_t1].cpu().numpy()}
            rec["emb_next"] = table_to_host(emb)
        outs.append(rec)
        layout = layout_next
    torch.cuda.synchronize()
    return d_table, d_state, outs


def run_steps_oracle(table, state, its, lr, eps):
    table, state = table.copy(), state.copy()
    num_rows = table.shape[0]
    layout = O.unique_ids(its[0].values, num_rows)
    outs = [{"emb": O.gather_jagged(table, its[0].values, its[0].offsets)}]
    for t in range(len(its)):
        last = t == len(its) - 1
        r = O.step(table, state, layout, its[t].grads, None if last else its[t + 1].values,
                   None if last else its[t + 1].offsets, lr, eps)
        outs.append(r)
        layout = r["layout_next"]
    return table, state, outs


def compare_runs(got_outs, want_outs, got_table, got_state, want_table, want_state):
    assert got_outs[0]["emb"].tobytes() == want_outs[0]["emb"].tobytes()
    for t, (g, w) in enumerate(zip(got_outs[1:], want_outs[1:])):
        sp = w["split"]
        assert g["counts"].tolist() == [len(sp["co"]), len(sp["ex"]), len(sp["ex_next"])], f"iteration {t}"
        for name in ("co", "ex", "ex_next"):
            assert np.array_equal(g[name], sp[name]), f"iteration {t} {name}"
            assert np.array_equal(g[name + "_slot"], sp[name + "_slot"]), f"iteration {t} {name}_slot"
        assert_close_f32(g["reduced"], w["reduced"], f"iteration {t} reduced gradients")
        if w["layout_next"] is not None:
            for k in ("unique", "seg_offsets", "perm", "inverse"):
                assert np.array_equal(g["layout_next"][k], w["layout_next"][k]), f"iteration {t} layout {k}"
            assert_rows_close(g["emb_next"], w["emb_next"], f"iteration {t} gathered rows")
    assert_close_f32(got_state, want_state, "final adagrad state")
    assert_rows_close(got_table, want_table, "final table")


@pytest.mark.parametrize("use_step_call", ["step", "fused_calls", "five_ops"])
def test_config0_tiny_full_run(ctx, use_step_call):
    cfg = CONFIGS[0]
    tab = cfg.tables[0]
    its = [x[0] for x in make_iterations(cfg)]
    rng = np.random.default_rng(0xF5CA1E00)
    table = (rng.standard_normal((tab.num_rows, tab.dim)) * 0.01).astype(np.float32)
    state = np.zeros(tab.num_rows, np.float32)
    d_table, d_state, got = run_steps_gpu(ctx, table, state, its, cfg.lr, cfg.eps, use_step_call)
    t_ref, s_ref, want = run_steps_oracle(table, state, its, cfg.lr, cfg.eps)
    compare_runs(got, want, table_to_host(d_table), d_state.cpu().numpy(), t_ref, s_ref)
    final = table_to_host(d_table)
    touched = np.union1d(its[0].values, its[1].values)
    untouched = np.setdiff1d(np.arange(tab.num_rows), touched)
    assert final[untouched].tobytes() == table[untouched].tobytes()


@pytest.mark.parametrize("dtype,dim", [("f32", 128), ("bf16", 128), ("f32", 64), ("f32", 256)])
def test_multi_iteration_schedule_matches_sequential_calls_bitwise(ctx, dtype, dim):
    """The two-stream schedule and its building blocks issued one after another give identical bits;
    the five plain operations (unfused, other summation grouping) agree within the tolerance."""
    rng = np.random.default_rng(77)
    rows = 20000
    table = rand_table(rng, rows, dim, dtype)
    state = np.zeros(rows, np.float32)

    class It:
        pass

    its = []
    for t in range(4):
        it = It()
        lens = rng.integers(0, 200, size=48)
        it.offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        it.values = zipf_ids(rng, int(it.offsets[-1]), rows, a=1.1)
        it.grads = rng.standard_normal((len(it.values), dim)).astype(np.float32)
        its.append(it)
    ta, sa, oa = run_steps_gpu(ctx, table, state, its, 0.01, 1e-8, "step")
    tb, sb, ob = run_steps_gpu(ctx, table, state, its, 0.01, 1e-8, "fused_calls")
    tc, sc, oc = run_steps_gpu(ctx, table, state, its, 0.01, 1e-8, "five_ops")
    assert_rows_close(table_to_host(tc), table_to_host(ta), "five plain operations vs step: table")
    assert_close_f32(sc.cpu().numpy(), sa.cpu().numpy(), "five plain operations vs step: state")
    for a, c in zip(oa[1:], oc[1:]):
        assert_close_f32(c["reduced"], a["reduced"], "five plain operations vs step: reduced gradients")
    assert torch.equal(ta.view(torch.int16 if dtype == "bf16" else torch.int32),
                       tb.view(torch.int16 if dtype == "bf16" else torch.int32))
    assert torch.equal(sa, sb)
    for a, b in zip(oa[1:], ob[1:]):
        assert a["reduced"].tobytes() == b["reduced"].tobytes()
        if "emb_next" in a:
            assert a["emb_next"].tobytes() == b["emb_next"].tobytes()
    t_ref, s_ref, want = run_steps_oracle(table, state, its, 0.01, 1e-8)
    compare_runs(oa, want, table_to_host(ta), sa.cpu().numpy(), t_ref, s_ref)


# ------------------------------------------------------------------------------------ host-visible errors of the step entry points
def test_step_entry_points_reject_bad_arguments(ctx):
    rng = np.random.default_rng(3)
    rows, dim = 1000, 64
    ids = zipf_ids(rng, 500, rows)
    table, state = table_to_dev(rand_table(rng, rows, dim, "f32")), torch.zeros(rows, device="cuda")
    grads = dev(rng.standard_normal((500, dim)).astype(np.float32))
    lay, sp = gpu_layout_and_classes(ctx, ids, ids, rows)
    with pytest.raises(fs.FreeScaleError) as e:
        fs.fs_reduce_update_class(ctx, 2, table, state, 0.01, 1e-8, grads, lay, sp)           # no such class
    assert e.value.code == fs.FS_EINVAL
    args = fs.make_step_args(table, state, 0.01, 1e-8, lay, grads, None, None, None, sp, None, None)
    args.cperm = None                                                                        # class order missing
    with pytest.raises(fs.FreeScaleError) as e:
        fs.fs_prioritized_step(ctx, args)
    assert e.value.code == fs.FS_EINVAL
    fresh = fs.Context(max_ids=1000, max_dim=64)
    out = fs.alloc_layout(500, "cuda")
    with pytest.raises(fs.FreeScaleError) as e:                                              # no pipelined call yet
        fs.fs_unique_ids_ahead(fresh, dev(ids), rows, out, stream=fs.FS_STREAM_LAST_STEP)
    assert e.value.code == fs.FS_EINVAL
    with pytest.raises(fs.FreeScaleError) as e:                                              # beyond the capacity
        big = dev(zipf_ids(rng, 2000, rows))
        fs.fs_unique_ids_ahead(fresh, big, rows, fs.alloc_layout(2000, "cuda"))
    assert e.value.code == fs.FS_ENOMEM
    assert fs.fs_check_async(fresh) == fs.FS_OK
    fresh.close()
    assert fs.fs_check_async(ctx) == fs.FS_OK


def test_many_ahead_dedups_outstanding(ctx):
    """More ahead-of-time dedups than the context tracks at once: the oldest finished ones are given up,
    every result is still correct."""
    rng = np.random.default_rng(4)
    rows = 5000
    batches = [zipf_ids(rng, 3000 + 100 * k, rows) for k in range(12)]
    outs = [fs.alloc_layout(len(b), "cuda") for b in batches]
    d_batches = [dev(b) for b in batches]                      # the IDs must stay in place until the dedups ran
    for d, o in zip(d_batches, outs):
        fs.fs_unique_ids_ahead(ctx, d, rows, o)
    assert fs.fs_check_async(ctx) == fs.FS_OK
    for b, o in zip(batches, outs):
        want = O.unique_ids(b, rows)
        u = int(o["n_unique"].item())
        assert np.array_equal(o["unique"][:u].cpu().numpy(), want["unique"])
        assert np.array_equal(o["perm"][:len(b)].cpu().numpy(), want["perm"])
        assert np.array_equal(o["inverse"][:len(b)].cpu().numpy(), want["inverse"])
