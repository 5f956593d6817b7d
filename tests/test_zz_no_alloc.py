"""fs_collision_split_static (the entry point that allocates nothing) against fs_collision_split.

Two calls in a row on the same GPU, the second with smaller inputs: the fixed scratch array keeps the first
call's flags and tile counts, and none of them may leak into the second result.  Every output is compared bit
for bit with what the context form gives for the same inputs (which the parity tests compare with the oracle).
"""
import numpy as np
import pytest
import torch

import paper_2604_24073_amd as fs

pytestmark = pytest.mark.gpu


def _lists(rng, n_t, n_t1, rows):
    u_t = np.unique(rng.integers(0, rows, size=n_t, dtype=np.int64))
    u_t1 = np.unique(rng.integers(0, rows, size=n_t1, dtype=np.int64))
    return u_t, u_t1


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _run_both(ctx, u_t, u_t1, pad_t, pad_t1):
    nt, nt1 = len(u_t), len(u_t1)
    cap_t, cap_t1 = (nt + pad_t if nt else 0), (nt1 + pad_t1 if nt1 else 0)
    pad = lambda a, k: _dev(np.concatenate([a, np.full(k, -7, dtype=np.int64)]))
    d_ut = pad(u_t, pad_t) if nt else None
    d_ut1 = pad(u_t1, pad_t1) if nt1 else None
    d_nt = _dev(np.array([nt], dtype=np.int64)) if nt else None
    d_nt1 = _dev(np.array([nt1], dtype=np.int64)) if nt1 else None
    want = fs.fs_collision_split(ctx, d_ut, d_nt, d_ut1, d_nt1, cap_t, cap_t1)
    torch.cuda.synchronize()
    # caller-owned outputs, poisoned so that an entry the call fails to write shows
    i64 = lambda k: torch.full((max(k, 1),), -99, dtype=torch.int64, device="cuda")
    i32 = lambda k: torch.full((max(k, 1),), -99, dtype=torch.int32, device="cuda")
    out = {"co": i64(cap_t), "co_slot": i32(cap_t), "ex": i64(cap_t), "ex_slot": i32(cap_t),
           "ex_next": i64(cap_t1), "ex_next_slot": i32(cap_t1), "counts": i64(3)}
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    fs.fs_collision_split_static(d_ut, d_nt, d_ut1, d_nt1, cap_t, cap_t1, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before                       # nothing taken from torch's allocator
    wc, gc = want["counts"].cpu().numpy(), out["counts"].cpu().numpy()
    assert gc.tolist() == wc.tolist()
    for name, cnt in (("co", wc[0]), ("ex", wc[1]), ("ex_next", wc[2])):
        assert torch.equal(out[name][:cnt], want[name][:cnt]), name
        assert torch.equal(out[name + "_slot"][:cnt], want[name + "_slot"][:cnt]), name
    return wc.tolist()


def test_static_split_equals_context_split_twice_in_a_row():
    ctx = fs.Context(max_ids=400_000, max_dim=64)
    rng = np.random.default_rng(77)
    # first call: several tiles per side, ragged tails, capacities beyond the counts
    u_t, u_t1 = _lists(rng, 300_000, 250_000, 900_000)
    c1 = _run_both(ctx, u_t, u_t1, 37, 1500)
    assert c1[0] > 0 and c1[1] > 0 and c1[2] > 0
    # second call, smaller: fewer tiles than the first left counts for, shorter lists than it left flags for
    u_t, u_t1 = _lists(rng, 3_000, 1_100, 5_000)
    c2 = _run_both(ctx, u_t, u_t1, 5, 0)
    assert 0 < c2[0] < c1[0]
    # degenerate inputs through the same array
    a = np.array([1, 5, 9, 12], dtype=np.int64)
    assert _run_both(ctx, a, a, 0, 0) == [4, 0, 0]
    assert _run_both(ctx, a, np.empty(0, dtype=np.int64), 0, 0) == [0, 4, 0]
    assert _run_both(ctx, np.empty(0, dtype=np.int64), a, 0, 0) == [0, 0, 4]
    assert _run_both(ctx, np.empty(0, dtype=np.int64), np.empty(0, dtype=np.int64), 0, 0) == [0, 0, 0]
    ctx.close()


def test_static_split_rejects_more_rows_than_its_array_holds():
    out = {k: None for k in ("co", "co_slot", "ex", "ex_slot", "ex_next", "ex_next_slot", "counts")}
    with pytest.raises(fs.FreeScaleError) as e:
        fs.fs_collision_split_static(None, None, None, None, fs.FS_STATIC_SPLIT_MAX_ROWS + 1, 0, out)
    assert e.value.code == fs.FS_ENOMEM and "FS_STATIC_SPLIT_MAX_ROWS" in str(e.value)
