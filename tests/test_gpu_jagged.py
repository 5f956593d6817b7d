"""The load balancer's data path on one GPU against the oracle: FBS partitioner (Section 4.1 of the paper)
and indexed permute of a jagged tensor (Section 4.2).  Index work: bit-exact."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_24073_amd as fs
from helpers import dev

pytestmark = pytest.mark.gpu


def powerlaw_lengths(rng, B, lo=16, hi=4096, alpha=1.5):
    u = rng.random(B)
    x = lo * (1.0 - u) ** (-1.0 / alpha)
    return np.clip(x, lo, hi).astype(np.int64)


@pytest.mark.parametrize("B,n,hi", [(0, 4, 64), (1, 1, 64), (3, 8, 64), (37, 5, 64), (1024, 8, 4096), (5000, 64, 4096),
                                    (20000, 512, 16384), (4097, 3, 100000), (2048, 2048, 64), (2049, 2048, 64)])
def test_fbs_partition_matches_oracle(B, n, hi):
    rng = np.random.default_rng(B * 7 + n)
    lengths = powerlaw_lengths(rng, B, 1, hi) if B else np.empty(0, np.int64)
    if B > 10:
        lengths[rng.integers(0, B, size=B // 10)] = 0             # empty samples, and many ties
    ctx = fs.Context(max_ids=max(B, 16), max_dim=8)
    sample_of, rank_offsets = fs.fs_partition_fbs(ctx, dev(lengths), hi, n)
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    want_s, want_r = O.partition_fbs(lengths, n)
    assert rank_offsets.cpu().numpy().tolist() == want_r.tolist()
    assert sample_of.cpu().numpy().tolist() == want_s.tolist()
    ctx.close()


def test_fbs_partition_reports_a_length_out_of_range():
    ctx = fs.Context(max_ids=64, max_dim=8)
    fs.fs_partition_fbs(ctx, dev(np.array([3, 9, 70, 1], dtype=np.int64)), 64, 2)
    assert fs.fs_check_async(ctx) == fs.FS_ERANGE
    with pytest.raises(fs.FreeScaleError) as e:
        fs.fs_partition_fbs(ctx, dev(np.zeros(65, dtype=np.int64)), 64, 2)
    assert e.value.code == fs.FS_ENOMEM
    with pytest.raises(fs.FreeScaleError) as e:
        fs.fs_partition_fbs(ctx, dev(np.zeros(4, dtype=np.int64)), 64, 0)
    assert e.value.code == fs.FS_EINVAL
    ctx.close()


def jagged(rng, lens, dtype, width):
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    n = int(offsets[-1])
    shape = (n,) if width == 0 else (n, width)
    if np.issubdtype(dtype, np.integer):
        values = rng.integers(0, 2**31 - 1, size=shape).astype(dtype)
    else:
        values = rng.standard_normal(shape).astype(dtype)
    return values, offsets


@pytest.mark.parametrize("dtype,width", [(np.int64, 0), (np.int32, 0), (np.float32, 32), (np.float32, 3), (np.int64, 2)])
def test_indexed_permute_matches_oracle(dtype, width):
    rng = np.random.default_rng(11 + width)
    B = 3000
    lens = powerlaw_lengths(rng, B, 1, 2000)
    lens[rng.integers(0, B, size=300)] = 0
    lens[17] = 16384                                              # one sample over several copy tiles
    values, offsets = jagged(rng, lens, dtype, width)
    ctx = fs.Context(max_ids=8192, max_dim=8)
    d_values, d_offsets = dev(values), dev(offsets)
    fbs, ro = O.partition_fbs(lens, 7)
    selections = [fbs,                                             # the partitioner's permutation
                  fbs[ro[3]:ro[4]],                                # one rank's share
                  np.array([17, 17, 5, 2999, 0, 17], dtype=np.int32),
                  np.empty(0, dtype=np.int32),
                  np.flatnonzero(lens == 0).astype(np.int32)]      # nothing but empty samples
    for sel in selections:
        want, want_off = O.jagged_indexed_permute(values, offsets, sel)
        cap = want.shape[0]
        out, out_off = fs.fs_jagged_indexed_permute(ctx, d_values, d_offsets, dev(sel) if sel.size else
                                                    torch.empty(0, dtype=torch.int32, device="cuda"), cap)
        assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
        assert out_off.cpu().numpy().tolist() == want_off.tolist()
        assert out.cpu().numpy().tobytes() == want.tobytes()
    ctx.close()


def test_indexed_permute_with_runs_of_empty_samples_longer_than_the_staged_window():
    # 6000 empty samples between two non-empty ones: a copy tile then touches more sample boundaries than it
    # stages in LDS and searches global memory instead
    rng = np.random.default_rng(3)
    lens = np.zeros(6100, dtype=np.int64)
    lens[:50] = rng.integers(1, 40, size=50)
    lens[-50:] = rng.integers(1, 40, size=50)
    values, offsets = jagged(rng, lens, np.int64, 0)
    ctx = fs.Context(max_ids=8192, max_dim=8)
    sel = np.arange(6100, dtype=np.int32)
    want, want_off = O.jagged_indexed_permute(values, offsets, sel)
    out, out_off = fs.fs_jagged_indexed_permute(ctx, dev(values), dev(offsets), dev(sel), want.shape[0])
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    assert out_off.cpu().numpy().tolist() == want_off.tolist()
    assert out.cpu().numpy().tolist() == want.tolist()
    ctx.close()


def test_indexed_permute_reports_bad_selections_and_short_outputs():
    rng = np.random.default_rng(5)
    lens = rng.integers(1, 30, size=100)
    values, offsets = jagged(rng, lens, np.int64, 0)
    ctx = fs.Context(max_ids=1024, max_dim=8)
    d_values, d_offsets = dev(values), dev(offsets)
    sel = np.arange(100, dtype=np.int32)
    # a sample index out of range: reported, treated as empty, everything else in place
    bad = sel.copy(); bad[40] = 100
    out, out_off = fs.fs_jagged_indexed_permute(ctx, d_values, d_offsets, dev(bad), values.shape[0])
    assert fs.fs_check_async(ctx) == fs.FS_ERANGE
    good = np.delete(sel, 40)
    want, _ = O.jagged_indexed_permute(values, offsets, good)
    assert out[:want.shape[0]].cpu().numpy().tolist() == want.tolist()
    # fewer output elements than needed: reported, the copy stops at the capacity, offsets are complete
    want, want_off = O.jagged_indexed_permute(values, offsets, sel)
    out, out_off = fs.fs_jagged_indexed_permute(ctx, d_values, d_offsets, dev(sel), 500)
    assert fs.fs_check_async(ctx) == fs.FS_ERANGE
    assert out_off.cpu().numpy().tolist() == want_off.tolist()
    assert out.cpu().numpy().tolist() == want[:500].tolist()
    # offsets that point outside the values
    broken = offsets.copy(); broken[-1] += 5
    fs.fs_jagged_indexed_permute(ctx, d_values, dev(broken), dev(sel), values.shape[0] + 5)
    assert fs.fs_check_async(ctx) == fs.FS_ERANGE
    with pytest.raises(fs.FreeScaleError) as e:
        fs.fs_jagged_indexed_permute(ctx, dev(np.zeros((4, 3), dtype=np.int16)), dev(np.array([0, 4], dtype=np.int64)),
                                     dev(np.array([0], dtype=np.int32)), 4)
    assert e.value.code == fs.FS_EINVAL
    ctx.close()
