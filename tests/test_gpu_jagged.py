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


def keyed(rng, F, B, dtype, width, hi=40):
    lens = rng.integers(0, hi, size=F * B)
    if F * B > 20:
        lens[rng.integers(0, F * B, size=F * B // 8)] = 0
    return jagged(rng, lens, dtype, width)


@pytest.mark.parametrize("F,B,dtype,width", [(8, 512, np.int64, 0), (1, 3000, np.int64, 0), (26, 1, np.int32, 0),
                                             (3, 700, np.float32, 16), (5, 0, np.int64, 0), (2, 4096, np.float32, 3)])
def test_keyed_transpose_matches_oracle(F, B, dtype, width):
    rng = np.random.default_rng(F * 1000 + B)
    values, offsets = keyed(rng, F, B, dtype, width)
    ctx = fs.Context(max_ids=max(F * B, 16), max_dim=8)
    out, out_off = fs.fs_jagged_keyed_transpose(ctx, dev(values), dev(offsets), F, B)
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    want, want_off = O.jagged_keyed_transpose(values, offsets, F, B)
    assert out_off.cpu().numpy().tolist() == want_off.tolist()
    assert out.cpu().numpy().tobytes() == want.tobytes()
    ctx.close()


@pytest.mark.parametrize("F,B,n_ranks,dtype,width", [(4, 1024, 8, np.int64, 0), (1, 2048, 512, np.int64, 0),
                                                     (6, 333, 32, np.float32, 8), (2, 5, 8, np.int64, 0),
                                                     (3, 1000, 1, np.int32, 0)])
def test_ranged_dispatch_and_combine_match_oracle(F, B, n_ranks, dtype, width):
    rng = np.random.default_rng(F * 77 + B + n_ranks)
    values, offsets = keyed(rng, F, B, dtype, width)
    # ranges as the FBS partitioner leaves them (some ranks may be empty when there are more ranks than samples)
    _, ro = O.partition_fbs(rng.integers(1, 100, size=B).astype(np.int64), n_ranks)
    ctx = fs.Context(max_ids=max(F * B, 16), max_dim=8)
    d_ro = dev(ro)
    out, out_off, splits = fs.fs_jagged_ranged_dispatch(ctx, dev(values), dev(offsets), F, B, d_ro)
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    want, want_off, want_splits = O.jagged_ranged_dispatch(values, offsets, F, B, ro)
    assert out_off.cpu().numpy().tolist() == want_off.tolist()
    assert splits.cpu().numpy().tolist() == want_splits.tolist()
    assert out.cpu().numpy().tobytes() == want.tobytes()
    back, back_off = fs.fs_jagged_ranged_combine(ctx, out, out_off, F, B, d_ro)
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    want_b, want_b_off = O.jagged_ranged_combine(want, want_off, F, B, ro)
    assert back_off.cpu().numpy().tolist() == want_b_off.tolist() == offsets.tolist()
    assert back.cpu().numpy().tobytes() == want_b.tobytes() == values.tobytes()
    ctx.close()


def test_ranged_dispatch_reports_ranges_that_do_not_cover_the_samples():
    rng = np.random.default_rng(8)
    values, offsets = keyed(rng, 2, 50, np.int64, 0)
    ctx = fs.Context(max_ids=256, max_dim=8)
    for ro in ([0, 20, 60], [0, 30, 20, 50], [5, 20, 50]):
        fs.fs_jagged_ranged_dispatch(ctx, dev(values), dev(offsets), 2, 50, dev(np.array(ro, dtype=np.int64)))
        assert fs.fs_check_async(ctx) == fs.FS_ERANGE, ro
        fs.fs_jagged_ranged_combine(ctx, dev(values), dev(offsets), 2, 50, dev(np.array(ro, dtype=np.int64)))
        assert fs.fs_check_async(ctx) == fs.FS_ERANGE, ro
    with pytest.raises(fs.FreeScaleError) as e:
        fs.fs_jagged_keyed_transpose(ctx, dev(values), dev(offsets), 2, 200)
    assert e.value.code == fs.FS_ENOMEM
    ctx.close()


@pytest.mark.timeout(300)
def test_balancer_path_at_the_size_the_bench_times():
    """64 ranks x 1024 samples of configuration 1's length rule (16.7 M IDs): partition, permute, dispatch,
    combine and transpose against the oracle, every byte."""
    from fs_workloads.generators import powerlaw_lengths as cfg_lengths
    rng = np.random.default_rng(20240)
    ranks, keys, Bg = 64, 4, 65536
    lens = cfg_lengths(rng, Bg, 1.5, 16, 4096)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    ng = int(offsets[-1])
    values = rng.integers(0, 4_000_000, size=ng).astype(np.int64)
    ctx = fs.Context(max_ids=Bg, max_dim=8)
    d_values, d_offsets = dev(values), dev(offsets)
    sample_of, rank_off = fs.fs_partition_fbs(ctx, dev(lens), 4096, ranks)
    want_s, want_r = O.partition_fbs(lens, ranks)
    assert sample_of.cpu().numpy().tolist() == want_s.tolist() and rank_off.cpu().numpy().tolist() == want_r.tolist()
    out, out_off = fs.fs_jagged_indexed_permute(ctx, d_values, d_offsets, sample_of, ng)
    want, want_off = O.jagged_indexed_permute(values, offsets, want_s)
    assert torch.equal(out_off.cpu(), torch.from_numpy(want_off)) and torch.equal(out.cpu(), torch.from_numpy(want))
    Bk = Bg // keys
    _, ro = O.partition_fbs(lens[:Bk], ranks)
    d_ro = dev(ro)
    disp, disp_off, splits = fs.fs_jagged_ranged_dispatch(ctx, d_values, d_offsets, keys, Bk, d_ro)
    w_disp, w_off, w_splits = O.jagged_ranged_dispatch(values, offsets, keys, Bk, ro)
    assert torch.equal(disp.cpu(), torch.from_numpy(w_disp)) and torch.equal(disp_off.cpu(), torch.from_numpy(w_off))
    assert splits.cpu().numpy().tolist() == w_splits.tolist()
    back, back_off = fs.fs_jagged_ranged_combine(ctx, disp, disp_off, keys, Bk, d_ro)
    assert torch.equal(back, d_values) and torch.equal(back_off, d_offsets)
    tr, tr_off = fs.fs_jagged_keyed_transpose(ctx, d_values, d_offsets, keys, Bk)
    w_tr, w_tr_off = O.jagged_keyed_transpose(values, offsets, keys, Bk)
    assert torch.equal(tr.cpu(), torch.from_numpy(w_tr)) and torch.equal(tr_off.cpu(), torch.from_numpy(w_tr_off))
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    ctx.close()


@pytest.mark.parametrize("B,n,hi,alpha", [(0, 4, 64, 1.0), (1, 3, 64, 1.0), (5, 8, 64, 2.0), (1024, 8, 4096, 1.5),
                                          (5000, 64, 4096, 1.0), (20000, 512, 16384, 1.7), (4097, 3, 300, 0.0),
                                          (65536, 64, 4096, 2.0)])
def test_vbs_partition_matches_oracle(B, n, hi, alpha):
    rng = np.random.default_rng(B * 3 + n)
    lengths = powerlaw_lengths(rng, B, 1, hi) if B else np.empty(0, np.int64)
    if B > 10:
        lengths[rng.integers(0, B, size=B // 10)] = 0
    weights = np.round(np.arange(hi + 1, dtype=np.float64) ** alpha * 1024).astype(np.int64)
    ctx = fs.Context(max_ids=max(B, 16), max_dim=8)
    sample_of, rank_offsets = fs.fs_partition_vbs(ctx, dev(lengths), dev(weights), n)
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    want_s, want_r = O.partition_vbs(lengths, weights, n)
    assert rank_offsets.cpu().numpy().tolist() == want_r.tolist()
    assert sample_of.cpu().numpy().tolist() == want_s.tolist()
    ctx.close()


def test_vbs_partition_reports_bad_weights():
    ctx = fs.Context(max_ids=64, max_dim=8)
    lengths = dev(np.array([3, 9, 7, 1], dtype=np.int64))
    w = np.arange(11, dtype=np.int64)
    w[7] = -1
    fs.fs_partition_vbs(ctx, lengths, dev(w), 2)                    # a negative weight
    assert fs.fs_check_async(ctx) == fs.FS_ERANGE
    big = np.full(11, 2**60, dtype=np.int64)
    _, ro = fs.fs_partition_vbs(ctx, lengths, dev(big), 4)          # n_ranks * total weight beyond 2^63
    assert fs.fs_check_async(ctx) == fs.FS_ERANGE
    assert ro.cpu().numpy().tolist() == [0, 4, 4, 4, 4]
    fs.fs_partition_vbs(ctx, dev(np.array([3, 11], dtype=np.int64)), dev(np.arange(11, dtype=np.int64)), 2)
    assert fs.fs_check_async(ctx) == fs.FS_ERANGE                   # a length beyond the table
    ctx.close()
