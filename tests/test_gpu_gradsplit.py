"""split() of Algorithm 2's Backward on the GPU (fs_split_grads) against the oracle, bit for bit, and the fused
passes reading the packed parts against the same passes reading the batch-major gradients."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_24073_amd as fs
from helpers import dev, table_to_dev, table_to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = fs.Context(max_ids=200_000, max_dim=256)
    yield c
    c.close()


def zipf_ids(rng, n, num_rows, a=1.2):
    ranks = np.minimum(rng.zipf(a, size=n), num_rows) - 1
    return ((ranks * 2654435761) % num_rows).astype(np.int64)


def layout_and_split(ctx, ids_t, ids_t1, rows):
    lay = fs.fs_unique_ids(ctx, dev(ids_t), rows)
    if ids_t1 is None or len(ids_t1) == 0:
        sp = fs.fs_collision_split_classes(ctx, lay, None, None, 0)
    else:
        lay1 = fs.fs_unique_ids(ctx, dev(ids_t1), rows)
        sp = fs.fs_collision_split_classes(ctx, lay, lay1["unique"], lay1["n_unique"], len(ids_t1))
    return lay, sp


@pytest.mark.parametrize("n,n1,rows,dim", [(1, 1, 2, 4), (1000, 800, 300, 64), (1023, 5000, 4000, 128), (1024, 10, 50, 20),
                                            (1025, 1025, 1025, 256), (70001, 60000, 20000, 128), (5000, 0, 700, 64)])
def test_split_grads_bit_exact(ctx, n, n1, rows, dim):
    rng = np.random.default_rng(n + dim)
    ids_t = zipf_ids(rng, n, rows, a=1.1)
    ids_t1 = zipf_ids(rng, n1, rows, a=1.1) if n1 else np.empty(0, np.int64)
    grads = rng.standard_normal((n, dim)).astype(np.float32)
    want = O.split_grads(grads, ids_t, np.unique(ids_t1))
    lay, sp = layout_and_split(ctx, ids_t, ids_t1, rows)
    got = fs.fs_split_grads(ctx, dev(grads), lay, sp)
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    n_co, n_ex = (int(x) for x in got["counts"].cpu().numpy())
    assert (n_co, n_ex) == (len(want["co_index"]), len(want["ex_index"]))
    assert np.array_equal(got["co_index"][:n_co].cpu().numpy(), want["co_index"])
    assert np.array_equal(got["ex_index"][:n_ex].cpu().numpy(), want["ex_index"])
    assert got["g_co"][:n_co].cpu().numpy().tobytes() == want["g_co"].tobytes()
    assert got["g_ex"][:n_ex].cpu().numpy().tobytes() == want["g_ex"].tobytes()
    pos = got["part_pos"][:n].cpu().numpy()
    assert np.array_equal(pos[want["co_index"]], np.arange(n_co))
    assert np.array_equal(pos[want["ex_index"]], -1 - np.arange(n_ex))


def test_split_grads_all_and_none(ctx):
    rng = np.random.default_rng(3)
    ids = zipf_ids(rng, 3000, 400)
    grads = rng.standard_normal((3000, 64)).astype(np.float32)
    for nxt in (ids.copy(), (ids + 100_000)):
        want = O.split_grads(grads, ids, np.unique(nxt))
        lay, sp = layout_and_split(ctx, ids, nxt, 200_000)
        got = fs.fs_split_grads(ctx, dev(grads), lay, sp)
        assert fs.fs_check_async(ctx) == fs.FS_OK
        assert got["counts"].cpu().numpy().tolist() == [len(want["co_index"]), len(want["ex_index"])]
        assert got["g_co"][:len(want["co_index"])].cpu().numpy().tobytes() == want["g_co"].tobytes()
        assert got["g_ex"][:len(want["ex_index"])].cpu().numpy().tobytes() == want["g_ex"].tobytes()
    empty = fs.fs_split_grads(ctx, torch.empty((0, 64), device="cuda"),
                              {"inverse": None}, {"co_slot": None, "counts": torch.zeros(3, dtype=torch.int64, device="cuda")})
    assert fs.fs_check_async(ctx) == fs.FS_OK and empty["counts"].cpu().numpy().tolist() == [0, 0]


@pytest.mark.parametrize("dim,dtype", [(128, "f32"), (64, "f32"), (128, "bf16")])
def test_fused_passes_read_the_packed_parts(ctx, dim, dtype):
    """Priority pass on g_co, deferred pass on g_ex (class order rewritten by fs_class_order_for_parts): table and
    state bit for bit what the passes on the batch-major gradients leave, long and cut segments included."""
    rng = np.random.default_rng(dim)
    rows = 3000
    ids = np.concatenate([np.full(6000, 7), np.full(700, 8), zipf_ids(rng, 20000, rows, a=1.1)]).astype(np.int64)
    ids = ids[rng.permutation(len(ids))]
    nxt = np.concatenate([np.array([7]), zipf_ids(rng, 9000, rows, a=1.1)]).astype(np.int64)
    n = len(ids)
    w = (rng.standard_normal((rows, dim)) * 0.05).astype(np.float32)
    table = w if dtype == "f32" else torch.from_numpy(w).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    state = (rng.random(rows) * 0.1).astype(np.float32)
    grads = dev(rng.standard_normal((n, dim)).astype(np.float32))
    lay, sp = layout_and_split(ctx, ids, nxt, rows)
    t_a, s_a = table_to_dev(table), dev(state)
    for cls in (0, 1):
        fs.fs_reduce_update_class(ctx, cls, t_a, s_a, 0.02, 1e-8, grads, lay, sp)
    parts = fs.fs_split_grads(ctx, grads, lay, sp)
    sp_parts = fs.fs_class_order_for_parts(ctx, parts, n, sp)
    t_b, s_b = table_to_dev(table), dev(state)
    fs.fs_reduce_update_class(ctx, 0, t_b, s_b, 0.02, 1e-8, parts["g_co"], lay, sp_parts)
    fs.fs_reduce_update_class(ctx, 1, t_b, s_b, 0.02, 1e-8, parts["g_ex"], lay, sp_parts)
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    n_co, n_ex = (int(x) for x in parts["counts"].cpu().numpy())
    assert n_co > 6000 and n_ex > 0
    assert table_to_host(t_b).tobytes() == table_to_host(t_a).tobytes()
    assert s_b.cpu().numpy().tobytes() == s_a.cpu().numpy().tobytes()
    assert table_to_host(t_a).tobytes() != table.tobytes()
