"""Soak of the hand-over between workgroups in the fused pass.

A row with tens of thousands of occurrences is cut into hundreds of position chunks; the pieces travel between
workgroups (on different XCDs, each with its own L2) as device-scope relaxed atomic stores, ordered against the
arrival counters by waiting for the stores' acknowledgement, and whoever arrives last adds them up.  Nothing but
repetition under contention can show a piece that is read before it has landed, so: the same two passes (both
classes, side by side on two streams, a lookup on a third stream keeping the memory system busy) 500 times from
a fresh table, every result compared bit for bit with the first.  The loop stops at the first mismatch.
"""
import numpy as np
import pytest
import torch

import paper_2604_24073_amd as fs
from helpers import dev, table_to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(300)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_last_arriver_handover_is_stable_under_contention(dtype):
    rng = np.random.default_rng(90107)
    rows, dim = 60_000, 128
    tail = ((np.minimum(rng.zipf(1.2, size=60_000), rows) - 1) * 2654435761 % rows).astype(np.int64)
    ids = np.concatenate([np.full(90_107, 11), np.full(5_000, 12), np.full(1_024, 13), np.full(65, 14),
                          np.full(64, 15), np.full(9, 16), tail]).astype(np.int64)
    ids = ids[rng.permutation(len(ids))]
    # the hottest row and some long rows collide with the next batch, others do not: long segments in both classes
    nxt = np.concatenate([np.array([11, 13, 15]), tail[::3]]).astype(np.int64)
    n = len(ids)
    ctx = fs.Context(max_ids=n, max_dim=dim)
    w = (rng.standard_normal((rows, dim)) * 0.05).astype(np.float32)
    table0 = dev(w) if dtype == "f32" else dev(w).to(torch.bfloat16)
    state0 = dev((rng.random(rows) * 0.1).astype(np.float32))
    grads = dev(rng.standard_normal((n, dim)).astype(np.float32))
    lay = fs.fs_unique_ids(ctx, dev(ids), rows)
    lay1 = fs.fs_unique_ids(ctx, dev(nxt), rows)
    sp = fs.fs_collision_split_classes(ctx, lay, lay1["unique"], lay1["n_unique"], len(nxt))
    assert fs.fs_check_async(ctx) == fs.FS_OK
    pos = sp["class_pos"].cpu().numpy()
    assert pos[0] > 90_000 and pos[1] - pos[0] > 5_000          # long segments in both classes
    # the lookup beside the passes works on a table of its own (a lookup of rows that are being updated would be a race)
    other = torch.randn((200_000, dim), device="cuda").to(table0.dtype)
    other_ids = torch.randint(0, 200_000, (300_000,), dtype=torch.int64, device="cuda")
    other_out = torch.empty((300_000, dim), dtype=table0.dtype, device="cuda")
    s0, s1, s2 = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    table, state = torch.empty_like(table0), torch.empty_like(state0)
    first = None
    view = torch.int16 if dtype == "bf16" else torch.int32
    for it in range(500):
        table.copy_(table0)
        state.copy_(state0)
        torch.cuda.synchronize()
        fs.fs_gather_jagged(ctx, other, other_ids, None, out=other_out, stream=s2)
        fs.fs_reduce_update_class(ctx, 0, table, state, 0.02, 1e-8, grads, lay, sp, stream=s0)
        fs.fs_reduce_update_class(ctx, 1, table, state, 0.02, 1e-8, grads, lay, sp, stream=s1)
        fs.fs_gather_jagged(ctx, other, other_ids, None, out=other_out, stream=s2)
        torch.cuda.synchronize()
        if first is None:
            first = (table.clone(), state.clone())
            assert not torch.equal(first[0].view(view), table0.view(view))
            continue
        same = torch.equal(table.view(view), first[0].view(view)) and torch.equal(state.view(torch.int32),
                                                                                  first[1].view(torch.int32))
        assert same, f"iteration {it}: the passes left other bits than the first time"
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    ctx.close()
