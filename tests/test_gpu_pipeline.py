"""The software-pipelined form of the step (index half of the next iteration beside the gradient
half of the current one, dedups optionally batches ahead) must give exactly the bits of its
building blocks issued one after another."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_24073_amd as fs
from helpers import assert_bf16_within_1ulp, assert_close_f32, assert_rows_close, dev, table_to_dev, table_to_host
from test_gpu_parity import compare_runs, rand_table, run_steps_gpu, run_steps_oracle, zipf_ids

pytestmark = pytest.mark.gpu


class It:
    pass


def make_its(rng, rows, dim, n_iter, users=40, max_len=300):
    its = []
    for _ in range(n_iter):
        it = It()
        lens = rng.integers(0, max_len, size=users)
        it.offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        it.values = zipf_ids(rng, int(it.offsets[-1]), rows, a=1.1)
        it.grads = rng.standard_normal((len(it.values), dim)).astype(np.float32)
        its.append(it)
    return its


def run_pipelined(ctx, table, state, its, lr, eps, ahead=False, sync_each=True, two_part=False, disturb=None,
                  inverse=True, between=None):
    """ahead: True / "last_step": dedup every batch with fs_unique_ids_ahead, three batches before the
    iteration that gathers it (five layout buffers in rotation; "last_step": ordered after the start
    of the previous pipelined call instead of the stream's current position, six layout buffers).
    "index" / "index_last_step": the whole index half of every iteration with fs_step_forward_ahead,
    two iterations ahead (six layouts, five split bundles).
    "batchK" / "batchK_last_step": the index halves of K consecutive iterations in shared launches
    (fs_step_forward_ahead_batch), issued D = K + 1 iterations before the first of them is stepped
    (K + D + 3 layouts, K + D + 2 split bundles).
    sync_each=False: no wait between the calls.
    two_part: fs_prioritized_step_two_part_multi (exclusive rows of the lookahead batch fetched by the call
    before, three output batches in rotation); disturb: iteration before whose call the pipeline is joined,
    the library told to forget what it fetched and the fetched part of the output batch overwritten (the call
    must then redo the whole lookup).
    inverse=False: layouts without the inverse map (optional for everything but the two-part lookup).
    between: called after every step call (other work on the same context between the steps)."""
    batch = int(ahead[5]) if isinstance(ahead, str) and ahead.startswith("batch") else 0
    index_ahead = ahead in ("index", "index_last_step")
    last_step = isinstance(ahead, str) and ahead.endswith("last_step")
    D = batch + 1
    if batch:
        L, P = batch + D + 3, batch + D + 2
    else:
        L = (6 if (last_step or index_ahead) else 5) if ahead else 3
        P = 5 if index_ahead else 3
    d_table, d_state = table_to_dev(table), dev(state)
    num_rows, dim = table.shape
    T = len(its)
    d_vals = [dev(it.values) for it in its]
    d_offs = [dev(it.offsets) for it in its]
    d_grads = [dev(it.grads) for it in its]
    n = [v.numel() for v in d_vals]
    nmax = max(n)
    layouts = [fs.alloc_layout(nmax, "cuda", inverse=inverse) for _ in range(L)]
    splits = [fs.alloc_split(nmax, nmax, "cuda") for _ in range(P)]
    reduced = [torch.empty((nmax, dim), dtype=torch.float32, device="cuda") for _ in range(2)]
    E = 3 if two_part else 2
    embs = [torch.empty((nmax, dim), dtype=d_table.dtype, device="cuda") for _ in range(E)]

    def args_for(t):
        lay_t = dict(layouts[t % L]); lay_t["n"] = n[t]
        last = t == T - 1
        return fs.make_step_args(d_table, d_state, lr, eps, lay_t, d_grads[t], None if last else d_vals[t + 1],
                                 None if last else d_offs[t + 1], None if last else layouts[(t + 1) % L],
                                 splits[t % P], reduced[t % 2], None if last else embs[t % E])

    stepped = [False]

    def order():
        return fs.FS_STREAM_LAST_STEP if (last_step and stepped[0]) else None

    def dedup_ahead(t):
        if ahead and not index_ahead and not batch and t < T:
            fs.fs_unique_ids_ahead(ctx, d_vals[t], num_rows, layouts[t % L], stream=order())

    def index_half_ahead(t):
        if index_ahead and t < T:
            fs.fs_step_forward_ahead(ctx, all_args[t], stream=order())

    def index_batch_ahead(first):
        if batch and first % batch == 0 and 0 <= first < T:
            fs.fs_step_forward_ahead_batch(ctx, all_args[first:min(first + batch, T)], stream=order())

    fs.fs_unique_ids(ctx, d_vals[0], num_rows, out=layouts[0])
    all_args = [args_for(t) for t in range(T)]
    dedup_ahead(1)
    if index_ahead:
        index_half_ahead(0)                                       # dedup of batch 1, split and class order of 0
        index_half_ahead(1)
    elif batch:
        for first in range(0, D):
            index_batch_ahead(first)
    else:
        fs.fs_step_forward(ctx, all_args[0])                      # primes the pipeline: layout 1, split 0
    dedup_ahead(2)
    outs = []
    for t in range(T):
        nxt = all_args[t + 1] if t + 1 < T else None
        dedup_ahead(t + 3)
        index_half_ahead(t + 2)
        index_batch_ahead(t + D)
        if two_part:
            if disturb == t:
                fs.fs_step_join(ctx)
                fs.fs_two_part_forget(ctx)
                torch.cuda.synchronize()
                embs[t % E].view(torch.int16 if d_table.dtype == torch.bfloat16 else torch.int32).fill_(-1)
            fs.fs_prioritized_step_two_part_multi(ctx, fs.step_args_array([all_args[t]]),
                                                  fs.step_args_array([nxt]) if nxt is not None else None)
        else:
            fs.fs_prioritized_step_pipelined(ctx, all_args[t], nxt)
        stepped[0] = True
        if between is not None:
            between(t)
        if not sync_each:
            continue
        assert fs.fs_check_async(ctx) == fs.FS_OK
        u = int(layouts[t % L]["n_unique"].item())
        rec = {"reduced": reduced[t % 2][:u].cpu().numpy(), "counts": splits[t % P]["counts"].cpu().numpy()}
        if t + 1 < T:
            rec["emb_next"] = table_to_host(embs[t % E][:n[t + 1]])
        outs.append(rec)
    assert fs.fs_check_async(ctx) == fs.FS_OK
    return d_table, d_state, outs


@pytest.mark.parametrize("dtype,dim", [("f32", 128), ("bf16", 128), ("f32", 64)])
def test_pipelined_steps_match_sequential_calls_bitwise(dtype, dim):
    ctx = fs.Context(max_ids=20000, max_dim=256)
    rng = np.random.default_rng(2024)
    rows = 30000
    table = rand_table(rng, rows, dim, dtype)
    state = np.zeros(rows, np.float32)
    its = make_its(rng, rows, dim, 7)
    tp, sp_, op = run_pipelined(ctx, table, state, its, 0.01, 1e-8)
    ts, ss, os_ = run_steps_gpu(ctx, table, state, its, 0.01, 1e-8, mode="fused_calls")
    view = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(tp.view(view), ts.view(view))
    assert torch.equal(sp_, ss)
    for a, b in zip(op, os_[1:]):
        assert a["reduced"].tobytes() == b["reduced"].tobytes()
        assert a["counts"].tolist() == b["counts"].tolist()
        if "emb_next" in a:
            assert a["emb_next"].tobytes() == b["emb_next"].tobytes()
    t_ref, s_ref, want = run_steps_oracle(table, state, its, 0.01, 1e-8)
    compare_runs(os_, want, table_to_host(ts), ss.cpu().numpy(), t_ref, s_ref)
    # dedups batches ahead on the index streams, with and without waits between the calls, with and
    # without the enqueueing threads: always the same bits
    for ahead, sync_each, threaded in ((True, True, True), (True, False, True), (False, False, True),
                                       (True, False, False), (False, True, False), ("last_step", False, True),
                                       ("last_step", True, False), ("index", False, True), ("index", True, True),
                                       ("index_last_step", False, True), ("index_last_step", False, False),
                                       ("index", True, False), ("batch2", False, True), ("batch2_last_step", False, True),
                                       ("batch3_last_step", False, True), ("batch4_last_step", False, False),
                                       ("batch2", True, True), ("batch4", True, False)):
        ctx.lib.fs_ctx_set_threaded_enqueue(ctx.handle, 1 if threaded else 0)
        ta, sa, oa = run_pipelined(ctx, table, state, its, 0.01, 1e-8, ahead=ahead, sync_each=sync_each)
        what = f"ahead={ahead} sync_each={sync_each} threaded={threaded}"
        assert torch.equal(ta.view(view), ts.view(view)), what
        assert torch.equal(sa, ss), what
        for a, b in zip(oa, os_[1:]):
            assert a["reduced"].tobytes() == b["reduced"].tobytes(), what
            if "emb_next" in a:
                assert a["emb_next"].tobytes() == b["emb_next"].tobytes(), what
    # the inverse map is optional for the step calls: without it, the same bits
    for ahead in (False, "batch2_last_step", "index"):
        ta, sa, oa = run_pipelined(ctx, table, state, its, 0.01, 1e-8, ahead=ahead, inverse=False)
        assert torch.equal(ta.view(view), ts.view(view)) and torch.equal(sa, ss), f"no inverse map, ahead={ahead}"
        for a, b in zip(oa, os_[1:]):
            assert a["reduced"].tobytes() == b["reduced"].tobytes() and a["counts"].tolist() == b["counts"].tolist()
            if "emb_next" in a:
                assert a["emb_next"].tobytes() == b["emb_next"].tobytes()
    ctx.close()


@pytest.mark.parametrize("dtype,dim", [("f32", 128), ("bf16", 128), ("f32", 32)])
def test_two_part_lookup_steps_match_the_plain_pipeline_and_the_oracle(dtype, dim):
    """Algorithm 2 with its lookup in two parts (exclusive rows of batch t+2 fetched on the side stream during
    iteration t, collision rows of batch t+1 after the priority pass): tables, states and merged batches bit for
    bit as from the one-part pipeline, which in turn matches the oracle; the oracle's own two-part run agrees."""
    ctx = fs.Context(max_ids=20000, max_dim=256)
    rng = np.random.default_rng(4242)
    rows = 30000
    table = rand_table(rng, rows, dim, dtype)
    state = np.zeros(rows, np.float32)
    its = make_its(rng, rows, dim, 7)
    ts, ss, os_ = run_pipelined(ctx, table, state, its, 0.01, 1e-8)
    view = torch.int16 if dtype == "bf16" else torch.int32
    # the oracle, taking the lookup in two parts as the algorithm does
    wo, so = table.copy(), state.copy()
    merged = O.run_two_phase(wo, so, [it.values for it in its], [it.grads for it in its], 0.01, 1e-8)
    for ahead, sync_each, threaded, disturb in ((False, True, True, None), (False, False, True, None),
                                                ("index", True, True, None), ("batch2", False, True, None),
                                                ("batch2_last_step", False, False, None), ("batch3_last_step", True, True, None),
                                                (True, True, False, None), ("batch2", True, True, 3), (False, True, True, 1)):
        ctx.lib.fs_ctx_set_threaded_enqueue(ctx.handle, 1 if threaded else 0)
        ta, sa, oa = run_pipelined(ctx, table, state, its, 0.01, 1e-8, ahead=ahead, sync_each=sync_each, two_part=True,
                                   disturb=disturb)
        what = f"ahead={ahead} sync_each={sync_each} threaded={threaded} disturb={disturb}"
        assert torch.equal(ta.view(view), ts.view(view)), what
        assert torch.equal(sa, ss), what
        for t, (a, b) in enumerate(zip(oa, os_)):
            assert a["reduced"].tobytes() == b["reduced"].tobytes(), what
            assert a["counts"].tolist() == b["counts"].tolist(), what
            if "emb_next" in a:
                assert a["emb_next"].tobytes() == b["emb_next"].tobytes(), (what, t)
                if dtype == "f32":
                    assert_close_f32(a["emb_next"], merged[t], f"merged batch of iteration {t + 1}")
                else:
                    assert_bf16_within_1ulp(a["emb_next"], merged[t], f"merged batch of iteration {t + 1}")
    ctx.lib.fs_ctx_set_threaded_enqueue(ctx.handle, 1)
    ctx.close()


@pytest.mark.parametrize("dtype,dim,n", [("f32", 128, 5000), ("bf16", 64, 3001), ("f32", 256, 700), ("f32", 8, 0)])
def test_class_lookup_matches_oracle(dtype, dim, n):
    """fs_gather_jagged_class: each part copies exactly the occurrences of its kind of row and leaves the
    others alone; both parts together are the whole lookup."""
    rng = np.random.default_rng(17 + n)
    rows = 4000
    ctx = fs.Context(max_ids=max(n, 16), max_dim=dim)
    table = rand_table(rng, rows, dim, dtype)
    values = zipf_ids(rng, n, rows, a=1.1) if n else np.empty(0, np.int64)
    u_t = np.unique(zipf_ids(rng, 3000, rows, a=1.1))
    lay = O.unique_ids(values, rows)
    flag = np.isin(lay["unique"], u_t).astype(np.uint8)
    d_table, d_values = table_to_dev(table), dev(values)
    d_inv, d_flag = dev(lay["inverse"].astype(np.int32)), dev(flag if flag.size else np.zeros(1, np.uint8))
    view = torch.int16 if dtype == "bf16" else torch.int32
    for order in ((0,), (1,), (0, 1), (1, 0)):
        out = torch.empty((n, dim), dtype=d_table.dtype, device="cuda")
        out.view(view).fill_(-3)
        want = table_to_host(out).copy()
        for which in order:
            fs.fs_gather_jagged_class(ctx, d_table, d_values, None, d_inv, d_flag, which, out)
            O.gather_jagged_class(table, values, u_t, which, want)
        assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
        assert table_to_host(out).tobytes() == want.tobytes(), order
    if n:
        with pytest.raises(fs.FreeScaleError) as e:
            fs.fs_gather_jagged_class(ctx, d_table, d_values, None, d_inv, d_flag, 2, out)
        assert e.value.code == fs.FS_EINVAL
    ctx.close()


def test_balancer_calls_between_the_steps_leave_the_pipeline_alone():
    """The partitioner and the jagged shuffles use the context's index workspace; called between pipelined
    steps (they first wait for what the side streams still do with it) they must neither disturb the steps nor
    be disturbed: same table, state and batches as without them, and their own results as from the oracle."""
    ctx = fs.Context(max_ids=20000, max_dim=128)
    rng = np.random.default_rng(31)
    rows, dim = 30000, 64
    table = rand_table(rng, rows, dim, "f32")
    state = np.zeros(rows, np.float32)
    its = make_its(rng, rows, dim, 6)
    ts, ss, os_ = run_pipelined(ctx, table, state, its, 0.01, 1e-8)
    lens = rng.integers(0, 500, size=3000).astype(np.int64)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    values = rng.integers(0, rows, size=int(offsets[-1])).astype(np.int64)
    d_lens, d_offsets, d_values = dev(lens), dev(offsets), dev(values)
    want_s, want_r = O.partition_fbs(lens, 16)
    want_v, want_o = O.jagged_indexed_permute(values, offsets, want_s)
    got = []

    def between(t):
        sample_of, rank_off = fs.fs_partition_fbs(ctx, d_lens, 500, 16)
        out, out_off = fs.fs_jagged_indexed_permute(ctx, d_values, d_offsets, sample_of, values.shape[0])
        got.append((sample_of, rank_off, out, out_off))

    for ahead, sync_each in (("batch2", False), (False, False), ("index", True)):
        got.clear()
        ta, sa, oa = run_pipelined(ctx, table, state, its, 0.01, 1e-8, ahead=ahead, sync_each=sync_each, between=between)
        assert torch.equal(ta, ts) and torch.equal(sa, ss), ahead
        for a, b in zip(oa, os_):
            if "emb_next" in a:
                assert a["emb_next"].tobytes() == b["emb_next"].tobytes(), ahead
        for sample_of, rank_off, out, out_off in got:
            assert sample_of.cpu().numpy().tolist() == want_s.tolist() and rank_off.cpu().numpy().tolist() == want_r.tolist()
            assert out.cpu().numpy().tolist() == want_v.tolist() and out_off.cpu().numpy().tolist() == want_o.tolist()
    ctx.close()


def test_index_halves_of_different_tables_share_their_launches():
    """One fs_step_forward_ahead_batch call for records of four different tables (rows, dims, dtypes, batch sizes
    all different, one of them without a lookahead batch); each table's step then only waits for its part.
    Everything bit for bit as with one self-contained step per table."""
    rng = np.random.default_rng(77)
    specs = [(30000, 128, "f32", 5000, 4000), (700, 64, "bf16", 9000, 9500), (100000, 32, "f32", 300, 0),
             (5000, 256, "f32", 1, 7)]
    ctx = fs.Context(max_ids=10000, max_dim=256)
    tabs = []
    for rows, dim, dtype, n, n1 in specs:
        t = It()
        t.table, t.state = rand_table(rng, rows, dim, dtype), (rng.random(rows) * 0.1).astype(np.float32)
        t.rows, t.dim, t.dtype = rows, dim, dtype
        t.ids = zipf_ids(rng, n, rows, a=1.1)
        t.ids1 = zipf_ids(rng, n1, rows, a=1.1) if n1 else None
        t.offs1 = np.array([0, n1 // 3, n1], dtype=np.int64) if n1 else None
        t.grads = rng.standard_normal((n, dim)).astype(np.float32)
        tabs.append(t)

    def run(batched):
        outs = []
        bufs = []
        for t in tabs:
            d_table, d_state = table_to_dev(t.table), dev(t.state)
            lay = fs.fs_unique_ids(ctx, dev(t.ids), t.rows)
            n1 = 0 if t.ids1 is None else len(t.ids1)
            lay1 = fs.alloc_layout(n1, "cuda") if n1 else None
            sp = fs.alloc_split(len(t.ids), n1, "cuda")
            emb = torch.empty((n1, t.dim), dtype=d_table.dtype, device="cuda") if n1 else None
            # the record holds plain pointers: the inputs stay alive (and in place) until everything has run
            keep = (dev(t.grads), dev(t.ids1) if n1 else None, dev(t.offs1) if n1 else None)
            args = fs.make_step_args(d_table, d_state, 0.02, 1e-8, lay, keep[0], keep[1], keep[2], lay1, sp, None, emb)
            bufs.append((d_table, d_state, lay, lay1, sp, emb, args, keep))
        if batched:
            fs.fs_step_forward_ahead_batch(ctx, [b[6] for b in bufs])
        for b in bufs:
            fs.fs_prioritized_step(ctx, b[6])
        assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
        for d_table, d_state, lay, lay1, sp, emb, args, _ in bufs:
            view = torch.int16 if d_table.dtype == torch.bfloat16 else torch.int32
            outs.append((d_table.view(view).cpu().numpy(), d_state.cpu().numpy(), sp["counts"].cpu().numpy(),
                         None if emb is None else emb.view(view).cpu().numpy(),
                         None if lay1 is None else lay1["unique"][:int(lay1["n_unique"].item())].cpu().numpy()))
        return outs

    plain, shared = run(False), run(True)
    for a, b in zip(plain, shared):
        for x, y in zip(a, b):
            assert (x is None and y is None) or x.tobytes() == y.tobytes()
    # and the plain run is right: final rows of the first table against the oracle
    t = tabs[0]
    t_ref, s_ref = t.table.copy(), t.state.copy()
    O.step(t_ref, s_ref, O.unique_ids(t.ids, t.rows), t.grads, t.ids1, t.offs1, 0.02, 1e-8)
    assert_rows_close(plain[0][0].view(np.float32).reshape(t.table.shape), t_ref, "rows of table 0")
    with pytest.raises(fs.FreeScaleError) as e:                     # more records than a batch takes
        fs.fs_step_forward_ahead_batch(ctx, [fs.fs_step_args()] * (fs.FS_MAX_AHEAD_BATCH + 1))
    assert e.value.code == fs.FS_EINVAL
    ctx.close()


@pytest.mark.parametrize("ahead,two_part", [(True, False), (False, False), (True, True), (False, True)])
def test_multi_table_step_matches_one_call_per_table(ahead, two_part):
    """fs_prioritized_step_pipelined_multi over six tables (different rows, dims, dtypes, batch sizes), the index
    halves of all of them in shared launches two iterations ahead (or done by the calls themselves): tables,
    states and gathered rows bit for bit as from one pipelined call per table.  two_part: the same through
    fs_prioritized_step_two_part_multi, every merged batch compared with the plain lookup on the table of its time."""
    rng = np.random.default_rng(99)
    # three tables of one row width and two of another share their launches; the sixth is on its own
    specs = [(30000, 128, "f32", 300), (2000, 64, "bf16", 120), (50000, 128, "f32", 40), (7000, 128, "f32", 500),
             (900, 64, "bf16", 200), (50000, 32, "f32", 40)]
    T = 6
    ctx = fs.Context(max_ids=20000, max_dim=128)
    tabs = []
    for rows, dim, dtype, max_len in specs:
        t = It()
        t.table, t.state = rand_table(rng, rows, dim, dtype), np.zeros(rows, np.float32)
        t.its = make_its(rng, rows, dim, T, users=30, max_len=max_len)
        tabs.append(t)
    # reference: one pipelined call per table and iteration
    ref = [run_pipelined(ctx, t.table, t.state, t.its, 0.01, 1e-8, ahead="index" if ahead else False, sync_each=False)
           for t in tabs]
    L, P = 6, 5
    for t in tabs:
        t.d_table, t.d_state = table_to_dev(t.table), dev(t.state)
        t.vals = [dev(it.values) for it in t.its]
        t.offs = [dev(it.offsets) for it in t.its]
        t.grads = [dev(it.grads) for it in t.its]
        nmax = max(v.numel() for v in t.vals)
        t.layouts = [fs.alloc_layout(nmax, "cuda") for _ in range(L)]
        t.splits = [fs.alloc_split(nmax, nmax, "cuda") for _ in range(P)]
        t.embs = [torch.empty((nmax, t.table.shape[1]), dtype=t.d_table.dtype, device="cuda") for _ in range(3)]
        t.args = []
        for s_ in range(T):
            lay = dict(t.layouts[s_ % L]); lay["n"] = t.vals[s_].numel()
            last = s_ == T - 1
            t.args.append(fs.make_step_args(t.d_table, t.d_state, 0.01, 1e-8, lay, t.grads[s_],
                                            None if last else t.vals[s_ + 1], None if last else t.offs[s_ + 1],
                                            None if last else t.layouts[(s_ + 1) % L], t.splits[s_ % P], None,
                                            None if last else t.embs[s_ % 3]))
        fs.fs_unique_ids(ctx, t.vals[0], t.table.shape[0], out=t.layouts[0])

    def index_halves(s_):
        if ahead and s_ < T:
            fs.fs_step_forward_ahead_batch(ctx, [t.args[s_] for t in tabs])

    if ahead:
        index_halves(0)
        index_halves(1)
    else:
        for t in tabs:
            fs.fs_step_forward(ctx, t.args[0])
    for s_ in range(T):
        index_halves(s_ + 2)
        cur = fs.step_args_array([t.args[s_] for t in tabs])
        nxt = fs.step_args_array([t.args[s_ + 1] for t in tabs]) if s_ + 1 < T else None
        if two_part:
            fs.fs_prioritized_step_two_part_multi(ctx, cur, nxt)
            if s_ + 1 < T:
                # the merged batch of every table against the plain lookup on the table as it stands: the rows
                # of the batch are final once the priority pass is through (stream order does the waiting)
                for t in tabs:
                    n1 = t.vals[s_ + 1].numel()
                    want = fs.fs_gather_jagged(ctx, t.d_table, t.vals[s_ + 1], t.offs[s_ + 1])
                    view = torch.int16 if t.d_table.dtype == torch.bfloat16 else torch.int32
                    assert torch.equal(t.embs[s_ % 3][:n1].view(view), want.view(view)), (s_, t.table.shape)
        else:
            fs.fs_prioritized_step_pipelined_multi(ctx, cur, nxt)
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    for t, (r_table, r_state, _) in zip(tabs, ref):
        view = torch.int16 if t.d_table.dtype == torch.bfloat16 else torch.int32
        assert torch.equal(t.d_table.view(view), r_table.view(view))
        assert torch.equal(t.d_state, r_state)
    with pytest.raises(fs.FreeScaleError) as e:                     # more tables than a call takes
        fs.fs_prioritized_step_pipelined_multi(ctx, fs.step_args_array([tabs[0].args[0]] * (fs.FS_MAX_STEP_TABLES + 1)), None)
    assert e.value.code == fs.FS_EINVAL
    ctx.close()


def test_batch_of_index_halves_with_empty_records():
    """A batch whose records are degenerate in every way a record can be: no gradients (empty iteration) but a
    lookahead batch, gradients but no lookahead, both empty, and an ordinary one: counts, class extents and the
    layouts of the lookahead batches must come out as from the plain calls."""
    rng = np.random.default_rng(5)
    rows, dim = 900, 32
    ctx = fs.Context(max_ids=4000, max_dim=dim)
    d_table, d_state = table_to_dev(rand_table(rng, rows, dim, "f32")), torch.zeros(rows, device="cuda")
    cases = [(0, 700), (600, 0), (0, 0), (3000, 2500)]
    keep, recs, want = [], [], []
    for n, n1 in cases:
        ids = zipf_ids(rng, n, rows, a=1.1) if n else np.empty(0, np.int64)
        ids1 = zipf_ids(rng, n1, rows, a=1.1) if n1 else None
        lay = fs.fs_unique_ids(ctx, dev(ids), rows) if n else fs.alloc_layout(0, "cuda")
        lay["n"] = n
        lay1 = fs.alloc_layout(n1, "cuda") if n1 else None
        sp = fs.alloc_split(max(n, 1), max(n1, 1), "cuda")
        sp["counts"].fill_(-7); sp["class_pos"].fill_(-7)
        bufs = (dev(rng.standard_normal((max(n, 1), dim)).astype(np.float32)), dev(ids1) if n1 else None,
                dev(np.array([0, n1], dtype=np.int64)) if n1 else None,
                torch.empty((n1, dim), device="cuda") if n1 else None)
        keep.append((lay, lay1, sp, bufs))
        recs.append(fs.make_step_args(d_table, d_state, 0.01, 1e-8, lay, bufs[0], bufs[1], bufs[2], lay1, sp, None, bufs[3]))
        lay_o = O.unique_ids(ids, rows)
        lay1_o = O.unique_ids(ids1, rows) if n1 else None
        sp_o = O.collision_split(lay_o["unique"], lay1_o["unique"] if n1 else np.empty(0, np.int64))
        want.append((lay1_o, sp_o))
    fs.fs_step_forward_ahead_batch(ctx, recs)
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    for (lay, lay1, sp, _), (lay1_o, sp_o), (n, n1) in zip(keep, want, cases):
        assert sp["counts"].cpu().tolist() == [len(sp_o["co"]), len(sp_o["ex"]), len(sp_o["ex_next"])], (n, n1)
        cp = sp["class_pos"].cpu().tolist()
        assert 0 <= cp[0] <= cp[1] <= n, (n, n1, cp)
        if n1:
            u1 = int(lay1["n_unique"].item())
            assert u1 == len(lay1_o["unique"])
            assert np.array_equal(lay1["unique"][:u1].cpu().numpy(), lay1_o["unique"])
            assert np.array_equal(lay1["perm"][:n1].cpu().numpy(), lay1_o["perm"])
            assert np.array_equal(sp["ex_next"][:len(sp_o["ex_next"])].cpu().numpy(), sp_o["ex_next"])
    ctx.close()


def _ping_pong(ctx, table, state, its, steps, use_graph):
    """Two batches stepped back and forth (three layout buffers, two split buffers: period 6)."""
    d_table, d_state = table_to_dev(table), dev(state)
    num_rows, dim = table.shape
    d_vals = [dev(it.values) for it in its]
    d_offs = [dev(it.offsets) for it in its]
    d_grads = [dev(it.grads) for it in its]
    n = [v.numel() for v in d_vals]
    nmax = max(n)
    layouts = [fs.alloc_layout(nmax, "cuda") for _ in range(3)]
    splits = [fs.alloc_split(nmax, nmax, "cuda") for _ in range(3)]
    reduced = [torch.empty((nmax, dim), dtype=torch.float32, device="cuda") for _ in range(2)]
    embs = [torch.empty((n[0], dim), dtype=d_table.dtype, device="cuda"),
            torch.empty((n[1], dim), dtype=d_table.dtype, device="cuda")]

    def args_for(s):
        lay = dict(layouts[s % 3]); lay["n"] = n[s % 2]
        nb = (s + 1) % 2
        return fs.make_step_args(d_table, d_state, 0.01, 1e-8, lay, d_grads[s % 2], d_vals[nb], d_offs[nb],
                                 layouts[(s + 1) % 3], splits[s % 3], reduced[s % 2], embs[nb])

    args = [args_for(s) for s in range(6)]
    fs.fs_unique_ids(ctx, d_vals[0], num_rows, out=layouts[0])
    fs.fs_step_forward(ctx, args[0])
    graphs = [fs.fs_graph_capture_pipelined(ctx, args[s], args[(s + 1) % 6]) for s in range(6)] if use_graph else None
    snaps = []
    for s in range(steps):
        if use_graph:
            fs.fs_graph_launch(ctx, graphs[s % 6])
        else:
            fs.fs_prioritized_step_pipelined(ctx, args[s % 6], args[(s + 1) % 6])
        # eager work and a synchronisation between replays
        assert fs.fs_check_async(ctx) == fs.FS_OK
        snaps.append((d_table.clone(), d_state.clone(), reduced[s % 2].clone(), embs[(s + 1) % 2].clone(),
                      splits[s % 3]["counts"].clone()))
    if use_graph:
        for g in graphs:
            fs.fs_graph_destroy(ctx, g)
    return snaps


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_graph_replays_match_eager_steps_bitwise(dtype):
    ctx = fs.Context(max_ids=20000, max_dim=128)
    rng = np.random.default_rng(31)
    rows, dim = 25000, 128
    table = rand_table(rng, rows, dim, dtype)
    state = np.zeros(rows, np.float32)
    its = make_its(rng, rows, dim, 2)
    eager = _ping_pong(ctx, table, state, its, 13, use_graph=False)
    graph = _ping_pong(ctx, table, state, its, 13, use_graph=True)
    view = torch.int16 if dtype == "bf16" else torch.int32
    for s, (e, g) in enumerate(zip(eager, graph)):
        assert torch.equal(e[0].view(view), g[0].view(view)), f"table after replay {s}"
        assert torch.equal(e[1], g[1]), f"state after replay {s}"
        assert torch.equal(e[3].view(view), g[3].view(view)), f"gathered rows after replay {s}"
        assert torch.equal(e[4], g[4]), f"split counts after replay {s}"
    ctx.close()


@pytest.mark.parametrize("seed", range(8))
def test_random_shapes_and_schedules_match_the_oracle(seed):
    """Seeded random table shapes, batch sizes, iteration counts and schedules (ahead mode, waits between the calls,
    enqueueing threads, one-part or two-part lookup): every one must give the oracle's run."""
    rng = np.random.default_rng(9000 + seed)
    dtype = ("f32", "bf16")[int(rng.integers(0, 2))]
    dim = int(rng.choice([8, 32, 64, 96, 128, 256]))
    rows = int(rng.choice([50, 3000, 200000]))
    T = int(rng.integers(2, 9))
    users, max_len = int(rng.integers(1, 60)), int(rng.choice([3, 40, 400]))
    ahead = [False, True, "last_step", "index", "index_last_step", "batch2", "batch3_last_step", "batch4"][int(rng.integers(0, 8))]
    sync_each, threaded, two_part = bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), seed % 2 == 1
    what = f"seed={seed} {dtype} dim={dim} rows={rows} T={T} users={users} max_len={max_len} ahead={ahead} " \
           f"sync_each={sync_each} threaded={threaded} two_part={two_part}"
    print(what, flush=True)
    table = rand_table(rng, rows, dim, dtype)
    state = (rng.random(rows) * 0.1).astype(np.float32)
    its = make_its(rng, rows, dim, T, users=users, max_len=max_len)
    ctx = fs.Context(max_ids=max(max(len(it.values) for it in its), 16), max_dim=dim)
    ctx.lib.fs_ctx_set_threaded_enqueue(ctx.handle, 1 if threaded else 0)
    ta, sa, oa = run_pipelined(ctx, table, state, its, 0.01, 1e-8, ahead=ahead, sync_each=sync_each, two_part=two_part)
    t_ref, s_ref, want = run_steps_oracle(table, state, its, 0.01, 1e-8)
    assert_rows_close(table_to_host(ta), t_ref, what)
    assert_close_f32(sa.cpu().numpy(), s_ref, what)
    for t, a in enumerate(oa):
        w = want[t + 1]
        sp = w["split"]
        assert a["counts"].tolist() == [len(sp["co"]), len(sp["ex"]), len(sp["ex_next"])], (what, t)
        assert_close_f32(a["reduced"], w["reduced"], f"{what} reduced {t}")
        if "emb_next" in a:
            assert_rows_close(a["emb_next"], w["emb_next"], f"{what} emb {t}")
    ctx.lib.fs_ctx_set_threaded_enqueue(ctx.handle, 1)
    ctx.close()
