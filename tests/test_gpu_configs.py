"""Full-size parity of the five workload configurations, in the launch configuration bench.py
times (pipelined steps, side stream, threaded enqueue).

The tables of configurations 1-4 are too big to hold on the host, so they are filled on the GPU
by the counter-based hash rule and the oracle works on a table that holds only the touched rows
(order-preserving renumbering: ascending order, slots, permutations and the collision partition
are unchanged by it).  Everything the path produces is compared: layout of every lookahead batch,
collision partition, reduced gradients, gathered rows, final rows and Adagrad state of every
touched row; a sample of untouched rows must still equal the initialisation rule bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_24073_amd as fs
from fs_workloads import CONFIGS, compact_rows, hash_init_rows, make_iterations
from helpers import assert_close_f32, assert_rows_close, exact_f32_to_bf16_bits, table_to_host

pytestmark = pytest.mark.gpu


def run_pipelined_full(ctx, d_table, d_state, its, lr, eps, collect=True, two_part=False):
    """All iterations through fs_prioritized_step_pipelined.

    collect=True: wait after every call and return host copies of everything it produced.
    collect=False: no wait between the calls (the way a training loop and bench.py drive it); only
    the table and the state are left to look at.
    two_part: through fs_prioritized_step_two_part_multi (the lookup in the two parts of Algorithm 2; three
    output batches in rotation).
    """
    dev = d_table.device
    num_rows, dim = d_table.shape
    T = len(its)
    d_vals = [torch.from_numpy(it.values).to(dev) for it in its]
    d_offs = [torch.from_numpy(it.offsets).to(dev) for it in its]
    n = [v.numel() for v in d_vals]
    nmax = max(n)
    layouts = [fs.alloc_layout(nmax, dev) for _ in range(3)]
    splits = [fs.alloc_split(nmax, nmax, dev) for _ in range(3)]
    reduced = [torch.empty((nmax, dim), dtype=torch.float32, device=dev) for _ in range(2)]
    E = 3 if two_part else 2
    embs = [torch.empty((nmax, dim), dtype=d_table.dtype, device=dev) for _ in range(E)]
    grads = [None, None]

    def args_for(t):
        lay_t = dict(layouts[t % 3]); lay_t["n"] = n[t]
        last = t == T - 1
        return fs.make_step_args(d_table, d_state, lr, eps, lay_t, grads[t % 2], None if last else d_vals[t + 1],
                                 None if last else d_offs[t + 1], None if last else layouts[(t + 1) % 3],
                                 splits[t % 3], reduced[t % 2], None if last else embs[t % E])

    fs.fs_unique_ids(ctx, d_vals[0], num_rows, out=layouts[0])
    emb0 = fs.fs_gather_jagged(ctx, d_table, d_vals[0], d_offs[0])
    outs = [{"emb": table_to_host(emb0)}]
    del emb0
    grads[0] = torch.from_numpy(its[0].grads).to(dev)
    cur = args_for(0)
    fs.fs_step_forward(ctx, cur)
    for t in range(T):
        nxt = None
        if t + 1 < T:
            grads[(t + 1) % 2] = torch.from_numpy(its[t + 1].grads).to(dev)
            nxt = args_for(t + 1)
        if two_part:
            fs.fs_prioritized_step_two_part_multi(ctx, fs.step_args_array([cur]),
                                                  fs.step_args_array([nxt]) if nxt is not None else None)
        else:
            fs.fs_prioritized_step_pipelined(ctx, cur, nxt)
        if not collect:
            cur = nxt
            continue
        assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
        u = int(layouts[t % 3]["n_unique"].item())
        sp = splits[t % 3]
        counts = sp["counts"].cpu().numpy()
        rec = {"reduced": reduced[t % 2][:u].cpu().numpy(), "counts": counts}
        for name, cnt in (("co", counts[0]), ("ex", counts[1]), ("ex_next", counts[2])):
            rec[name] = sp[name][:cnt].cpu().numpy()
            rec[name + "_slot"] = sp[name + "_slot"][:cnt].cpu().numpy()
        if t + 1 < T:
            ln = layouts[(t + 1) % 3]
            u1 = int(ln["n_unique"].item())
            rec["layout_next"] = {"unique": ln["unique"][:u1].cpu().numpy(),
                                  "seg_offsets": ln["seg_offsets"][:u1 + 1].cpu().numpy(),
                                  "perm": ln["perm"][:n[t + 1]].cpu().numpy(),
                                  "inverse": ln["inverse"][:n[t + 1]].cpu().numpy()}
            rec["emb_next"] = table_to_host(embs[t % E][:n[t + 1]])
        outs.append(rec)
        cur = nxt
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    return outs


def check_config_table(cfg_index, table_index):
    cfg = CONFIGS[cfg_index]
    tab = cfg.tables[table_index]
    its_all = make_iterations(cfg, tables=[table_index])
    its = [x[table_index] for x in its_all]
    del its_all
    dim = tab.dim
    # ---- oracle on the touched rows
    touched, remapped = compact_rows([it.values for it in its])
    if tab.init == "hash":
        w0 = np.concatenate([hash_init_rows(touched[i:i + 65536], dim, tab.dtype)
                             for i in range(0, len(touched), 65536)])
    else:
        full = (np.random.default_rng(0xF5CA1E00).standard_normal((tab.num_rows, dim)) * 0.01).astype(np.float32)
        w0 = full[touched]
    t_ref = exact_f32_to_bf16_bits(w0) if tab.dtype == "bf16" else w0.copy()
    s_ref = np.zeros(len(touched), np.float32)
    layout = O.unique_ids(remapped[0], len(touched))
    want = [{"emb": O.gather_jagged(t_ref, remapped[0], its[0].offsets)}]
    for t in range(len(its)):
        last = t == len(its) - 1
        r = O.step(t_ref, s_ref, layout, its[t].grads, None if last else remapped[t + 1],
                   None if last else its[t + 1].offsets, cfg.lr, cfg.eps)
        want.append(r)
        layout = r["layout_next"]

    # ---- GPU on the full table
    tdtype = torch.float32 if tab.dtype == "f32" else torch.bfloat16
    ctx = fs.Context(max_ids=max(len(it.values) for it in its), max_dim=dim)
    d_table = torch.empty((tab.num_rows, dim), dtype=tdtype, device="cuda")
    if tab.init == "hash":
        fs.fs_init_table_hash(ctx, d_table)
    else:
        d_table.copy_(torch.from_numpy(full))
    d_state = torch.zeros(tab.num_rows, dtype=torch.float32, device="cuda")
    got = run_pipelined_full(ctx, d_table, d_state, its, cfg.lr, cfg.eps)

    # ---- compare (oracle IDs are indices into `touched`)
    assert_rows_close(got[0]["emb"], want[0]["emb"], "initial gather")
    assert got[0]["emb"].tobytes() == want[0]["emb"].tobytes()          # no update yet: bit-exact
    for t, (g, w) in enumerate(zip(got[1:], want[1:])):
        sp = w["split"]
        assert g["counts"].tolist() == [len(sp["co"]), len(sp["ex"]), len(sp["ex_next"])], f"iteration {t}"
        for name in ("co", "ex", "ex_next"):
            assert np.array_equal(g[name], touched[sp[name]]), f"iteration {t} {name}"
            assert np.array_equal(g[name + "_slot"], sp[name + "_slot"]), f"iteration {t} {name}_slot"
        assert_close_f32(g["reduced"], w["reduced"], f"iteration {t} reduced gradients")
        if w["layout_next"] is not None:
            assert np.array_equal(g["layout_next"]["unique"], touched[w["layout_next"]["unique"]])
            for k in ("seg_offsets", "perm", "inverse"):
                assert np.array_equal(g["layout_next"][k], w["layout_next"][k]), f"iteration {t} layout {k}"
            assert_rows_close(g["emb_next"], w["emb_next"], f"iteration {t} gathered rows")
    idx = torch.from_numpy(touched).cuda()
    assert_rows_close(table_to_host(d_table[idx]), t_ref, "final rows of the touched set")
    assert_close_f32(d_state[idx].cpu().numpy(), s_ref, "final adagrad state")
    # untouched rows: still the initialisation rule, state still zero
    rng = np.random.default_rng(5)
    cand = rng.integers(0, tab.num_rows, size=4000)
    cand = np.setdiff1d(cand, touched)[:2000]
    if tab.init == "hash":
        rule = hash_init_rows(cand, dim, tab.dtype)
        rule = exact_f32_to_bf16_bits(rule) if tab.dtype == "bf16" else rule
    else:
        rule = full[cand]
    cidx = torch.from_numpy(cand).cuda()
    assert table_to_host(d_table[cidx]).tobytes() == rule.tobytes()
    assert float(d_state[cidx].abs().max().item()) == 0.0
    # the same iterations again without a wait between the calls: same bits in table and state
    if tab.init == "hash":
        rows_1, state_1 = d_table[idx].clone(), d_state[idx].clone()
        fs.fs_init_table_hash(ctx, d_table)
        d_state.zero_()
        run_pipelined_full(ctx, d_table, d_state, its, cfg.lr, cfg.eps, collect=False)
        assert torch.equal(d_table[idx].view(torch.int16 if tab.dtype == "bf16" else torch.int32),
                           rows_1.view(torch.int16 if tab.dtype == "bf16" else torch.int32))
        assert torch.equal(d_state[idx], state_1)
        if cfg_index in (1, 3):
            # and with the lookup in its two parts: every merged batch, the table and the state bit for bit
            fs.fs_init_table_hash(ctx, d_table)
            d_state.zero_()
            got2 = run_pipelined_full(ctx, d_table, d_state, its, cfg.lr, cfg.eps, two_part=True)
            for t, (g2, g) in enumerate(zip(got2[1:], got[1:])):
                if "emb_next" in g:
                    assert g2["emb_next"].tobytes() == g["emb_next"].tobytes(), f"two-part lookup, iteration {t}"
            assert torch.equal(d_table[idx].view(torch.int16 if tab.dtype == "bf16" else torch.int32),
                               rows_1.view(torch.int16 if tab.dtype == "bf16" else torch.int32))
            assert torch.equal(d_state[idx], state_1)
    n_it = [len(it.values) for it in its]
    print(f"config {cfg_index} table {table_index}: N={n_it[:3]} touched={len(touched)} ok")
    ctx.close()
    del d_table, d_state
    torch.cuda.empty_cache()


@pytest.mark.timeout(600)
def test_config0_tiny():
    check_config_table(0, 0)


@pytest.mark.timeout(600)
def test_config1_shard_4m_d128():
    check_config_table(1, 0)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("table_index", range(8))
def test_config2_eight_tables(table_index):
    check_config_table(2, table_index)


@pytest.mark.timeout(600)
def test_config3_long_sequences_bf16():
    check_config_table(3, 0)


@pytest.mark.timeout(900)
def test_config4_streaming_ten_iterations():
    check_config_table(4, 0)
