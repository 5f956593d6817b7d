"""CPU oracle (test infrastructure only): numpy front end of ``freescale_oracle.c``.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  It never imports the HIP binding.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "freescale_oracle.c")
_LIB = os.path.join(_HERE, "libfs_oracle.so")

F32, BF16 = 0, 1
OK, EINVAL, ENOMEM, ERANGE = 0, -1, -2, -5


def build(force: bool = False) -> str:
    """Compile the oracle with the host C compiler (no FMA contraction, plain -O2)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.fso_f32_to_bf16.restype = ctypes.c_uint16
        _lib.fso_f32_to_bf16.argtypes = [ctypes.c_float]
        _lib.fso_bf16_to_f32.restype = ctypes.c_float
        _lib.fso_bf16_to_f32.argtypes = [ctypes.c_uint16]
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where} failed with status {code}")
        self.code = code


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(code: int, where: str) -> None:
    if code != OK:
        raise OracleError(code, where)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def dtype_code(table: np.ndarray) -> int:
    """fp32 tables are float32 arrays; bf16 tables are uint16 arrays of bf16 bit patterns."""
    if table.dtype == np.float32:
        return F32
    if table.dtype == np.uint16:
        return BF16
    raise TypeError(f"table dtype {table.dtype} (want float32, or uint16 holding bf16 bits)")


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Element-wise through the oracle's own scalar conversion (slow; for tests)."""
    x = _c(x, np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    f = lib().fso_f32_to_bf16
    flat_in, flat_out = x.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = f(float(flat_in[i]))
    return out


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    """Exact widening (a bit shift; no arithmetic of the method)."""
    h = _c(h, np.uint16)
    return (h.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---- the five operations ---------------------------------------------------------------
def gather_jagged(table: np.ndarray, values: np.ndarray, offsets: Optional[np.ndarray]) -> np.ndarray:
    assert table.ndim == 2 and table.flags.c_contiguous
    values = _c(values, np.int64)
    n = values.shape[0]
    if offsets is None:
        offsets = np.array([0, n], dtype=np.int64)
    offsets = _c(offsets, np.int64)
    out = np.empty((n, table.shape[1]), dtype=table.dtype)
    rc = lib().fso_gather_jagged(_p(table), ctypes.c_int64(table.shape[0]), ctypes.c_int32(table.shape[1]),
                                 ctypes.c_int(dtype_code(table)), _p(values), _p(offsets),
                                 ctypes.c_int64(offsets.shape[0] - 1), ctypes.c_int64(n), _p(out))
    _check(rc, "fso_gather_jagged")
    return out


def unique_ids(ids: np.ndarray, num_rows: int = 0) -> Dict[str, np.ndarray]:
    ids = _c(ids, np.int64)
    n = ids.shape[0]
    unique = np.empty(max(n, 1), dtype=np.int64)
    seg = np.empty(n + 1, dtype=np.int32)
    perm = np.empty(max(n, 1), dtype=np.int32)
    inv = np.empty(max(n, 1), dtype=np.int32)
    nu = ctypes.c_int64(0)
    rc = lib().fso_unique_ids(_p(ids), ctypes.c_int64(n), ctypes.c_int64(num_rows), _p(unique), _p(seg),
                              _p(perm), _p(inv), ctypes.byref(nu))
    _check(rc, "fso_unique_ids")
    u = nu.value
    return {"unique": unique[:u].copy(), "seg_offsets": seg[:u + 1].copy(), "perm": perm[:n].copy(),
            "inverse": inv[:n].copy(), "n_unique": u}


def collision_split(u_t: np.ndarray, u_t1: np.ndarray) -> Dict[str, np.ndarray]:
    u_t, u_t1 = _c(u_t, np.int64), _c(u_t1, np.int64)
    nt, nt1 = u_t.shape[0], u_t1.shape[0]
    co, cos = np.empty(max(nt, 1), np.int64), np.empty(max(nt, 1), np.int32)
    ex, exs = np.empty(max(nt, 1), np.int64), np.empty(max(nt, 1), np.int32)
    exn, exns = np.empty(max(nt1, 1), np.int64), np.empty(max(nt1, 1), np.int32)
    counts = np.zeros(3, dtype=np.int64)
    rc = lib().fso_collision_split(_p(u_t), ctypes.c_int64(nt), _p(u_t1), ctypes.c_int64(nt1),
                                   _p(co), _p(cos), _p(ex), _p(exs), _p(exn), _p(exns), _p(counts))
    _check(rc, "fso_collision_split")
    a, b, c = (int(x) for x in counts)
    return {"co": co[:a].copy(), "co_slot": cos[:a].copy(), "ex": ex[:b].copy(), "ex_slot": exs[:b].copy(),
            "ex_next": exn[:c].copy(), "ex_next_slot": exns[:c].copy()}


def segment_reduce_grads(grads: np.ndarray, perm: np.ndarray, seg_offsets: np.ndarray) -> np.ndarray:
    grads = _c(grads, np.float32)
    perm, seg_offsets = _c(perm, np.int32), _c(seg_offsets, np.int32)
    n, dim = grads.shape
    nu = seg_offsets.shape[0] - 1
    out = np.empty((nu, dim), dtype=np.float32)
    rc = lib().fso_segment_reduce_grads(_p(grads), ctypes.c_int64(n), ctypes.c_int32(dim), _p(perm),
                                        _p(seg_offsets), ctypes.c_int64(nu), _p(out))
    _check(rc, "fso_segment_reduce_grads")
    return out


def rowwise_adagrad_update(table: np.ndarray, state: np.ndarray, rows: np.ndarray, slots: np.ndarray,
                           reduced: np.ndarray, lr: float, eps: float) -> None:
    """In place on ``table`` and ``state``."""
    assert table.flags.c_contiguous and state.flags.c_contiguous and state.dtype == np.float32
    rows, slots = _c(rows, np.int64), _c(slots, np.int32)
    reduced = _c(reduced, np.float32)
    rc = lib().fso_rowwise_adagrad_update(_p(table), ctypes.c_int(dtype_code(table)), _p(state),
                                          ctypes.c_int64(table.shape[0]), ctypes.c_int32(table.shape[1]),
                                          _p(rows), _p(slots), ctypes.c_int64(rows.shape[0]), _p(reduced),
                                          ctypes.c_float(lr), ctypes.c_float(eps))
    _check(rc, "fso_rowwise_adagrad_update")


def gather_jagged_class(table: np.ndarray, values: np.ndarray, u_t: np.ndarray, which: int, out: np.ndarray) -> None:
    """Lookup of the occurrences whose row is (which=1) / is not (which=0) in u_t, into ``out`` in place."""
    assert table.ndim == 2 and table.flags.c_contiguous and out.flags.c_contiguous
    assert out.dtype == table.dtype and out.shape == (values.shape[0], table.shape[1])
    values = _c(values, np.int64)
    u_t = _c(u_t, np.int64)
    rc = lib().fso_gather_jagged_class(_p(table), ctypes.c_int64(table.shape[0]), ctypes.c_int32(table.shape[1]),
                                       ctypes.c_int(dtype_code(table)), _p(values), ctypes.c_int64(values.shape[0]),
                                       _p(u_t), ctypes.c_int64(u_t.shape[0]), ctypes.c_int(which), _p(out))
    _check(rc, "fso_gather_jagged_class")


def split_grads(grads: np.ndarray, values: np.ndarray, u_t1: np.ndarray) -> Dict[str, np.ndarray]:
    """split(G, I_co, I_ex) of Algorithm 2's Backward: the gradient rows (batch order) of the occurrences whose
    row is / is not in u_t1, with the occurrence numbers of both parts."""
    grads = _c(grads, np.float32)
    values, u_t1 = _c(values, np.int64), _c(u_t1, np.int64)
    n, dim = grads.shape
    assert values.shape[0] == n
    co_i, ex_i = np.empty(max(n, 1), np.int32), np.empty(max(n, 1), np.int32)
    g_co, g_ex = np.empty((max(n, 1), dim), np.float32), np.empty((max(n, 1), dim), np.float32)
    counts = np.zeros(2, dtype=np.int64)
    rc = lib().fso_split_grads(_p(grads), ctypes.c_int64(n), ctypes.c_int32(dim), _p(values), _p(u_t1),
                               ctypes.c_int64(u_t1.shape[0]), _p(co_i), _p(g_co), _p(ex_i), _p(g_ex), _p(counts))
    _check(rc, "fso_split_grads")
    a, b = (int(x) for x in counts)
    return {"co_index": co_i[:a].copy(), "g_co": g_co[:a].copy(), "ex_index": ex_i[:b].copy(), "g_ex": g_ex[:b].copy()}


def partition_fbs(lengths: np.ndarray, n_ranks: int) -> Tuple[np.ndarray, np.ndarray]:
    """FBS partitioner: (sample_of [B] rank-major, rank_offsets [n_ranks + 1])."""
    lengths = _c(lengths, np.int64)
    B = lengths.shape[0]
    sample_of = np.empty(max(B, 1), dtype=np.int32)
    rank_offsets = np.empty(n_ranks + 1, dtype=np.int64)
    rc = lib().fso_partition_fbs(_p(lengths), ctypes.c_int64(B), ctypes.c_int32(n_ranks), _p(sample_of), _p(rank_offsets))
    _check(rc, "fso_partition_fbs")
    return sample_of[:B], rank_offsets


def partition_vbs(lengths: np.ndarray, weight_of_len: np.ndarray, n_ranks: int) -> Tuple[np.ndarray, np.ndarray]:
    """VBS partitioner: (sample_of [B] = the length-sorted order, rank_offsets [n_ranks + 1])."""
    lengths = _c(lengths, np.int64)
    weight_of_len = _c(weight_of_len, np.int64)
    B = lengths.shape[0]
    sample_of = np.empty(max(B, 1), dtype=np.int32)
    rank_offsets = np.empty(n_ranks + 1, dtype=np.int64)
    rc = lib().fso_partition_vbs(_p(lengths), ctypes.c_int64(B), _p(weight_of_len),
                                 ctypes.c_int64(weight_of_len.shape[0] - 1), ctypes.c_int32(n_ranks), _p(sample_of),
                                 _p(rank_offsets))
    _check(rc, "fso_partition_vbs")
    return sample_of[:B], rank_offsets


def jagged_indexed_permute(values: np.ndarray, offsets: np.ndarray, sample_of: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """The samples sample_of[...] of the jagged tensor (values, offsets), concatenated: (out_values, out_offsets)."""
    assert values.flags.c_contiguous
    offsets = _c(offsets, np.int64)
    sample_of = _c(sample_of, np.int32)
    B = offsets.shape[0] - 1
    lens = offsets[1:] - offsets[:-1]
    in_range = sample_of[(sample_of >= 0) & (sample_of < B)]
    total = int(lens[in_range].sum()) if B > 0 else 0
    out = np.empty((total,) + values.shape[1:], dtype=values.dtype)
    out_offsets = np.empty(sample_of.shape[0] + 1, dtype=np.int64)
    elem = values.dtype.itemsize * int(np.prod(values.shape[1:], dtype=np.int64))
    rc = lib().fso_jagged_indexed_permute(_p(values), ctypes.c_int32(elem), _p(offsets), ctypes.c_int64(B), _p(sample_of),
                                          ctypes.c_int64(sample_of.shape[0]), _p(out), _p(out_offsets))
    _check(rc, "fso_jagged_indexed_permute")
    return out, out_offsets


def _shuffle(fn_name, values, offsets, F, B, rank_offsets=None, want_splits=False):
    assert values.flags.c_contiguous
    offsets = _c(offsets, np.int64)
    assert offsets.shape[0] == F * B + 1
    out = np.empty_like(values)
    out_offsets = np.empty(F * B + 1, dtype=np.int64)
    elem = values.dtype.itemsize * int(np.prod(values.shape[1:], dtype=np.int64))
    args = [_p(values), ctypes.c_int32(elem), _p(offsets), ctypes.c_int64(F), ctypes.c_int64(B)]
    splits = None
    if rank_offsets is not None:
        rank_offsets = _c(rank_offsets, np.int64)
        args += [_p(rank_offsets), ctypes.c_int32(rank_offsets.shape[0] - 1)]
    args += [_p(out), _p(out_offsets)]
    if want_splits:
        splits = np.empty(rank_offsets.shape[0] - 1, dtype=np.int64)
        args.append(_p(splits))
    _check(getattr(lib(), fn_name)(*args), fn_name)
    return (out, out_offsets, splits) if want_splits else (out, out_offsets)


def jagged_keyed_transpose(values, offsets, F, B):
    """Feature-major [F keys x B samples] -> batch-major: (out_values, out_offsets)."""
    return _shuffle("fso_jagged_keyed_transpose", values, offsets, F, B)


def jagged_ranged_dispatch(values, offsets, F, B, rank_offsets):
    """Feature-major -> AllToAll input (rank, key, sample): (out_values, out_offsets, splits)."""
    return _shuffle("fso_jagged_ranged_dispatch", values, offsets, F, B, rank_offsets, want_splits=True)


def jagged_ranged_combine(values, offsets, F, B, rank_offsets):
    """AllToAll output (source rank, key, sample) -> feature-major: (out_values, out_offsets)."""
    return _shuffle("fso_jagged_ranged_combine", values, offsets, F, B, rank_offsets)


# ---- one step of the prioritized schedule -------------------------------------------------
SCHEDULES = ("co_then_ex", "ex_then_co", "all_at_once", "gather_between")


def step(table: np.ndarray, state: np.ndarray, layout_t: Dict[str, np.ndarray], grads_t: np.ndarray,
         values_next: Optional[np.ndarray], offsets_next: Optional[np.ndarray], lr: float, eps: float,
         schedule: str = "co_then_ex") -> Dict[str, object]:
    """Iteration t on one shard (Algorithm 2 with the collectives removed).

    layout_t is unique_ids(values_t).  With a lookahead batch (values_next): dedup it, split U_t
    against U_{t+1}, reduce G_t, update the collision rows, update the exclusive rows, gather the
    rows of the lookahead batch.  Without one (last iteration) every row of U_t is exclusive.
    ``schedule`` permutes the order of the passes; all orders must give identical results
    (Section 3.2: strict write-read ordering is only needed on collision rows).
    """
    num_rows = table.shape[0]
    g = segment_reduce_grads(grads_t, layout_t["perm"], layout_t["seg_offsets"])
    u_t = layout_t["unique"]
    if values_next is None:
        layout_next = None
        sp = collision_split(u_t, np.empty(0, dtype=np.int64))
    else:
        layout_next = unique_ids(values_next, num_rows)
        sp = collision_split(u_t, layout_next["unique"])
    emb = None

    def upd(rows, slots):
        rowwise_adagrad_update(table, state, rows, slots, g, lr, eps)

    def gat():
        return None if values_next is None else gather_jagged(table, values_next, offsets_next)

    if schedule == "co_then_ex":
        upd(sp["co"], sp["co_slot"]); upd(sp["ex"], sp["ex_slot"]); emb = gat()
    elif schedule == "ex_then_co":
        upd(sp["ex"], sp["ex_slot"]); upd(sp["co"], sp["co_slot"]); emb = gat()
    elif schedule == "all_at_once":
        upd(u_t, np.arange(u_t.shape[0], dtype=np.int32)); emb = gat()
    elif schedule == "gather_between":
        upd(sp["co"], sp["co_slot"]); emb = gat(); upd(sp["ex"], sp["ex_slot"])
    else:
        raise ValueError(schedule)
    return {"reduced": g, "split": sp, "layout_next": layout_next, "emb_next": emb}


def run_two_phase(table: np.ndarray, state: np.ndarray, values_seq: Sequence[np.ndarray],
                  grads_seq: Sequence[np.ndarray], lr: float, eps: float,
                  prefetch_before_deferred: bool = False) -> List[np.ndarray]:
    """Algorithm 2 over the iterations 0..T-1 of one shard, with its two-part lookup.

    Iteration i owns batch ``values_seq[i]`` and receives ``grads_seq[i]``; ``values_seq`` has one
    batch more than ``grads_seq`` has gradients or the same number (then the last iteration has no
    lookahead).  In the order of the algorithm:

      Forward(i+1's indices): finish update_embedding(I_ex^{i-1}, G_ex^{i-1}); compute_collision(I^i,
        I^{i+1}); E_ex^{i+1} = Lookup(I_ex^{i+1})   - before the gradients of i exist;
      Backward(G^i): E_co^{i+1} = update_embedding(I_co^i, G_co^i) - the rows as the update leaves them;
      next Forward returns merge(E_ex^{i+1}, E_co^{i+1}).

    Returns the merged input batch of every iteration 1..T (the batch of iteration 0 is a plain
    lookup and not returned).  ``prefetch_before_deferred`` plants the mistake of fetching the
    exclusive rows of i+1 before the deferred update of i-1 has landed (for the pins).
    """
    num_rows = table.shape[0]
    layouts = [unique_ids(v, num_rows) for v in values_seq]
    merged: List[np.ndarray] = []
    pending = None                                   # (rows, slots, reduced) of the deferred update
    for i, grads in enumerate(grads_seq):
        lay = layouts[i]
        has_next = i + 1 < len(values_seq)
        nxt = layouts[i + 1]["unique"] if has_next else np.empty(0, dtype=np.int64)
        sp = collision_split(lay["unique"], nxt)
        batch = np.zeros((values_seq[i + 1].shape[0], table.shape[1]), dtype=table.dtype) if has_next else None
        # Forward
        if prefetch_before_deferred and has_next:
            gather_jagged_class(table, values_seq[i + 1], lay["unique"], 0, batch)
        if pending is not None:
            rowwise_adagrad_update(table, state, pending[0], pending[1], pending[2], lr, eps)
        if has_next and not prefetch_before_deferred:
            gather_jagged_class(table, values_seq[i + 1], lay["unique"], 0, batch)
        # Backward
        g = segment_reduce_grads(grads, lay["perm"], lay["seg_offsets"])
        rowwise_adagrad_update(table, state, sp["co"], sp["co_slot"], g, lr, eps)
        if has_next:
            gather_jagged_class(table, values_seq[i + 1], lay["unique"], 1, batch)
            merged.append(batch)
        pending = (sp["ex"], sp["ex_slot"], g)
    if pending is not None:
        rowwise_adagrad_update(table, state, pending[0], pending[1], pending[2], lr, eps)
    return merged
