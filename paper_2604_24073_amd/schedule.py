"""The steady-state call sequence of the pipelined iteration, written once for everything that drives it
(bench.py times it, the full-size parity tests compare its results with the oracle).

Nothing of the method is computed here: the module allocates the rotating buffers, fills argument records
(pointers) and issues the C-ABI calls in their order.  Per step s and group of tables:

    every K steps   fs_step_forward_ahead_batch(records of iterations s+D .. s+D+K-1 of every table of the group)
                    - the index halves, D = K + 1 iterations before their first record is stepped, ordered after
                    the start of the most recent pipelined call (FS_STREAM_LAST_STEP) once there has been one
    every step      fs_prioritized_step_pipelined_multi(cur = records of s, next = records of s + 1)

Iteration s works on batch s mod T of its table (T batches given), with batch (s + 1) mod T as its lookahead.
No call waits for the GPU; `join` is the only barrier.
"""
from __future__ import annotations

import itertools
import math
from typing import Dict, List, Optional, Sequence

import torch

from . import binding as fs


class TableBuffers:
    """One table of a shard: its T batches on the device, the rotating layout / split buffers and the argument
    record of every step of one period."""

    def __init__(self, table: torch.Tensor, state: torch.Tensor, values: Sequence[torch.Tensor],
                 offsets: Sequence[torch.Tensor], grads: Sequence[torch.Tensor], lr: float, eps: float):
        self.table, self.state = table, state
        self.values, self.offsets, self.grads = list(values), list(offsets), list(grads)
        self.lr, self.eps = lr, eps
        self.T = len(self.values)
        self.n = [int(v.numel()) for v in self.values]
        self.dim = int(table.shape[1])
        self.w = table.element_size()
        self.layouts: List[Dict[str, torch.Tensor]] = []
        self.splits: List[Dict[str, torch.Tensor]] = []
        self.embs: List[torch.Tensor] = []
        self.reduced: List[Optional[torch.Tensor]] = []
        self.args: List[fs.fs_step_args] = []

    def allocate(self, L: int, P: int, n_records: int, emb_rotation: Optional[int], keep_reduced: bool,
                 inverse: bool, row_ordered_lookup: bool = True) -> None:
        dev, nmax = self.table.device, max(self.n)
        self.layouts = [fs.alloc_layout(nmax, dev, inverse=inverse, sorted_ids=row_ordered_lookup) for _ in range(L)]
        self.splits = [fs.alloc_split(nmax, nmax, dev) for _ in range(P)]
        # output batches: one per batch of the cycle (each step overwrites the batch it looks ahead to), or
        # `emb_rotation` buffers of the largest size in turn (a test that wants to look at every batch afterwards)
        if emb_rotation is None:
            self.embs = [torch.empty((self.n[b], self.dim), dtype=self.table.dtype, device=dev) for b in range(self.T)]
        else:
            self.embs = [torch.empty((nmax, self.dim), dtype=self.table.dtype, device=dev) for _ in range(emb_rotation)]
        self.reduced = ([torch.empty((nmax, self.dim), dtype=torch.float32, device=dev) for _ in range(2)]
                        if keep_reduced else [None, None])
        self.emb_rotation = emb_rotation
        self.args = [self._record(s, L, P) for s in range(n_records)]

    def emb_of_step(self, s: int) -> torch.Tensor:
        """The buffer that step s gathers its lookahead batch (s + 1) mod T into."""
        if self.emb_rotation is None:
            return self.embs[(s + 1) % self.T]
        return self.embs[s % self.emb_rotation]

    def _record(self, s: int, L: int, P: int) -> fs.fs_step_args:
        b, nb = s % self.T, (s + 1) % self.T
        lay = dict(self.layouts[s % L])
        lay["n"] = self.n[b]
        return fs.make_step_args(self.table, self.state, self.lr, self.eps, lay, self.grads[b], self.values[nb],
                                 self.offsets[nb], self.layouts[(s + 1) % L], self.splits[s % P], self.reduced[s % 2],
                                 self.emb_of_step(s))


def group_tables(tabs: Sequence[TableBuffers], G: int) -> List[List[TableBuffers]]:
    """The tables of a shard in G groups (one context, stream and call sequence each).  Tables of one row width
    share the launches of their class passes and gathers inside a call, so a group should hold few widths, and
    the groups run side by side, so they should be about equally heavy: every assignment is tried (a shard has a
    handful of tables) and the one with the smallest (heaviest group / mean group + 0.05 x launch classes) kept."""
    tabs = list(tabs)
    if G <= 1 or len(tabs) > 12:
        return [tabs[g::max(G, 1)] for g in range(max(G, 1))]
    load = [sum(t.n) * t.dim * t.w for t in tabs]
    mean = sum(load) / G
    best, best_cost = None, None
    for assign in itertools.product(range(G), repeat=len(tabs)):
        if len(set(assign)) < G:
            continue
        heavy = max(sum(l for l, a in zip(load, assign) if a == g) for g in range(G))
        classes = len({(a, t.dim * t.w) for a, t in zip(assign, tabs)})
        cost = heavy / mean + 0.05 * classes
        if best_cost is None or cost < best_cost - 1e-12:
            best, best_cost = assign, cost
    return [[t for t, a in zip(tabs, best) if a == g] for g in range(G)]


_hip = None


def new_hip_stream() -> torch.cuda.Stream:
    """One plain HIP stream (non-blocking, default priority), wrapped for torch's event and wait calls.  A stream
    taken from torch's own pool brings that whole pool of streams into being, and with more streams than the
    chip has hardware queues the step's passes end up sharing queues (measured: 124 instead of 99 us per step)."""
    global _hip
    import ctypes
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
    h = ctypes.c_void_p()
    rc = _hip.hipStreamCreateWithFlags(ctypes.byref(h), ctypes.c_uint(1))     # hipStreamNonBlocking
    if rc != 0 or not h.value:
        raise RuntimeError(f"hipStreamCreateWithFlags failed with {rc}")
    return torch.cuda.ExternalStream(h.value)


class StepLoop:
    """The tables of one shard stepped in `groups` groups; K iterations of every table of a group share one
    chain of index launches (K * tables of the group <= FS_MAX_AHEAD_BATCH)."""

    def __init__(self, tables: Sequence[TableBuffers], groups: int = 1, iters_per_chain: Optional[int] = None,
                 emb_rotation: Optional[int] = None, keep_reduced: bool = False, two_part: bool = False,
                 lookahead: Optional[int] = None, row_ordered_lookup: bool = True):
        self.tables = list(tables)
        G = max(1, min(groups, len(self.tables)))
        self.groups = group_tables(self.tables, G)
        widest = max(len(g) for g in self.groups)
        if widest > min(fs.FS_MAX_AHEAD_BATCH, fs.FS_MAX_STEP_TABLES):
            raise ValueError("more tables in a group than one call takes")
        K = iters_per_chain if iters_per_chain is not None else (2 if widest == 1 else 1)
        self.K = max(1, min(K, fs.FS_MAX_AHEAD_BATCH // widest))
        # a chain is issued D iterations before its first record is stepped (at least K + 1: the chain before it
        # must have been issued); the IDs of a batch are needed D + K iterations before its gradients
        self.D = max(self.K + 1, lookahead if lookahead is not None else self.K + 1)
        self.L, self.P = self.K + self.D + 3, self.K + self.D + 2
        T = {t.T for t in self.tables}
        if len(T) != 1:
            raise ValueError("the tables of a shard step through the same number of batches")
        self.T = T.pop()
        # the argument records repeat with this period (buffer rotations, batches of the cycle, chains)
        self.period = math.lcm(self.L, self.P, self.T, self.K, 2, emb_rotation or 1)
        self.n_records = self.period
        self.two_part = two_part
        for t in self.tables:
            t.allocate(self.L, self.P, self.n_records, emb_rotation, keep_reduced, inverse=two_part,
                       row_ordered_lookup=row_ordered_lookup)
        self.ctxs = [fs.Context(max_ids=max(max(t.n) for t in g), max_dim=max(t.dim for t in g)) for g in self.groups]
        # The chip gives a process four hardware queues and a context owns three streams, so the first group is
        # stepped on the default stream (the fourth queue); a stream of its own for it costs 25 % (5 queues in use).
        self.streams = [torch.cuda.default_stream()] + [new_hip_stream() for _ in self.groups[1:]]
        # one contiguous array of records per group and step: what the step call takes; and per chain start
        self.step_records = [[fs.step_args_array([t.args[s] for t in g]) for s in range(self.n_records)]
                             for g in self.groups]
        self.chain_records = [{s: fs.step_args_array([t.args[self._rec(s + k)] for k in range(self.K) for t in g])
                               for s in range(0, self.n_records, self.K)} for g in self.groups]
        self.stepped = False
        self.primed = False

    def _rec(self, s: int) -> int:
        return s % self.n_records

    def close(self) -> None:
        for c in self.ctxs:
            c.close()
        self.ctxs = []

    def _ahead(self, first: int) -> None:
        """The index halves of iterations first .. first+K-1, when `first` starts a chain."""
        if first % self.K != 0:
            return
        for c, st, chains in zip(self.ctxs, self.streams, self.chain_records):
            fs.fs_step_forward_ahead_batch(c, chains[first % self.n_records],
                                           stream=fs.FS_STREAM_LAST_STEP if self.stepped else st)

    def prime(self) -> None:
        """Layout of batch 0 (no earlier step produced it) and the chains a loop that had run for ever would have
        issued before step 0."""
        for c, st, g in zip(self.ctxs, self.streams, self.groups):
            for t in g:
                fs.fs_unique_ids(c, t.values[0], t.table.shape[0], out=t.layouts[0], stream=st)
        for first in range(0, self.D):
            self._ahead(first)
        self.primed = True

    def run(self, s0: int, k: int) -> None:
        """Steps s0 .. s0+k-1; returns as soon as they are enqueued."""
        if not self.primed:
            self.prime()
        step_call = fs.fs_prioritized_step_two_part_multi if self.two_part else fs.fs_prioritized_step_pipelined_multi
        for s in range(s0, s0 + k):
            self._ahead(s + self.D)
            for c, st, rec in zip(self.ctxs, self.streams, self.step_records):
                step_call(c, rec[self._rec(s)], rec[self._rec(s + 1)], stream=st)
            self.stepped = True

    def join(self, check: bool = False) -> None:
        """Every stream of every group has finished (check: and no kernel has raised a device flag)."""
        for c, st in zip(self.ctxs, self.streams):
            if check:
                rc = fs.fs_check_async(c, st)
                if rc != fs.FS_OK:
                    raise fs.FreeScaleError(rc, "fs_check_async", c.last_error())
            else:
                fs.fs_step_join(c, st)
        for st in self.streams:
            st.synchronize()
