"""ctypes binding of libfreescale_hip.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/freescale.h) and does
nothing but turn torch device tensors into pointers, allocate outputs through torch and pass
the current stream.  No step of the method is computed here, and there is no CPU fallback: if
the HIP library is missing, importing succeeds but the first call raises.
"""
from __future__ import annotations

import ctypes
import os
import re
from typing import Dict, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfreescale_hip.so")

FS_F32, FS_BF16 = 0, 1
FS_OK, FS_EINVAL, FS_ENOMEM, FS_EHIP, FS_ENOTIMPL, FS_ERANGE = 0, -1, -2, -3, -4, -5
FS_MAX_DIM = 256
FS_SHORT_SEGMENT = 8
FS_MAX_AHEAD_BATCH = 8
FS_MAX_STEP_TABLES = 16
SHORT_REC_INTS = 12

c_i64, c_i32, c_vp, c_f = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_float


class fs_step_args(ctypes.Structure):
    _fields_ = [
        ("table", c_vp), ("state", c_vp), ("num_rows", c_i64), ("dim", c_i32), ("dtype", c_i32),
        ("lr", c_f), ("eps", c_f),
        ("u_t", c_vp), ("seg_offsets_t", c_vp), ("perm_t", c_vp), ("inverse_t", c_vp), ("n_unique_t_dev", c_vp),
        ("grads_t", c_vp), ("n_t", c_i64),
        ("values_t1", c_vp), ("offsets_t1", c_vp), ("batch_t1", c_i64), ("n_t1", c_i64),
        ("u_t1", c_vp), ("seg_offsets_t1", c_vp), ("perm_t1", c_vp), ("inverse_t1", c_vp), ("n_unique_t1_dev", c_vp),
        ("co", c_vp), ("co_slot", c_vp), ("ex", c_vp), ("ex_slot", c_vp), ("ex_next", c_vp), ("ex_next_slot", c_vp),
        ("counts_dev", c_vp),
        ("cperm", c_vp), ("cslot", c_vp), ("cstart", c_vp), ("class_pos_dev", c_vp), ("short_rec", c_vp),
        ("reduced", c_vp), ("emb_t1", c_vp),
        ("co_flag_t1", c_vp),
        ("sorted_ids_t1", c_vp),
    ]


class FreeScaleError(RuntimeError):
    def __init__(self, code: int, where: str, detail: str = ""):
        super().__init__(f"{where} failed with status {code}" + (f": {detail}" if detail else ""))
        self.code = code


_lib: Optional[ctypes.CDLL] = None


def load_library() -> ctypes.CDLL:
    """Loads the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_24073_amd.build` "
                                "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    S = c_vp  # stream
    sig = {
        "fs_version": (ctypes.c_int, []),
        "fs_ctx_create": (ctypes.c_int, [ctypes.POINTER(c_vp), ctypes.c_int, c_i64, c_i32]),
        "fs_ctx_destroy": (ctypes.c_int, [c_vp]),
        "fs_last_error": (ctypes.c_char_p, [c_vp]),
        "fs_check_async": (ctypes.c_int, [c_vp, S]),
        "fs_ctx_workspace_bytes": (ctypes.c_size_t, [c_vp]),
        "fs_gather_jagged": (ctypes.c_int, [c_vp, c_vp, c_i64, c_i32, ctypes.c_int, c_vp, c_vp, c_i64, c_i64, c_vp, S]),
        "fs_gather_jagged_class": (ctypes.c_int, [c_vp, c_vp, c_i64, c_i32, ctypes.c_int, c_vp, c_vp, c_i64, c_i64, c_vp,
                                                  c_vp, ctypes.c_int, c_vp, S]),
        "fs_unique_ids": (ctypes.c_int, [c_vp, c_vp, c_i64, c_i64, c_vp, c_vp, c_vp, c_vp, c_vp, S]),
        "fs_jagged_keyed_transpose": (ctypes.c_int, [c_vp, c_vp, c_i64, c_i32, c_vp, c_i64, c_i64, c_vp, c_vp, S]),
        "fs_jagged_ranged_dispatch": (ctypes.c_int, [c_vp, c_vp, c_i64, c_i32, c_vp, c_i64, c_i64, c_vp, c_i32, c_vp,
                                                     c_vp, c_vp, S]),
        "fs_jagged_ranged_combine": (ctypes.c_int, [c_vp, c_vp, c_i64, c_i32, c_vp, c_i64, c_i64, c_vp, c_i32, c_vp,
                                                    c_vp, S]),
        "fs_partition_vbs": (ctypes.c_int, [c_vp, c_vp, c_i64, c_vp, c_i64, c_i32, c_vp, c_vp, S]),
        "fs_partition_fbs": (ctypes.c_int, [c_vp, c_vp, c_i64, c_i64, c_i32, c_vp, c_vp, S]),
        "fs_jagged_indexed_permute": (ctypes.c_int, [c_vp, c_vp, c_i64, c_i32, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64,
                                                     c_vp, S]),
        "fs_collision_split": (ctypes.c_int, [c_vp, c_vp, c_vp, c_vp, c_vp, c_i64, c_i64, c_vp, c_vp, c_vp, c_vp,
                                              c_vp, c_vp, c_vp, S]),
        "fs_collision_split_static": (ctypes.c_int, [c_vp, c_vp, c_vp, c_vp, c_i64, c_i64, c_vp, c_vp, c_vp, c_vp,
                                                     c_vp, c_vp, c_vp, S]),
        "fs_split_grads": (ctypes.c_int, [c_vp, c_vp, c_i64, c_i32, c_vp, c_vp, c_vp, c_i64, c_vp, c_vp, c_vp, c_vp, c_vp,
                                          c_vp, S]),
        "fs_class_order_for_parts": (ctypes.c_int, [c_vp, c_vp, c_i64, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, S]),
        "fs_segment_reduce_grads": (ctypes.c_int, [c_vp, c_vp, c_i64, c_i32, c_vp, c_vp, c_vp, c_vp, c_vp, S]),
        "fs_rowwise_adagrad_update": (ctypes.c_int, [c_vp, c_vp, ctypes.c_int, c_vp, c_i64, c_i32, c_vp, c_vp, c_vp,
                                                     c_i64, c_vp, c_f, c_f, S]),
        "fs_collision_split_classes": (ctypes.c_int, [c_vp, c_vp, c_vp, c_vp, c_vp, c_i64, c_i64, c_vp, c_vp, c_vp,
                                                      c_i64, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp,
                                                      c_vp, c_vp, c_vp, S]),
        "fs_reduce_update_class": (ctypes.c_int, [c_vp, ctypes.c_int, c_vp, ctypes.c_int, c_vp, c_i64, c_i32, c_f, c_f,
                                                  c_vp, c_i64, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, S]),
        "fs_unique_ids_ahead": (ctypes.c_int, [c_vp, c_vp, c_i64, c_i64, c_vp, c_vp, c_vp, c_vp, c_vp, S]),
        "fs_prioritized_step": (ctypes.c_int, [c_vp, ctypes.POINTER(fs_step_args), S]),
        "fs_step_forward": (ctypes.c_int, [c_vp, ctypes.POINTER(fs_step_args), S]),
        "fs_step_forward_ahead": (ctypes.c_int, [c_vp, ctypes.POINTER(fs_step_args), S]),
        "fs_step_forward_ahead_batch": (ctypes.c_int, [c_vp, ctypes.POINTER(fs_step_args), ctypes.c_int, S]),
        "fs_prioritized_step_pipelined_multi": (ctypes.c_int, [c_vp, ctypes.POINTER(fs_step_args),
                                                                ctypes.POINTER(fs_step_args), ctypes.c_int, S]),
        "fs_prioritized_step_two_part_multi": (ctypes.c_int, [c_vp, ctypes.POINTER(fs_step_args),
                                                               ctypes.POINTER(fs_step_args), ctypes.c_int, S]),
        "fs_prioritized_step_pipelined": (ctypes.c_int, [c_vp, ctypes.POINTER(fs_step_args),
                                                         ctypes.POINTER(fs_step_args), S]),
        "fs_graph_capture_pipelined": (ctypes.c_int, [c_vp, ctypes.POINTER(fs_step_args), ctypes.POINTER(fs_step_args),
                                                      ctypes.POINTER(c_vp)]),
        "fs_ctx_set_threaded_enqueue": (ctypes.c_int, [c_vp, ctypes.c_int]),
        "fs_step_join": (ctypes.c_int, [c_vp, S]),
        "fs_two_part_forget": (ctypes.c_int, [c_vp]),
        "fs_ctx_host_times": (ctypes.c_int, [c_vp, ctypes.POINTER(ctypes.c_double), ctypes.c_int]),
        "fs_graph_launch": (ctypes.c_int, [c_vp, c_vp, S]),
        "fs_graph_destroy": (ctypes.c_int, [c_vp]),
        "fs_ctx_set_kernel_timing": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.c_int]),
        "fs_ctx_get_kernel_timing": (ctypes.c_int, [c_vp, ctypes.c_int, ctypes.POINTER(c_f), ctypes.c_int,
                                                    ctypes.POINTER(ctypes.c_int)]),
        "fs_init_table_hash": (ctypes.c_int, [c_vp, c_vp, c_i64, c_i32, ctypes.c_int, S]),
        "fs_stream_copy": (ctypes.c_int, [c_vp, c_vp, c_vp, c_i64, S]),
        "fs_stream_row_read": (ctypes.c_int, [c_vp, c_vp, c_i64, c_i32, c_vp, c_i64, c_vp, S]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def declared_symbols(header_paths=None):
    """Names of the functions declared in include/*.h (what a -DFS_TRACE build adds is left out)."""
    if header_paths is None:
        inc = os.path.join(os.path.dirname(_HERE), "include")
        header_paths = sorted(os.path.join(inc, f) for f in os.listdir(inc) if f.endswith(".h"))
    names = set()
    for path in header_paths:
        text = open(path).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        text = re.sub(r"#ifdef FS_TRACE.*?#endif", "", text, flags=re.S)
        names.update(re.findall(r"\b(fs_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        h = stream.cuda_stream
    else:
        h = int(stream)
    return h if h else None


def table_dtype_code(table: torch.Tensor) -> int:
    if table.dtype == torch.float32:
        return FS_F32
    if table.dtype == torch.bfloat16:
        return FS_BF16
    raise TypeError(f"table dtype {table.dtype}: fp32 or bf16 only")


class Context:
    """Owner of an fs_ctx (device workspace, side streams, events)."""

    def __init__(self, max_ids: int, max_dim: int = FS_MAX_DIM, device: Optional[int] = None):
        self.lib = load_library()
        if device is None:
            device = torch.cuda.current_device()
        self.device = device
        h = c_vp()
        rc = self.lib.fs_ctx_create(ctypes.byref(h), device, max_ids, max_dim)
        if rc != FS_OK:
            raise FreeScaleError(rc, "fs_ctx_create")
        self.handle = h
        self.max_ids, self.max_dim = max_ids, max_dim

    def close(self) -> None:
        if getattr(self, "handle", None):
            self.lib.fs_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def last_error(self) -> str:
        return self.lib.fs_last_error(self.handle).decode()

    def check(self, rc: int, where: str) -> None:
        if rc != FS_OK:
            raise FreeScaleError(rc, where, self.last_error())

    def workspace_bytes(self) -> int:
        return int(self.lib.fs_ctx_workspace_bytes(self.handle))


def fs_check_async(ctx: Context, stream=None) -> int:
    return ctx.lib.fs_check_async(ctx.handle, _stream(stream))


FS_TIME_REDUCE, FS_TIME_GATHER, FS_TIME_UPDATE_CO, FS_TIME_UPDATE_EX = 0, 1, 2, 3


def fs_ctx_set_kernel_timing(ctx: Context, slots: int, every: int = 1) -> None:
    ctx.check(ctx.lib.fs_ctx_set_kernel_timing(ctx.handle, slots, every), "fs_ctx_set_kernel_timing")


def fs_ctx_get_kernel_timing(ctx: Context, which: int, max_out: int = 65536):
    buf = (c_f * max_out)()
    n = ctypes.c_int(0)
    ctx.check(ctx.lib.fs_ctx_get_kernel_timing(ctx.handle, which, buf, max_out, ctypes.byref(n)),
              "fs_ctx_get_kernel_timing")
    return [buf[i] for i in range(n.value)]


def fs_gather_jagged(ctx: Context, table: torch.Tensor, values: torch.Tensor, offsets: Optional[torch.Tensor],
                     out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    n = values.numel()
    if out is None:
        out = torch.empty((n, table.shape[1]), dtype=table.dtype, device=table.device)
    batch = 0 if offsets is None else offsets.numel() - 1
    rc = ctx.lib.fs_gather_jagged(ctx.handle, _ptr(table), table.shape[0], table.shape[1], table_dtype_code(table),
                                  _ptr(values), _ptr(offsets), batch, n, _ptr(out), _stream(stream))
    ctx.check(rc, "fs_gather_jagged")
    return out


def fs_gather_jagged_class(ctx: Context, table: torch.Tensor, values: torch.Tensor, offsets: Optional[torch.Tensor],
                           inverse: torch.Tensor, co_flag: torch.Tensor, which: int, out: torch.Tensor,
                           stream=None) -> torch.Tensor:
    n = values.numel()
    batch = 0 if offsets is None else offsets.numel() - 1
    rc = ctx.lib.fs_gather_jagged_class(ctx.handle, _ptr(table), table.shape[0], table.shape[1],
                                        table_dtype_code(table), _ptr(values), _ptr(offsets), batch, n, _ptr(inverse),
                                        _ptr(co_flag), which, _ptr(out), _stream(stream))
    ctx.check(rc, "fs_gather_jagged_class")
    return out


def fs_partition_fbs(ctx: Context, lengths: torch.Tensor, max_len: int, n_ranks: int, stream=None, out=None):
    """(sample_of [B] int32, rank_offsets [n_ranks + 1] int64) of the FBS partitioner; `out`: the caller's pair."""
    B = lengths.numel()
    if out is not None:
        sample_of, rank_offsets = out
    else:
        sample_of = torch.empty(max(B, 1), dtype=torch.int32, device=lengths.device)
        rank_offsets = torch.empty(n_ranks + 1, dtype=torch.int64, device=lengths.device)
    rc = ctx.lib.fs_partition_fbs(ctx.handle, _ptr(lengths), B, max_len, n_ranks, _ptr(sample_of), _ptr(rank_offsets),
                                  _stream(stream))
    ctx.check(rc, "fs_partition_fbs")
    return sample_of[:B], rank_offsets


def fs_partition_vbs(ctx: Context, lengths: torch.Tensor, weight_of_len: torch.Tensor, n_ranks: int, stream=None):
    """(sample_of [B] int32 = the length-sorted order, rank_offsets [n_ranks + 1] int64) of the VBS partitioner;
    weight_of_len [max_len + 1] int64."""
    B = lengths.numel()
    sample_of = torch.empty(max(B, 1), dtype=torch.int32, device=lengths.device)
    rank_offsets = torch.empty(n_ranks + 1, dtype=torch.int64, device=lengths.device)
    rc = ctx.lib.fs_partition_vbs(ctx.handle, _ptr(lengths), B, _ptr(weight_of_len), weight_of_len.numel() - 1, n_ranks,
                                  _ptr(sample_of), _ptr(rank_offsets), _stream(stream))
    ctx.check(rc, "fs_partition_vbs")
    return sample_of[:B], rank_offsets


def fs_jagged_indexed_permute(ctx: Context, values: torch.Tensor, offsets: torch.Tensor, sample_of: torch.Tensor,
                              cap_out: int, stream=None, out=None):
    """(out_values [cap_out, ...], out_offsets [n_out + 1]); values is [n] or [n, width], any 4- or 8-byte dtype.
    `out`: the caller's (out_values, out_offsets)."""
    n_values = values.shape[0]
    elem = _elem_bytes(values)
    n_out = sample_of.numel()
    if out is not None:
        out, out_offsets = out
    else:
        out = torch.empty((cap_out,) + tuple(values.shape[1:]), dtype=values.dtype, device=values.device)
        out_offsets = torch.empty(n_out + 1, dtype=torch.int64, device=values.device)
    rc = ctx.lib.fs_jagged_indexed_permute(ctx.handle, _ptr(values), n_values, elem, _ptr(offsets), offsets.numel() - 1,
                                           _ptr(sample_of), n_out, _ptr(out), cap_out, _ptr(out_offsets),
                                           _stream(stream))
    ctx.check(rc, "fs_jagged_indexed_permute")
    return out, out_offsets


def _elem_bytes(values: torch.Tensor) -> int:
    elem = values.element_size()
    for d in values.shape[1:]:
        elem *= d
    return elem


def fs_jagged_keyed_transpose(ctx: Context, values: torch.Tensor, offsets: torch.Tensor, F: int, B: int, stream=None,
                              out=None):
    out, out_offsets = out if out is not None else (torch.empty_like(values), torch.empty_like(offsets))
    rc = ctx.lib.fs_jagged_keyed_transpose(ctx.handle, _ptr(values), values.shape[0], _elem_bytes(values), _ptr(offsets),
                                           F, B, _ptr(out), _ptr(out_offsets), _stream(stream))
    ctx.check(rc, "fs_jagged_keyed_transpose")
    return out, out_offsets


def fs_jagged_ranged_dispatch(ctx: Context, values: torch.Tensor, offsets: torch.Tensor, F: int, B: int,
                              rank_offsets: torch.Tensor, stream=None, out=None):
    """`out`: the caller's (out_values, out_offsets, splits [n_ranks])."""
    n_ranks = rank_offsets.numel() - 1
    if out is not None:
        out, out_offsets, splits = out
    else:
        out, out_offsets = torch.empty_like(values), torch.empty_like(offsets)
        splits = torch.empty(max(n_ranks, 1), dtype=torch.int64, device=values.device)
    rc = ctx.lib.fs_jagged_ranged_dispatch(ctx.handle, _ptr(values), values.shape[0], _elem_bytes(values), _ptr(offsets),
                                           F, B, _ptr(rank_offsets), n_ranks, _ptr(out), _ptr(out_offsets), _ptr(splits),
                                           _stream(stream))
    ctx.check(rc, "fs_jagged_ranged_dispatch")
    return out, out_offsets, splits[:n_ranks]


def fs_jagged_ranged_combine(ctx: Context, values: torch.Tensor, offsets: torch.Tensor, F: int, B: int,
                             rank_offsets: torch.Tensor, stream=None, out=None):
    out, out_offsets = out if out is not None else (torch.empty_like(values), torch.empty_like(offsets))
    rc = ctx.lib.fs_jagged_ranged_combine(ctx.handle, _ptr(values), values.shape[0], _elem_bytes(values), _ptr(offsets),
                                          F, B, _ptr(rank_offsets), rank_offsets.numel() - 1, _ptr(out),
                                          _ptr(out_offsets), _stream(stream))
    ctx.check(rc, "fs_jagged_ranged_combine")
    return out, out_offsets


def fs_unique_ids(ctx: Context, ids: torch.Tensor, num_rows: int, out: Optional[Dict[str, torch.Tensor]] = None,
                  stream=None) -> Dict[str, torch.Tensor]:
    n = ids.numel()
    dev = ids.device
    if out is None:
        out = {
            "unique": torch.empty(max(n, 1), dtype=torch.int64, device=dev),
            "seg_offsets": torch.empty(n + 1, dtype=torch.int32, device=dev),
            "perm": torch.empty(max(n, 1), dtype=torch.int32, device=dev),
            "inverse": torch.empty(max(n, 1), dtype=torch.int32, device=dev),
            "n_unique": torch.zeros(1, dtype=torch.int64, device=dev),
        }
    rc = ctx.lib.fs_unique_ids(ctx.handle, _ptr(ids), n, num_rows, _ptr(out["unique"]), _ptr(out["seg_offsets"]),
                               _ptr(out["perm"]), _ptr(out.get("inverse")), _ptr(out["n_unique"]), _stream(stream))
    ctx.check(rc, "fs_unique_ids")
    out["n"] = n
    return out


def fs_collision_split(ctx: Context, u_t: Optional[torch.Tensor], n_t_dev: Optional[torch.Tensor],
                       u_t1: Optional[torch.Tensor], n_t1_dev: Optional[torch.Tensor], cap_t: int, cap_t1: int,
                       out: Optional[Dict[str, torch.Tensor]] = None, stream=None) -> Dict[str, torch.Tensor]:
    dev = (u_t if u_t is not None else u_t1).device if (u_t is not None or u_t1 is not None) else torch.device("cuda")
    if out is None:
        i64 = lambda k: torch.empty(max(k, 1), dtype=torch.int64, device=dev)
        i32 = lambda k: torch.empty(max(k, 1), dtype=torch.int32, device=dev)
        out = {"co": i64(cap_t), "co_slot": i32(cap_t), "ex": i64(cap_t), "ex_slot": i32(cap_t),
               "ex_next": i64(cap_t1), "ex_next_slot": i32(cap_t1),
               "counts": torch.zeros(3, dtype=torch.int64, device=dev)}
    rc = ctx.lib.fs_collision_split(ctx.handle, _ptr(u_t), _ptr(n_t_dev), _ptr(u_t1), _ptr(n_t1_dev), cap_t, cap_t1,
                                    _ptr(out["co"]), _ptr(out["co_slot"]), _ptr(out["ex"]), _ptr(out["ex_slot"]),
                                    _ptr(out["ex_next"]), _ptr(out["ex_next_slot"]), _ptr(out["counts"]),
                                    _stream(stream))
    ctx.check(rc, "fs_collision_split")
    return out


FS_STATIC_SPLIT_MAX_ROWS = 1 << 20


def fs_collision_split_static(u_t: Optional[torch.Tensor], n_t_dev: Optional[torch.Tensor],
                              u_t1: Optional[torch.Tensor], n_t1_dev: Optional[torch.Tensor], cap_t: int, cap_t1: int,
                              out: Dict[str, torch.Tensor], stream=None) -> Dict[str, torch.Tensor]:
    """The split without a context and without any allocation: `out` (a bundle as fs_collision_split returns
    it) is the caller's."""
    lib = load_library()
    rc = lib.fs_collision_split_static(_ptr(u_t), _ptr(n_t_dev), _ptr(u_t1), _ptr(n_t1_dev), cap_t, cap_t1,
                                       _ptr(out["co"]), _ptr(out["co_slot"]), _ptr(out["ex"]), _ptr(out["ex_slot"]),
                                       _ptr(out["ex_next"]), _ptr(out["ex_next_slot"]), _ptr(out["counts"]),
                                       _stream(stream))
    if rc != FS_OK:
        raise FreeScaleError(rc, "fs_collision_split_static", lib.fs_last_error(None).decode())
    return out


def fs_collision_split_classes(ctx: Context, layout_t: Dict[str, torch.Tensor], u_t1: Optional[torch.Tensor],
                               n_t1_dev: Optional[torch.Tensor], cap_t1: int,
                               out: Optional[Dict[str, torch.Tensor]] = None, stream=None) -> Dict[str, torch.Tensor]:
    """layout_t: what fs_unique_ids returned for batch t (with its "n")."""
    n_t = layout_t["n"]
    dev = layout_t["unique"].device
    if out is None:
        out = alloc_split(n_t, cap_t1, dev)
    rc = ctx.lib.fs_collision_split_classes(
        ctx.handle, _ptr(layout_t["unique"]), _ptr(layout_t["n_unique"]), _ptr(u_t1), _ptr(n_t1_dev), n_t, cap_t1,
        _ptr(layout_t["seg_offsets"]), _ptr(layout_t["perm"]), _ptr(layout_t.get("inverse")), n_t,
        _ptr(out["co"]), _ptr(out["co_slot"]), _ptr(out["ex"]), _ptr(out["ex_slot"]), _ptr(out["ex_next"]),
        _ptr(out["ex_next_slot"]), _ptr(out["counts"]), _ptr(out["cperm"]), _ptr(out["cslot"]), _ptr(out["cstart"]),
        _ptr(out["class_pos"]), _ptr(out["short_rec"]), _stream(stream))
    ctx.check(rc, "fs_collision_split_classes")
    return out


def fs_split_grads(ctx: Context, grads: torch.Tensor, layout_t: Dict[str, torch.Tensor], split: Dict[str, torch.Tensor],
                   out: Optional[Dict[str, torch.Tensor]] = None, stream=None) -> Dict[str, torch.Tensor]:
    """split() of Algorithm 2's Backward.  layout_t: the batch's layout with its inverse map; split: its collision
    split (co_slot, counts).  Returns co_index, g_co, ex_index, g_ex, part_pos, counts ([2] occurrences per part)."""
    n, dim = grads.shape
    dev = grads.device
    if out is None:
        i32 = lambda: torch.empty(max(n, 1), dtype=torch.int32, device=dev)
        f32 = lambda: torch.empty((max(n, 1), dim), dtype=torch.float32, device=dev)
        out = {"co_index": i32(), "g_co": f32(), "ex_index": i32(), "g_ex": f32(), "part_pos": i32(),
               "counts": torch.zeros(2, dtype=torch.int64, device=dev)}
    rc = ctx.lib.fs_split_grads(ctx.handle, _ptr(grads), n, dim, _ptr(layout_t.get("inverse")), _ptr(split["co_slot"]),
                                _ptr(split["counts"]), n, _ptr(out["co_index"]), _ptr(out["g_co"]),
                                _ptr(out["ex_index"]), _ptr(out["g_ex"]), _ptr(out["part_pos"]), _ptr(out["counts"]),
                                _stream(stream))
    ctx.check(rc, "fs_split_grads")
    return out


def fs_class_order_for_parts(ctx: Context, parts: Dict[str, torch.Tensor], n_t: int, split: Dict[str, torch.Tensor],
                             stream=None) -> Dict[str, torch.Tensor]:
    """A copy of `split` whose class order and records address the packed parts of fs_split_grads."""
    out = dict(split)
    out["cperm"] = torch.empty_like(split["cperm"])
    out["short_rec"] = torch.empty_like(split["short_rec"])
    rc = ctx.lib.fs_class_order_for_parts(ctx.handle, _ptr(parts["part_pos"]), n_t, _ptr(split["cperm"]),
                                          _ptr(split["class_pos"]), _ptr(split["short_rec"]), _ptr(split["counts"]),
                                          _ptr(out["cperm"]), _ptr(out["short_rec"]), _stream(stream))
    ctx.check(rc, "fs_class_order_for_parts")
    return out


def fs_reduce_update_class(ctx: Context, cls: int, table: torch.Tensor, state: torch.Tensor, lr: float, eps: float,
                           grads: torch.Tensor, layout_t: Dict[str, torch.Tensor], split: Dict[str, torch.Tensor],
                           reduced: Optional[torch.Tensor] = None, stream=None) -> None:
    n, dim = grads.shape
    rc = ctx.lib.fs_reduce_update_class(
        ctx.handle, cls, _ptr(table), table_dtype_code(table), _ptr(state), table.shape[0], dim, lr, eps,
        _ptr(grads), n, _ptr(layout_t["unique"]), _ptr(layout_t["seg_offsets"]),
        split["short_rec"].data_ptr() + cls * 4 * SHORT_REC_INTS * n,
        split["counts"].data_ptr() + 8 * cls, _ptr(split["cperm"]),
        _ptr(split["cslot"]), _ptr(split["cstart"]), _ptr(split["class_pos"]), _ptr(reduced), _stream(stream))
    ctx.check(rc, "fs_reduce_update_class")


FS_STREAM_LAST_STEP = "last_step"


def fs_unique_ids_ahead(ctx: Context, ids: torch.Tensor, num_rows: int, out: Dict[str, torch.Tensor],
                        stream=None) -> Dict[str, torch.Tensor]:
    n = ids.numel()
    stream_arg = ctypes.c_void_p(-1) if stream == FS_STREAM_LAST_STEP else _stream(stream)
    rc = ctx.lib.fs_unique_ids_ahead(ctx.handle, _ptr(ids), n, num_rows, _ptr(out["unique"]),
                                     _ptr(out["seg_offsets"]), _ptr(out["perm"]), _ptr(out.get("inverse")),
                                     _ptr(out["n_unique"]), stream_arg)
    ctx.check(rc, "fs_unique_ids_ahead")
    out["n"] = n
    return out


def fs_segment_reduce_grads(ctx: Context, grads: torch.Tensor, perm: torch.Tensor, seg_offsets: torch.Tensor,
                            n_unique_dev: torch.Tensor, out: Optional[torch.Tensor] = None, stream=None,
                            inverse: Optional[torch.Tensor] = None) -> torch.Tensor:
    n, dim = grads.shape
    if out is None:
        out = torch.empty((max(n, 1), dim), dtype=torch.float32, device=grads.device)
    rc = ctx.lib.fs_segment_reduce_grads(ctx.handle, _ptr(grads), n, dim, _ptr(perm), _ptr(seg_offsets),
                                         _ptr(inverse), _ptr(n_unique_dev), _ptr(out), _stream(stream))
    ctx.check(rc, "fs_segment_reduce_grads")
    return out


def fs_rowwise_adagrad_update(ctx: Context, table: torch.Tensor, state: torch.Tensor, rows: torch.Tensor,
                              slots: torch.Tensor, n_rows_dev: torch.Tensor, cap: int, reduced: torch.Tensor,
                              lr: float, eps: float, stream=None) -> None:
    rc = ctx.lib.fs_rowwise_adagrad_update(ctx.handle, _ptr(table), table_dtype_code(table), _ptr(state),
                                           table.shape[0], table.shape[1], _ptr(rows), _ptr(slots), _ptr(n_rows_dev),
                                           cap, _ptr(reduced), lr, eps, _stream(stream))
    ctx.check(rc, "fs_rowwise_adagrad_update")


def fs_prioritized_step(ctx: Context, args: fs_step_args, stream=None) -> None:
    rc = ctx.lib.fs_prioritized_step(ctx.handle, ctypes.byref(args), _stream(stream))
    ctx.check(rc, "fs_prioritized_step")


def fs_step_forward(ctx: Context, args: fs_step_args, stream=None) -> None:
    rc = ctx.lib.fs_step_forward(ctx.handle, ctypes.byref(args), _stream(stream))
    ctx.check(rc, "fs_step_forward")


def fs_step_forward_ahead(ctx: Context, args: fs_step_args, stream=None) -> None:
    stream_arg = ctypes.c_void_p(-1) if stream == FS_STREAM_LAST_STEP else _stream(stream)
    rc = ctx.lib.fs_step_forward_ahead(ctx.handle, ctypes.byref(args), stream_arg)
    ctx.check(rc, "fs_step_forward_ahead")


def fs_step_forward_ahead_batch(ctx: Context, args, stream=None) -> None:
    """args: sequence of 1..FS_MAX_AHEAD_BATCH argument records (copied into one contiguous array), or such an
    array from step_args_array (passed as it is)."""
    arr = args if isinstance(args, ctypes.Array) else (fs_step_args * len(args))(*args)
    stream_arg = ctypes.c_void_p(-1) if stream == FS_STREAM_LAST_STEP else _stream(stream)
    rc = ctx.lib.fs_step_forward_ahead_batch(ctx.handle, arr, len(args), stream_arg)
    ctx.check(rc, "fs_step_forward_ahead_batch")


def fs_prioritized_step_pipelined(ctx: Context, cur: fs_step_args, nxt: Optional[fs_step_args], stream=None) -> None:
    rc = ctx.lib.fs_prioritized_step_pipelined(ctx.handle, ctypes.byref(cur),
                                               ctypes.byref(nxt) if nxt is not None else None, _stream(stream))
    ctx.check(rc, "fs_prioritized_step_pipelined")


def step_args_array(records):
    """Contiguous copy of a sequence of argument records (for the calls that take several)."""
    return (fs_step_args * len(records))(*records)


def fs_prioritized_step_pipelined_multi(ctx: Context, cur, nxt, stream=None) -> None:
    """cur / nxt: fs_step_args arrays from step_args_array (nxt may be None), one record per table."""
    rc = ctx.lib.fs_prioritized_step_pipelined_multi(ctx.handle, cur, nxt, len(cur), _stream(stream))
    ctx.check(rc, "fs_prioritized_step_pipelined_multi")


def fs_prioritized_step_two_part_multi(ctx: Context, cur, nxt, stream=None) -> None:
    """As fs_prioritized_step_pipelined_multi, the lookup taken in its two parts (records need co_flag_t1)."""
    rc = ctx.lib.fs_prioritized_step_two_part_multi(ctx.handle, cur, nxt, len(cur), _stream(stream))
    ctx.check(rc, "fs_prioritized_step_two_part_multi")


def fs_two_part_forget(ctx: Context) -> None:
    ctx.check(ctx.lib.fs_two_part_forget(ctx.handle), "fs_two_part_forget")


def fs_ctx_host_times(ctx: Context, reset: bool = False):
    buf = (ctypes.c_double * 7)()
    ctx.check(ctx.lib.fs_ctx_host_times(ctx.handle, buf, 1 if reset else 0), "fs_ctx_host_times")
    return [buf[i] for i in range(7)]


def fs_step_join(ctx: Context, stream=None) -> None:
    ctx.check(ctx.lib.fs_step_join(ctx.handle, _stream(stream)), "fs_step_join")


def fs_graph_capture_pipelined(ctx: Context, cur: fs_step_args, nxt: Optional[fs_step_args]) -> c_vp:
    g = c_vp()
    rc = ctx.lib.fs_graph_capture_pipelined(ctx.handle, ctypes.byref(cur),
                                            ctypes.byref(nxt) if nxt is not None else None, ctypes.byref(g))
    ctx.check(rc, "fs_graph_capture_pipelined")
    return g


def fs_graph_launch(ctx: Context, graph: c_vp, stream=None) -> None:
    ctx.check(ctx.lib.fs_graph_launch(ctx.handle, graph, _stream(stream)), "fs_graph_launch")


def fs_graph_destroy(ctx: Context, graph: c_vp) -> None:
    ctx.lib.fs_graph_destroy(graph)


def fs_init_table_hash(ctx: Context, table: torch.Tensor, stream=None) -> None:
    rc = ctx.lib.fs_init_table_hash(ctx.handle, _ptr(table), table.shape[0], table.shape[1], table_dtype_code(table),
                                    _stream(stream))
    ctx.check(rc, "fs_init_table_hash")


def fs_stream_copy(ctx: Context, src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    rc = ctx.lib.fs_stream_copy(ctx.handle, _ptr(src), _ptr(dst), nbytes, _stream(stream))
    ctx.check(rc, "fs_stream_copy")


def fs_stream_row_read(ctx: Context, rows: torch.Tensor, index: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """rows [num_rows, width] of any dtype with width * itemsize a multiple of 16; index int64; sink [1024] int32."""
    row_bytes = rows.shape[1] * rows.element_size()
    rc = ctx.lib.fs_stream_row_read(ctx.handle, _ptr(rows), rows.shape[0], row_bytes, _ptr(index), index.numel(),
                                    _ptr(sink), _stream(stream))
    ctx.check(rc, "fs_stream_row_read")


# ---- buffer bundles for the whole-iteration call (allocation only) -----------------------------
def alloc_layout(n: int, device, inverse: bool = True, sorted_ids: bool = False) -> Dict[str, torch.Tensor]:
    """inverse=False: no inverse map (the step calls do not need it; the two-part lookup does).
    sorted_ids=True: room for the ascending list of all IDs (the row-ordered lookup of the step calls reads it)."""
    out = {
        "unique": torch.empty(max(n, 1), dtype=torch.int64, device=device),
        "seg_offsets": torch.empty(n + 1, dtype=torch.int32, device=device),
        "perm": torch.empty(max(n, 1), dtype=torch.int32, device=device),
        "n_unique": torch.zeros(1, dtype=torch.int64, device=device),
        "n": n,
    }
    if inverse:
        out["inverse"] = torch.empty(max(n, 1), dtype=torch.int32, device=device)
    if sorted_ids:
        out["sorted_ids"] = torch.empty(max(n, 1), dtype=torch.int64, device=device)
    return out


def alloc_split(cap_t: int, cap_t1: int, device) -> Dict[str, torch.Tensor]:
    i64 = lambda k: torch.empty(max(k, 1), dtype=torch.int64, device=device)
    i32 = lambda k: torch.empty(max(k, 1), dtype=torch.int32, device=device)
    return {"co": i64(cap_t), "co_slot": i32(cap_t), "ex": i64(cap_t), "ex_slot": i32(cap_t),
            "ex_next": i64(cap_t1), "ex_next_slot": i32(cap_t1),
            "counts": torch.zeros(3, dtype=torch.int64, device=device),
            "cperm": i32(cap_t), "cslot": i32(cap_t), "cstart": i32(cap_t),
            "short_rec": i32(2 * SHORT_REC_INTS * cap_t),
            "co_flag_t1": torch.empty(max(cap_t1, 1), dtype=torch.uint8, device=device),
            "class_pos": torch.zeros(2, dtype=torch.int32, device=device)}


def make_step_args(table: torch.Tensor, state: torch.Tensor, lr: float, eps: float,
                   layout_t: Dict[str, torch.Tensor], grads_t: Optional[torch.Tensor],
                   values_t1: Optional[torch.Tensor], offsets_t1: Optional[torch.Tensor],
                   layout_t1: Optional[Dict[str, torch.Tensor]], split: Dict[str, torch.Tensor],
                   reduced: Optional[torch.Tensor], emb_t1: Optional[torch.Tensor]) -> fs_step_args:
    """Fills the argument record of fs_prioritized_step from tensors (pointers only)."""
    a = fs_step_args()
    a.table, a.state = _ptr(table), _ptr(state)
    a.num_rows, a.dim, a.dtype = table.shape[0], table.shape[1], table_dtype_code(table)
    a.lr, a.eps = lr, eps
    a.u_t, a.seg_offsets_t, a.perm_t = _ptr(layout_t["unique"]), _ptr(layout_t["seg_offsets"]), _ptr(layout_t["perm"])
    a.inverse_t = _ptr(layout_t.get("inverse"))
    a.n_unique_t_dev = _ptr(layout_t["n_unique"])
    a.grads_t = _ptr(grads_t)
    a.n_t = layout_t["n"]
    if values_t1 is not None:
        a.values_t1, a.offsets_t1 = _ptr(values_t1), _ptr(offsets_t1)
        a.batch_t1 = 0 if offsets_t1 is None else offsets_t1.numel() - 1
        a.n_t1 = values_t1.numel()
        a.u_t1, a.seg_offsets_t1 = _ptr(layout_t1["unique"]), _ptr(layout_t1["seg_offsets"])
        a.perm_t1, a.inverse_t1 = _ptr(layout_t1["perm"]), _ptr(layout_t1.get("inverse"))
        a.n_unique_t1_dev = _ptr(layout_t1["n_unique"])
        a.sorted_ids_t1 = _ptr(layout_t1.get("sorted_ids"))
        a.emb_t1 = _ptr(emb_t1)
    else:
        a.n_t1, a.batch_t1 = 0, 0
    a.co, a.co_slot, a.ex, a.ex_slot = _ptr(split["co"]), _ptr(split["co_slot"]), _ptr(split["ex"]), _ptr(split["ex_slot"])
    a.ex_next, a.ex_next_slot = _ptr(split["ex_next"]), _ptr(split["ex_next_slot"])
    a.counts_dev = _ptr(split["counts"])
    a.cperm, a.cslot, a.cstart = _ptr(split["cperm"]), _ptr(split["cslot"]), _ptr(split["cstart"])
    a.class_pos_dev = _ptr(split["class_pos"])
    a.short_rec = _ptr(split["short_rec"])
    a.co_flag_t1 = _ptr(split.get("co_flag_t1"))
    a.reduced = _ptr(reduced)
    return a
