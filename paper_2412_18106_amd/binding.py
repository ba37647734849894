"""ctypes binding of libxyattn.so: same names as the C ABI, argument marshalling only.

Nothing is computed here.  Tensors handed to ``xy_attn_run`` are torch tensors
on the GPU (torch is used for device memory and streams only); their data
pointers and element strides are passed straight through.  If the shared
library has not been built this module raises at import: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import itertools
import os

import numpy as np
import torch  # noqa: F401  (first: the library must bind to the HIP runtime torch has already loaded)

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libxyattn.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(
        f"{_LIB_PATH} is missing: build it first (python -m paper_2412_18106_amd.build); "
        "there is no CPU fallback")
from . import build as _build  # noqa: E402  (no compiler is run here: only the digest of the sources is compared)

if not _build.is_current():
    raise ImportError(
        f"{_LIB_PATH} was not built from the sources in this tree (csrc/, include/ or the build script changed "
        "since): build it again (python -m paper_2412_18106_amd.build); a stale library is never loaded")
_lib = C.CDLL(_LIB_PATH)

XY_OK, XY_ERR_ARG, XY_ERR_DESC, XY_ERR_CAPACITY, XY_ERR_WORKSPACE, XY_ERR_HIP, XY_ERR_NOMEM = 0, -1, -2, -3, -4, -5, -6
XY_PREFILL, XY_DECODE, XY_VERIFY = 0, 1, 2
XY_MASK_CAUSAL, XY_MASK_TREE = 0, 1
XY_PHASE_UNITS, XY_PHASE_MERGE = 1, 2
XY_ASSIGN_SNAKE, XY_ASSIGN_LEAST_LOADED, XY_ASSIGN_DYNAMIC = 0, 1, 2
XY_SPLIT_AUTO = -1
XY_TILE_AUTO = -1


class xy_seq_desc(C.Structure):
    _fields_ = [("query_len", C.c_int32), ("context_len", C.c_int32), ("kind", C.c_int32),
                ("mask_kind", C.c_int32), ("mask_word_offset", C.c_int64)]


class xy_attn_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "num_q_heads", "num_kv_heads", "head_dim", "block_size", "max_blocks_per_seq", "num_workers",
        "prefill_tile_tokens", "prefill_heads_per_unit", "verify_tile_tokens", "split_kv_blocks",
        "cost_row_floor", "assign_policy")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class xy_work_unit(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "seq", "head_begin", "head_count", "q_begin", "q_count", "kv_block_begin", "kv_block_end",
        "split_index", "num_splits", "kind_flags")] + [("cost", C.c_int64), ("ws_offset", C.c_int64)]


class xy_merge_item(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("seq", "head_begin", "head_count", "q_begin", "q_count",
                                           "num_splits")] + [("ws_offset", C.c_int64)]


class xy_kv_copy(C.Structure):
    _fields_ = [("src_block", C.c_int32), ("dst_block", C.c_int32), ("rows", C.c_int32)]


class xy_queue_entry(C.Structure):
    _fields_ = [("request", C.c_int32), ("kind", C.c_int32), ("tokens", C.c_int32), ("context_len", C.c_int32)]


class xy_chunk_entry(C.Structure):
    _fields_ = [("request", C.c_int32), ("kind", C.c_int32), ("query_len", C.c_int32), ("context_len", C.c_int32)]


_plan_p = C.c_void_p
_lib.xy_attn_default_config.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(xy_attn_config)]
_lib.xy_attn_plan_create.argtypes = [C.POINTER(xy_attn_config), C.c_void_p, C.c_int32, C.POINTER(_plan_p)]
_lib.xy_attn_plan_get.argtypes = [_plan_p, C.POINTER(C.POINTER(xy_work_unit)), C.POINTER(C.c_int64),
                                  C.POINTER(C.POINTER(C.c_int32)), C.POINTER(C.POINTER(xy_merge_item)),
                                  C.POINTER(C.c_int64)]
_lib.xy_attn_plan_workspace_bytes.argtypes = [_plan_p, C.POINTER(C.c_size_t)]
_lib.xy_attn_plan_upload.argtypes = [_plan_p]
_lib.xy_attn_plan_upload_async.argtypes = [_plan_p, C.c_void_p]
_lib.xy_attn_plan_rebuild.argtypes = [_plan_p, C.POINTER(xy_attn_config), C.c_void_p, C.c_int32]
_lib.xy_attn_run.argtypes = [_plan_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                             C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                             C.c_int64, C.c_int64, C.c_void_p, C.c_size_t, C.c_float, C.c_void_p]
_lib.xy_attn_run_phase.argtypes = [C.c_int] + list(_lib.xy_attn_run.argtypes)
_lib.xy_attn_run_static.argtypes = list(_lib.xy_attn_run.argtypes[:14]) + [C.c_float, C.c_void_p]
_lib.xy_attn_append_kv.argtypes = [_plan_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                   C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]
_lib.xy_attn_run_fused_qkv.argtypes = list(_lib.xy_attn_run.argtypes)
_lib.xy_attn_copy_block_rows.argtypes = [C.POINTER(xy_kv_copy), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                         C.c_int64, C.c_int64, C.c_int64, C.c_void_p]
_lib.xy_serve_schedule_chunk.argtypes = [C.c_int32, C.c_int32, C.POINTER(xy_queue_entry), C.c_int32,
                                         C.POINTER(xy_chunk_entry), C.POINTER(C.c_int32)]
_lib.xy_kv_create.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
_lib.xy_kv_destroy.argtypes = [C.c_void_p]
_lib.xy_kv_destroy.restype = None
_lib.xy_kv_open.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                            C.POINTER(xy_kv_copy), C.POINTER(C.c_int32)]
_lib.xy_kv_extend.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_int32]
_lib.xy_kv_block_row.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32),
                                 C.POINTER(C.c_int32)]
_lib.xy_kv_close.argtypes = [C.c_void_p, C.c_int32]
_lib.xy_kv_stats.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
_lib.xy_probe_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
_lib.xy_probe_stream_read_once.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
_lib.xy_probe_mfma.argtypes = [C.c_int32, C.c_void_p, C.c_void_p]
_lib.xy_probe_issue_mix.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.xy_attn_plan_destroy.argtypes = [_plan_p]
_lib.xy_attn_plan_destroy.restype = None
_lib.xy_attn_strerror.argtypes = [C.c_int]
_lib.xy_attn_strerror.restype = C.c_char_p
for _f in ("xy_attn_default_config", "xy_attn_plan_create", "xy_attn_plan_rebuild", "xy_attn_plan_get",
           "xy_attn_plan_workspace_bytes", "xy_attn_plan_upload", "xy_attn_plan_upload_async", "xy_attn_run", "xy_attn_run_phase",
           "xy_attn_run_static", "xy_attn_append_kv", "xy_attn_run_fused_qkv", "xy_probe_stream_read", "xy_probe_stream_read_once",
           "xy_probe_mfma", "xy_probe_issue_mix", "xy_attn_copy_block_rows", "xy_serve_schedule_chunk", "xy_kv_create", "xy_kv_open",
           "xy_kv_extend", "xy_kv_block_row", "xy_kv_close", "xy_kv_stats"):
    getattr(_lib, _f).restype = C.c_int

EXPORTED = ("xy_attn_default_config", "xy_attn_plan_create", "xy_attn_plan_rebuild", "xy_attn_plan_get",
            "xy_attn_plan_workspace_bytes", "xy_attn_plan_upload", "xy_attn_plan_upload_async", "xy_attn_run", "xy_attn_run_phase",
            "xy_attn_run_static", "xy_attn_append_kv", "xy_attn_run_fused_qkv", "xy_attn_copy_block_rows",
            "xy_attn_plan_destroy", "xy_attn_strerror")
EXPORTED_PROBE = ("xy_probe_stream_read", "xy_probe_stream_read_once", "xy_probe_mfma", "xy_probe_issue_mix")
EXPORTED_SERVE = ("xy_serve_schedule_chunk", "xy_kv_create", "xy_kv_destroy", "xy_kv_open", "xy_kv_extend",
                  "xy_kv_block_row", "xy_kv_close", "xy_kv_stats")


class XyError(RuntimeError):
    def __init__(self, status):
        self.status = int(status)
        super().__init__(f"xy_attn status {status}: {xy_attn_strerror(status)}")


def _check(status):
    if status != XY_OK:
        raise XyError(status)


def xy_attn_strerror(status):
    return _lib.xy_attn_strerror(int(status)).decode()


def xy_attn_default_config(num_q_heads, num_kv_heads, max_blocks_per_seq, **overrides):
    cfg = xy_attn_config()
    _check(_lib.xy_attn_default_config(num_q_heads, num_kv_heads, max_blocks_per_seq, C.byref(cfg)))
    for k, v in overrides.items():
        if not hasattr(cfg, k):
            raise AttributeError(k)
        setattr(cfg, k, int(v))
    return cfg


_DESC_DTYPE = np.dtype([("query_len", np.int32), ("context_len", np.int32), ("kind", np.int32),
                        ("mask_kind", np.int32), ("mask_word_offset", np.int64)])
assert _DESC_DTYPE.itemsize == C.sizeof(xy_seq_desc)


def make_descs(seqs):
    """[(query_len, context_len, kind, mask_kind, mask_word_offset)] -> array of xy_seq_desc records (numpy, C layout)."""
    if isinstance(seqs, np.ndarray) and seqs.dtype == _DESC_DTYPE:
        return np.ascontiguousarray(seqs)
    n = len(seqs)
    arr = np.zeros(max(1, n), dtype=_DESC_DTYPE)
    if n:
        if any(len(s) != 5 for s in seqs):
            raise ValueError("a sequence descriptor has five fields")
        flat = np.fromiter(itertools.chain.from_iterable(seqs), dtype=np.int64, count=5 * n).reshape(n, 5)
        arr.view(np.int32).reshape(-1, 6)[:n, :4] = flat[:, :4]
        arr["mask_word_offset"][:n] = flat[:, 4]
    return arr


def xy_attn_plan_create(cfg, seqs):
    """Returns an opaque plan handle (ctypes void pointer); free it with xy_attn_plan_destroy."""
    plan = _plan_p()
    descs = make_descs(seqs)
    _check(_lib.xy_attn_plan_create(C.byref(cfg), descs.ctypes.data, len(seqs), C.byref(plan)))
    return plan


def xy_attn_plan_rebuild(plan, cfg, seqs):
    """Plan the next batch in an existing plan object (keeps its host buffers and its memory on the GPU)."""
    descs = make_descs(seqs)
    _check(_lib.xy_attn_plan_rebuild(plan, C.byref(cfg), descs.ctypes.data, len(seqs)))


def xy_attn_plan_get(plan):
    """(units, worker_offsets, merges) as numpy arrays copied out of the plan."""
    up, n = C.POINTER(xy_work_unit)(), C.c_int64()
    op = C.POINTER(C.c_int32)()
    mp, nm = C.POINTER(xy_merge_item)(), C.c_int64()
    _check(_lib.xy_attn_plan_get(plan, C.byref(up), C.byref(n), C.byref(op), C.byref(mp), C.byref(nm)))
    unit_dt = np.dtype(xy_work_unit)
    merge_dt = np.dtype(xy_merge_item)
    units = np.zeros(n.value, dtype=unit_dt)
    if n.value:
        C.memmove(units.ctypes.data, up, n.value * C.sizeof(xy_work_unit))
    merges = np.zeros(nm.value, dtype=merge_dt)
    if nm.value:
        C.memmove(merges.ctypes.data, mp, nm.value * C.sizeof(xy_merge_item))
    # worker count is not returned by the C call; offsets end where the last entry equals num_units
    return units, op, merges


def plan_arrays(plan, num_workers):
    units, op, merges = xy_attn_plan_get(plan)
    offsets = np.ctypeslib.as_array(op, shape=(num_workers + 1,)).copy()
    return units, offsets, merges


def xy_attn_plan_workspace_bytes(plan):
    b = C.c_size_t()
    _check(_lib.xy_attn_plan_workspace_bytes(plan, C.byref(b)))
    return int(b.value)


def xy_attn_plan_upload(plan):
    _check(_lib.xy_attn_plan_upload(plan))


def xy_attn_plan_upload_async(plan, stream=None):
    """One asynchronous copy of the plan's tables on the stream (default: the current one)."""
    s = torch.cuda.current_stream() if stream is None else stream
    _check(_lib.xy_attn_plan_upload_async(plan, C.c_void_p(s.cuda_stream)))


def xy_attn_plan_destroy(plan):
    _lib.xy_attn_plan_destroy(plan)


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _run_args(plan, q, k_cache, v_cache, block_table, tree_masks, out, workspace, softmax_scale, stream):
    assert q.stride(-1) == 1 and out.stride(-1) == 1 and k_cache.stride(-1) == 1 and v_cache.stride(-1) == 1
    assert k_cache.stride() == v_cache.stride() and block_table.is_contiguous()
    s = torch.cuda.current_stream() if stream is None else stream
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return (plan, _ptr(q), q.stride(0), q.stride(1), _ptr(k_cache), _ptr(v_cache),
            k_cache.stride(0), k_cache.stride(1), k_cache.stride(2), _ptr(block_table),
            _ptr(tree_masks), _ptr(out), out.stride(0), out.stride(1), _ptr(workspace),
            ws_bytes, float(softmax_scale), C.c_void_p(s.cuda_stream))


def xy_attn_run(plan, q, k_cache, v_cache, block_table, tree_masks, out, workspace, softmax_scale,
                stream=None):
    """q, out: [tokens, Hq, D] bf16; k_cache, v_cache: [blocks, Hkv, B, D] bf16 (any strides with D
    contiguous); block_table int32 [num_seqs, max_blocks] contiguous; tree_masks int32/uint32 words or
    None; workspace: any tensor of at least xy_attn_plan_workspace_bytes bytes or None.  stream: a
    torch.cuda.Stream (defaults to the current one).  Asynchronous."""
    _check(_lib.xy_attn_run(*_run_args(plan, q, k_cache, v_cache, block_table, tree_masks, out, workspace,
                                       softmax_scale, stream)))


XY_STATIC_WORKSPACE_BYTES = 64 * 1024 * 1024


def xy_attn_run_static(plan, q, k_cache, v_cache, block_table, tree_masks, out, softmax_scale, stream=None):
    """xy_attn_run without a workspace: K/V-split partial results go to the library's fixed device array
    (at most XY_STATIC_WORKSPACE_BYTES; the plan must have been uploaded).  Allocates nothing."""
    a = _run_args(plan, q, k_cache, v_cache, block_table, tree_masks, out, None, softmax_scale, stream)
    _check(_lib.xy_attn_run_static(*a[:14], a[16], a[17]))


def xy_attn_run_phase(phases, plan, q, k_cache, v_cache, block_table, tree_masks, out, workspace,
                      softmax_scale, stream=None):
    """One or both of the launches of xy_attn_run (XY_PHASE_UNITS | XY_PHASE_MERGE)."""
    _check(_lib.xy_attn_run_phase(int(phases), *_run_args(plan, q, k_cache, v_cache, block_table, tree_masks,
                                                          out, workspace, softmax_scale, stream)))


def xy_attn_append_kv(plan, k_new, v_new, k_cache, v_cache, block_table, stream=None):
    """k_new, v_new: [tokens, Hkv, D] bf16 with equal strides, D contiguous (views into a fused QKV tensor
    are fine); the caches and the block table as for xy_attn_run.  Asynchronous."""
    assert k_new.stride(-1) == 1 and k_new.stride() == v_new.stride()
    assert k_cache.stride(-1) == 1 and k_cache.stride() == v_cache.stride() and block_table.is_contiguous()
    s = torch.cuda.current_stream() if stream is None else stream
    _check(_lib.xy_attn_append_kv(plan, _ptr(k_new), _ptr(v_new), k_new.stride(0), k_new.stride(1),
                                  _ptr(k_cache), _ptr(v_cache), k_cache.stride(0), k_cache.stride(1),
                                  k_cache.stride(2), _ptr(block_table), C.c_void_p(s.cuda_stream)))


def xy_attn_run_fused_qkv(plan, qkv, k_cache, v_cache, block_table, tree_masks, out, workspace, softmax_scale,
                          stream=None):
    """qkv: [tokens, Hq + 2 Hkv, D] bf16 (any token / head strides, D contiguous): K/V rows are appended
    to the cache, then attention runs with Q read in place.  Other arguments as for xy_attn_run."""
    _check(_lib.xy_attn_run_fused_qkv(*_run_args(plan, qkv, k_cache, v_cache, block_table, tree_masks, out,
                                                 workspace, softmax_scale, stream)))


def xy_probe_stream_read(src, sink, stream=None):
    """Read every byte of the tensor src once (see xy_attn.h); sink: any device tensor of >= 4 bytes."""
    s = torch.cuda.current_stream() if stream is None else stream
    _check(_lib.xy_probe_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), C.c_void_p(s.cuda_stream)))


def xy_probe_stream_read_once(src, sink, stream=None):
    """The same read with the non-temporal hint on every load."""
    s = torch.cuda.current_stream() if stream is None else stream
    _check(_lib.xy_probe_stream_read_once(_ptr(src), src.numel() * src.element_size(), _ptr(sink), C.c_void_p(s.cuda_stream)))


def xy_probe_mfma(iters, sink, stream=None):
    """2048 wavefronts x iters x 16 bf16 MFMAs of 32768 FLOPs (see xy_attn.h)."""
    s = torch.cuda.current_stream() if stream is None else stream
    _check(_lib.xy_probe_mfma(int(iters), _ptr(sink), C.c_void_p(s.cuda_stream)))


XY_MIX = {"none": 0, "even_4": 1, "uneven_8_0": 2, "dot2": 3, "scalar_2": 4, "attention": 5}


def xy_probe_issue_mix(mix, iters, cycles, sink, stream=None):
    """One wavefront per SIMD: iters x 32 MFMAs with the instructions of mix between them (see xy_attn.h);
    cycles: device int64 tensor of 1024 elements."""
    s = torch.cuda.current_stream() if stream is None else stream
    assert cycles.numel() >= 1024 and cycles.element_size() == 8
    _check(_lib.xy_probe_issue_mix(int(mix), int(iters), _ptr(cycles), _ptr(sink), C.c_void_p(s.cuda_stream)))


def xy_attn_copy_block_rows(copies, num_kv_heads, k_cache, v_cache, stream=None):
    """copies: list of (src_block, dst_block, rows): the copy-on-write copies of a step (see xy_attn.h)."""
    if not copies:
        return
    arr = (xy_kv_copy * len(copies))(*[xy_kv_copy(*map(int, c)) for c in copies])
    s = torch.cuda.current_stream() if stream is None else stream
    _check(_lib.xy_attn_copy_block_rows(arr, len(copies), int(num_kv_heads), _ptr(k_cache), _ptr(v_cache),
                                        k_cache.stride(0), k_cache.stride(1), k_cache.stride(2),
                                        C.c_void_p(s.cuda_stream)))


def xy_serve_schedule_chunk(token_budget, reserved_decode_slots, queue):
    """queue: list of (request, kind, tokens, context_len); returns [(request, kind, query_len, context_len)]."""
    n = len(queue)
    q = (xy_queue_entry * max(n, 1))(*[xy_queue_entry(*map(int, e)) for e in queue])
    out = (xy_chunk_entry * max(n, 1))()
    m = C.c_int32(0)
    _check(_lib.xy_serve_schedule_chunk(int(token_budget), int(reserved_decode_slots), q, n, out, C.byref(m)))
    return [(out[i].request, out[i].kind, out[i].query_len, out[i].context_len) for i in range(m.value)]


_i32_p = C.POINTER(C.c_int32)


def _tokens(tokens):
    """Token ids as a contiguous int32 array (no copy when they already are one)."""
    return np.ascontiguousarray(tokens, dtype=np.int32)


class KvManager:
    """The radix-tree K/V block manager (xy_serve.h); methods mirror the C calls."""

    def __init__(self, num_blocks, block_size):
        self._m = C.c_void_p()
        _check(_lib.xy_kv_create(int(num_blocks), int(block_size), C.byref(self._m)))

    def open(self, tokens):
        """Returns (seq, cached_tokens, [(src, dst, rows)]); raises XyError(XY_ERR_CAPACITY) when no block is to be had."""
        arr = _tokens(tokens)
        seq, cached, ncp, cp = C.c_int32(), C.c_int32(), C.c_int32(), xy_kv_copy()
        _check(_lib.xy_kv_open(self._m, arr.ctypes.data_as(_i32_p), len(arr), C.byref(seq), C.byref(cached),
                               C.byref(cp), C.byref(ncp)))
        return seq.value, cached.value, ([(cp.src_block, cp.dst_block, cp.rows)] if ncp.value else [])

    def extend(self, seq, tokens):
        arr = _tokens(tokens)
        _check(_lib.xy_kv_extend(self._m, int(seq), arr.ctypes.data_as(_i32_p), len(arr)))

    def block_row(self, seq):
        nb, ln = C.c_int32(), C.c_int32()
        _check(_lib.xy_kv_block_row(self._m, int(seq), None, 0, C.byref(nb), C.byref(ln)))
        row = (C.c_int32 * max(nb.value, 1))()
        _check(_lib.xy_kv_block_row(self._m, int(seq), row, nb.value, C.byref(nb), C.byref(ln)))
        return list(row[:nb.value])

    def block_row_into(self, seq, row):
        """The sequence's physical blocks written into row (a contiguous int32 array with room for them);
        returns their number."""
        nb, ln = C.c_int32(), C.c_int32()
        _check(_lib.xy_kv_block_row(self._m, int(seq), row.ctypes.data_as(_i32_p), len(row), C.byref(nb), C.byref(ln)))
        return nb.value

    def length(self, seq):
        ln = C.c_int32()
        _check(_lib.xy_kv_block_row(self._m, int(seq), None, 0, None, C.byref(ln)))
        return ln.value

    def close(self, seq):
        _check(_lib.xy_kv_close(self._m, int(seq)))

    def stats(self):
        out = (C.c_int64 * 4)()
        _check(_lib.xy_kv_stats(self._m, out))
        return {"free": out[0], "cached": out[1], "evictions": out[2], "open": out[3]}

    def destroy(self):
        if self._m:
            _lib.xy_kv_destroy(self._m)
            self._m = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
