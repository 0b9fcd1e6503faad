"""ctypes binding of libspex_tree.so: argument marshalling only.

Every step of the hot path (page table, planning, kernels) runs inside the
library; this module turns torch tensors into device pointers and Python lists
into int32 arrays.  There is no fallback: if the library has not been built the
import fails.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

from .build import LIB_PATH

NO_NODE = -1
F32, BF16, FP8_E4M3 = 0, 1, 2
_DTYPES = {"f32": F32, "bf16": BF16, "fp8_e4m3": FP8_E4M3}
_TORCH_KV = {F32: torch.float32, BF16: torch.bfloat16, FP8_E4M3: torch.uint8}

STATUS_NAMES = ["OK", "INVALID_ARG", "BAD_NODE", "NOT_LEAF", "OOM_PAGES", "EMPTY_PATH",
                "UNSUPPORTED", "DEVICE", "CAPACITY"]


class SpexError(RuntimeError):
    def __init__(self, status: int, detail: str = ""):
        self.status = status
        self.name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__(f"SPEX_ERR_{self.name}" + (f": {detail}" if detail else ""))


class Config(C.Structure):
    _fields_ = [
        ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("page_size", C.c_int32), ("q_dtype", C.c_int32), ("kv_dtype", C.c_int32),
        ("num_pages", C.c_int64),
        ("k_pool", C.c_void_p), ("v_pool", C.c_void_p),
        ("k_scale", C.c_void_p), ("v_scale", C.c_void_p),
        ("free_order", C.POINTER(C.c_int32)),
        ("prefix_chunk_pages", C.c_int32), ("suffix_chunk_pages", C.c_int32),
        ("kernel_mode", C.c_int32), ("page_stride_tiles", C.c_int32),
        ("walk_row_tiles", C.c_int32), ("walk_waves", C.c_int32),
    ]


class NodeInfo(C.Structure):
    _fields_ = [("parent", C.c_int32), ("n_tokens", C.c_int32), ("n_pages", C.c_int32),
                ("n_live_children", C.c_int32)]


_I32P = C.POINTER(C.c_int32)
_U32P = C.POINTER(C.c_uint32)


class PlanView(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_leaves", "n_qtok", "n_groups", "n_tasks",
                                         "n_prefix_tasks", "n_pg", "n_qt_list", "n_parts",
                                         "n_merge_qt")] + \
               [("n_partial_rows", C.c_int64), ("prefix_chunk_pages", C.c_int32),
                ("suffix_chunk_pages", C.c_int32)] + \
               [(n, _I32P) for n in ("leaf_indptr", "leaf_pages", "leaf_valid", "qt_limit",
                                     "group_node", "task_pg_begin", "task_pg_count",
                                     "task_qt_begin", "task_qt_count", "task_pbase", "task_flags",
                                     "pg_id", "pg_valid", "pg_pos", "qt_list", "part_indptr",
                                     "part_base", "part_hstride", "merge_qt")]


class WalkView(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("available", "row_tiles", "waves", "n_row_blocks", "n_blocks", "n_qt",
                                         "n_items", "plan_state")] + \
               [(n, _I32P) for n in ("row_blocks", "blocks", "qt", "items")]


EXPORTS = [
    "spex_pool_bytes", "spex_status_string", "spex_last_device_error", "spex_tree_create",
    "spex_tree_destroy", "spex_tree_fork", "spex_tree_append_step", "spex_tree_append_new_pages",
    "spex_tree_prune", "spex_tree_decode_attention", "spex_tree_decode_attention_masked",
    "spex_tree_decode_attention_static", "spex_tree_node_info", "spex_tree_path_pages",
    "spex_tree_free_pages", "spex_tree_stats", "spex_tree_plan_dump", "spex_tree_gather_kv",
    "spex_tree_set_tuning", "spex_tree_set_profiling", "spex_tree_read_profile",
    "spex_tree_last_launch_info", "spex_tree_walk_dump", "spex_tree_append_tokens", "spex_tree_append_tokens_quantize", "spex_tree_append_step_quantize",
]
# spex_sched.h: host-side scheduling primitives
SCHED_EXPORTS = [
    "spex_sched_rebase_widths", "spex_sched_ucb_select", "spex_sched_dfs_speculate",
    "spex_sched_allocate_budget", "spex_sched_early_termination", "spex_tree_path_kv_bytes",
]


class SearchTreeView(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("parent", C.POINTER(C.c_int32)), ("visits", C.POINTER(C.c_int64)),
                ("value_sum", C.POINTER(C.c_double)), ("state", C.POINTER(C.c_int32)),
                ("spec_reward", C.POINTER(C.c_double)), ("c", C.c_double)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2605_10195_amd.build` "
            "(there is no fallback implementation)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    lib.spex_pool_bytes.argtypes = [C.POINTER(Config), C.POINTER(C.c_size_t)]
    lib.spex_status_string.argtypes = [C.c_int]
    lib.spex_status_string.restype = C.c_char_p
    lib.spex_last_device_error.restype = C.c_char_p
    lib.spex_tree_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
    lib.spex_tree_destroy.argtypes = [vp]
    lib.spex_tree_destroy.restype = None
    lib.spex_tree_fork.argtypes = [vp, i32, i32, _I32P]
    lib.spex_tree_append_step.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp]
    lib.spex_tree_append_step_quantize.argtypes = [vp, i32, i32, vp, vp, vp]
    lib.spex_tree_append_new_pages.argtypes = [vp, i32, i32, _I32P]
    lib.spex_tree_append_tokens.argtypes = [vp, _I32P, i32, vp, vp, vp, vp, vp]
    lib.spex_tree_append_tokens_quantize.argtypes = [vp, _I32P, i32, vp, vp, vp, vp, vp]
    lib.spex_tree_prune.argtypes = [vp, i32]
    lib.spex_tree_decode_attention.argtypes = [vp, _I32P, _I32P, i32, vp, vp, vp, f32, vp]
    lib.spex_tree_decode_attention_masked.argtypes = [vp, _I32P, _I32P, _U32P, i32, vp, vp, vp, f32, vp]
    lib.spex_tree_decode_attention_static.argtypes = [vp, _I32P, _I32P, i32, vp, vp, vp, f32, vp]
    lib.spex_tree_node_info.argtypes = [vp, i32, C.POINTER(NodeInfo)]
    lib.spex_tree_path_pages.argtypes = [vp, i32, _I32P, _I32P, i32, _I32P]
    lib.spex_tree_free_pages.argtypes = [vp, _I32P, i32, _I32P]
    lib.spex_tree_stats.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
    lib.spex_tree_plan_dump.argtypes = [vp, _I32P, _I32P, i32, C.POINTER(PlanView)]
    lib.spex_tree_gather_kv.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp]
    lib.spex_tree_set_tuning.argtypes = [vp, i32, i32, i32, i32, i32]
    lib.spex_tree_walk_dump.argtypes = [vp, _I32P, _I32P, _U32P, i32, C.POINTER(WalkView)]
    lib.spex_tree_set_profiling.argtypes = [vp, i32]
    lib.spex_tree_read_profile.argtypes = [vp, C.POINTER(f32), i32, _I32P]
    lib.spex_tree_last_launch_info.argtypes = [vp, C.POINTER(i64)]
    _F64P = C.POINTER(C.c_double)
    lib.spex_sched_rebase_widths.argtypes = [_F64P, i32, i32, C.c_double, _I32P]
    lib.spex_sched_ucb_select.argtypes = [C.POINTER(SearchTreeView), _I32P]
    lib.spex_sched_dfs_speculate.argtypes = [C.POINTER(SearchTreeView), i32, _I32P, _I32P]
    lib.spex_sched_allocate_budget.argtypes = [_I32P, _F64P, _F64P, i32, C.c_double, C.c_double, i32, _I32P, _F64P]
    lib.spex_sched_early_termination.argtypes = [_I32P, _F64P, i32, i32, C.c_double, _I32P, _I32P]
    lib.spex_tree_path_kv_bytes.argtypes = [vp, i32, _F64P]
    for name in EXPORTS + SCHED_EXPORTS:
        fn = getattr(lib, name)
        if name not in ("spex_status_string", "spex_last_device_error", "spex_tree_destroy"):
            fn.restype = C.c_int
    return lib


lib = _load()


def _check(status: int):
    if status != 0:
        detail = lib.spex_last_device_error().decode() if status == 7 else ""
        raise SpexError(status, detail)


def _i32(seq) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(seq, dtype=np.int32))


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_I32P)


def _u32(seq) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(seq, dtype=np.uint32))


def _uptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_U32P)


def _dev(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream) if torch.cuda.is_available() else None


class SpexTree:
    """One forest over one page pool (spex_tree_t).  Method names follow the C entry points."""

    def __init__(self, num_q_heads: int, num_kv_heads: int, head_dim: int, page_size: int = 16,
                 q_dtype: str = "bf16", kv_dtype: str = "bf16", num_pages: int = 0,
                 device="cuda", free_order: Optional[Sequence[int]] = None,
                 prefix_chunk_pages: int = 0, suffix_chunk_pages: int = 0, kernel_mode: int = 0,
                 walk_row_tiles: int = 0, walk_waves: int = 0, host_only: bool = False, pool_fill: Optional[int] = None,
                 interleave_kv: bool = False):
        self.Hq, self.Hkv, self.D, self.P = num_q_heads, num_kv_heads, head_dim, page_size
        self.q_dtype, self.kv_dtype = _DTYPES[q_dtype], _DTYPES[kv_dtype]
        self.num_pages = int(num_pages)
        self.device = torch.device(device)
        self.host_only = host_only
        cfg = Config()
        cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim = num_q_heads, num_kv_heads, head_dim
        cfg.page_size, cfg.q_dtype, cfg.kv_dtype = page_size, self.q_dtype, self.kv_dtype
        cfg.num_pages = self.num_pages
        cfg.prefix_chunk_pages, cfg.suffix_chunk_pages = prefix_chunk_pages, suffix_chunk_pages
        cfg.kernel_mode = kernel_mode
        cfg.walk_row_tiles = walk_row_tiles
        cfg.walk_waves = walk_waves
        self.k_pool = self.v_pool = self.k_scale = self.v_scale = None
        if not host_only:
            nbytes = C.c_size_t()
            _check(lib.spex_pool_bytes(C.byref(cfg), C.byref(nbytes)))
            fill = 0 if pool_fill is None else pool_fill
            if interleave_kv:
                # one buffer, [page][K tiles of all heads | V tiles of all heads]
                esz = {F32: 4, BF16: 2, FP8_E4M3: 1}[self.kv_dtype]
                half = num_kv_heads * page_size * head_dim * esz
                self.k_pool = torch.full((max(2 * half * self.num_pages, 16),), fill, dtype=torch.uint8,
                                         device=self.device)
                self.v_pool = self.k_pool[half:]
                cfg.page_stride_tiles = 2 * num_kv_heads
            else:
                self.k_pool = torch.full((max(nbytes.value, 16),), fill, dtype=torch.uint8, device=self.device)
                self.v_pool = torch.full((max(nbytes.value, 16),), fill, dtype=torch.uint8, device=self.device)
            cfg.k_pool, cfg.v_pool = self.k_pool.data_ptr(), self.v_pool.data_ptr()
            if self.kv_dtype == FP8_E4M3:
                n = max(self.num_pages * num_kv_heads, 1)
                self.k_scale = torch.full((n,), float("nan"), dtype=torch.float32, device=self.device)
                self.v_scale = torch.full((n,), float("nan"), dtype=torch.float32, device=self.device)
                cfg.k_scale, cfg.v_scale = self.k_scale.data_ptr(), self.v_scale.data_ptr()
        self._order = None
        if free_order is not None:
            self._order = _i32(free_order)
            cfg.free_order = self._order.ctypes.data_as(_I32P)
        self._h = C.c_void_p()
        _check(lib.spex_tree_create(C.byref(cfg), C.byref(self._h)))

    def close(self):
        if getattr(self, "_h", None) and self._h.value:
            lib.spex_tree_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the five calls ------------------------------------------------------------------
    def fork(self, parent: int, n_children: int) -> List[int]:
        out = np.empty(max(n_children, 1), dtype=np.int32)
        _check(lib.spex_tree_fork(self._h, parent, n_children, _ptr(out)))
        return out[:n_children].tolist()

    def append_step(self, node: int, k: Optional[torch.Tensor], v: Optional[torch.Tensor],
                    k_scales: Optional[torch.Tensor] = None, v_scales: Optional[torch.Tensor] = None,
                    n_tokens: Optional[int] = None, quantize: bool = False) -> None:
        if k is None:
            _check(lib.spex_tree_append_step(self._h, node, int(n_tokens), None, None, None, None, None))
            return
        if quantize:                     # bf16 in, e4m3 codes and page scales made by the library
            assert k.dtype == torch.bfloat16 and v.dtype == torch.bfloat16 and k_scales is None
            assert k.is_contiguous() and v.is_contiguous() and k.device.type == self.device.type
            assert tuple(k.shape) == (k.shape[0], self.Hkv, self.D) and tuple(v.shape) == tuple(k.shape)
            _check(lib.spex_tree_append_step_quantize(self._h, node, k.shape[0], _dev(k), _dev(v), _stream()))
            return
        want = _TORCH_KV[self.kv_dtype]
        assert k.dtype == want and v.dtype == want, (k.dtype, want)
        assert k.is_contiguous() and v.is_contiguous() and k.device.type == self.device.type
        n = k.shape[0]
        assert tuple(k.shape) == (n, self.Hkv, self.D) and tuple(v.shape) == tuple(k.shape)
        if k_scales is not None:
            k_scales = k_scales.to(device=self.device, dtype=torch.float32).contiguous()
            v_scales = v_scales.to(device=self.device, dtype=torch.float32).contiguous()
        _check(lib.spex_tree_append_step(self._h, node, n, _dev(k), _dev(v), _dev(k_scales),
                                         _dev(v_scales), _stream()))
        # The scatter runs on torch's current stream, so the caching allocator cannot hand the
        # source buffers to later work before the scatter has read them.

    # name used by the trace replay
    def append(self, node, k, v, k_scales=None, v_scales=None, n_tokens=None):
        self.append_step(node, k, v, k_scales, v_scales, n_tokens)

    def append_tokens(self, nodes: Sequence[int], k: Optional[torch.Tensor], v: Optional[torch.Tensor],
                      k_scales: Optional[torch.Tensor] = None, v_scales: Optional[torch.Tensor] = None,
                      quantize: bool = False):
        """One token per node, one launch.  k, v: [len(nodes), Hkv, D] on the tree's device, in the
        pool's dtype, or -- quantize=True, fp8 pools -- in bf16, encoded by the library."""
        na = _i32(nodes)
        if k is not None:
            assert k.is_contiguous() and v.is_contiguous() and k.shape == (len(na), self.Hkv, self.D)
            assert not quantize or (k.dtype == torch.bfloat16 and v.dtype == torch.bfloat16)
        fn = lib.spex_tree_append_tokens_quantize if quantize else lib.spex_tree_append_tokens
        _check(fn(self._h, _ptr(na), len(na), _dev(k), _dev(v), _dev(k_scales), _dev(v_scales), _stream()))

    def prune(self, node: int) -> None:
        _check(lib.spex_tree_prune(self._h, node))

    def decode_attention(self, leaves: Sequence[int], q_lens: Optional[Sequence[int]],
                         q: torch.Tensor, sm_scale: float, out: Optional[torch.Tensor] = None,
                         lse: Optional[torch.Tensor] = None, want_lse: bool = True,
                         draft_masks: Optional[Sequence[int]] = None, static_scratch: bool = False):
        """static_scratch: go through spex_tree_decode_attention_static (the entry point that
        allocates nothing; out and lse must then be given)."""
        la = _i32(leaves)
        qa = None if q_lens is None else _i32(q_lens)
        nq = len(la) if qa is None else int(qa.sum())
        ma = None if draft_masks is None else _u32(draft_masks)
        assert ma is None or len(ma) == nq
        assert q.is_contiguous() and tuple(q.shape) == (nq, self.Hq, self.D), q.shape
        assert q.dtype == (torch.float32 if self.q_dtype == F32 else torch.bfloat16)
        if out is None:
            out = torch.empty((nq, self.Hq, self.D), dtype=torch.float32, device=q.device)
        if lse is None and want_lse:
            lse = torch.empty((nq, self.Hq), dtype=torch.float32, device=q.device)
        if static_scratch:
            assert ma is None, "the static entry point takes no draft masks"
            _check(lib.spex_tree_decode_attention_static(self._h, _ptr(la), _ptr(qa), len(la), _dev(q),
                                                         _dev(out), _dev(lse), float(sm_scale), _stream()))
        elif ma is None:
            _check(lib.spex_tree_decode_attention(self._h, _ptr(la), _ptr(qa), len(la), _dev(q),
                                                  _dev(out), _dev(lse), float(sm_scale), _stream()))
        else:
            _check(lib.spex_tree_decode_attention_masked(self._h, _ptr(la), _ptr(qa), _uptr(ma), len(la),
                                                         _dev(q), _dev(out), _dev(lse), float(sm_scale),
                                                         _stream()))
        return out, lse

    # ---- introspection -------------------------------------------------------------------
    def append_new_pages(self, node: int, n_tokens: int) -> int:
        n = C.c_int32()
        _check(lib.spex_tree_append_new_pages(self._h, node, n_tokens, C.byref(n)))
        return n.value

    def node_info(self, node: int) -> dict:
        info = NodeInfo()
        _check(lib.spex_tree_node_info(self._h, node, C.byref(info)))
        return dict(parent=info.parent, n_tokens=info.n_tokens, n_pages=info.n_pages,
                    n_live_children=info.n_live_children)

    def path_pages(self, node: int):
        n = C.c_int32()
        st = lib.spex_tree_path_pages(self._h, node, None, None, 0, C.byref(n))
        if st not in (0, 8):
            _check(st)
        pages = np.empty(max(n.value, 1), dtype=np.int32)
        valid = np.empty(max(n.value, 1), dtype=np.int32)
        _check(lib.spex_tree_path_pages(self._h, node, _ptr(pages), _ptr(valid), n.value, C.byref(n)))
        return pages[:n.value].tolist(), valid[:n.value].tolist()

    def free_pages(self) -> List[int]:
        n = C.c_int32()
        st = lib.spex_tree_free_pages(self._h, None, 0, C.byref(n))
        if st not in (0, 8):
            _check(st)
        pages = np.empty(max(n.value, 1), dtype=np.int32)
        _check(lib.spex_tree_free_pages(self._h, _ptr(pages), n.value, C.byref(n)))
        return pages[:n.value].tolist()

    def stats(self):
        a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
        _check(lib.spex_tree_stats(self._h, C.byref(a), C.byref(b), C.byref(c)))
        return a.value, b.value, c.value

    def plan_dump(self, leaves: Sequence[int], q_lens: Optional[Sequence[int]]) -> dict:
        la = _i32(leaves)
        qa = None if q_lens is None else _i32(q_lens)
        v = PlanView()
        _check(lib.spex_tree_plan_dump(self._h, _ptr(la), _ptr(qa), len(la), C.byref(v)))

        def arr(name, n):
            p = getattr(v, name)
            return [] if n == 0 else np.ctypeslib.as_array(p, shape=(n,)).tolist()

        return dict(
            leaf_indptr=arr("leaf_indptr", v.n_leaves + 1),
            leaf_pages=arr("leaf_pages", arr("leaf_indptr", v.n_leaves + 1)[-1]),
            leaf_valid=arr("leaf_valid", arr("leaf_indptr", v.n_leaves + 1)[-1]),
            qt_limit=arr("qt_limit", v.n_qtok), group_node=arr("group_node", v.n_groups),
            n_prefix_tasks=v.n_prefix_tasks, n_partial_rows=v.n_partial_rows,
            task_pg_begin=arr("task_pg_begin", v.n_tasks), task_pg_count=arr("task_pg_count", v.n_tasks),
            task_qt_begin=arr("task_qt_begin", v.n_tasks), task_qt_count=arr("task_qt_count", v.n_tasks),
            task_pbase=arr("task_pbase", v.n_tasks), task_flags=arr("task_flags", v.n_tasks),
            pg_id=arr("pg_id", v.n_pg), pg_valid=arr("pg_valid", v.n_pg), pg_pos=arr("pg_pos", v.n_pg),
            qt_list=arr("qt_list", v.n_qt_list),
            part_indptr=arr("part_indptr", v.n_qtok + 1), part_base=arr("part_base", v.n_parts),
            part_hstride=arr("part_hstride", v.n_parts), merge_qt=arr("merge_qt", v.n_merge_qt),
            prefix_chunk_pages=v.prefix_chunk_pages, suffix_chunk_pages=v.suffix_chunk_pages,
        )

    def gather_kv(self, node: int, first: int, n: int):
        dt = _TORCH_KV[self.kv_dtype]
        k = torch.empty((n, self.Hkv, self.D), dtype=dt, device=self.device)
        v = torch.empty_like(k)
        ks = vs = None
        if self.kv_dtype == FP8_E4M3:
            ks = torch.empty((n, self.Hkv), dtype=torch.float32, device=self.device)
            vs = torch.empty_like(ks)
        _check(lib.spex_tree_gather_kv(self._h, node, first, n, _dev(k), _dev(v), _dev(ks), _dev(vs),
                                       _stream()))
        return k, v, ks, vs

    def set_tuning(self, prefix_chunk_pages: int = 0, suffix_chunk_pages: int = 0, kernel_mode: int = 0,
                   walk_row_tiles: int = 0, walk_waves: int = 0):
        _check(lib.spex_tree_set_tuning(self._h, prefix_chunk_pages, suffix_chunk_pages, kernel_mode,
                                        walk_row_tiles, walk_waves))

    def walk_dump(self, leaves: Sequence[int], q_lens: Optional[Sequence[int]],
                  draft_masks: Optional[Sequence[int]] = None) -> dict:
        la = _i32(leaves)
        qa = None if q_lens is None else _i32(q_lens)
        ma = None if draft_masks is None else _u32(draft_masks)
        v = WalkView()
        _check(lib.spex_tree_walk_dump(self._h, _ptr(la), _ptr(qa), _uptr(ma), len(la), C.byref(v)))

        def arr(name, n):
            p = getattr(v, name)
            return [] if n == 0 else np.ctypeslib.as_array(p, shape=(n,)).tolist()

        nw = v.waves
        return dict(available=v.available, row_tiles=v.row_tiles, waves=nw, plan_state=v.plan_state,
                    row_blocks=arr("row_blocks", (3 + 3 * nw) * v.n_row_blocks),
                    blocks=arr("blocks", 8 * v.n_blocks), qt=arr("qt", 2 * v.n_qt),
                    items=arr("items", (16 if nw <= 4 else 32) * v.n_items))

    def set_profiling(self, enabled: bool):
        _check(lib.spex_tree_set_profiling(self._h, int(enabled)))

    def read_profile(self) -> np.ndarray:
        """[n_calls, 4] milliseconds (prefix, suffix, merge, tree-walk) of the calls recorded so far."""
        ms = np.zeros((256, 4), dtype=np.float32)
        n = C.c_int32()
        _check(lib.spex_tree_read_profile(self._h, ms.ctypes.data_as(C.POINTER(C.c_float)), 256,
                                          C.byref(n)))
        return ms[:n.value].copy()

    def last_launch_info(self) -> dict:
        info = (C.c_int64 * 8)()
        _check(lib.spex_tree_last_launch_info(self._h, info))
        names = ["kv_tokens", "prefix_tokens", "suffix_tokens", "prefix_items", "suffix_items",
                 "partial_rows", "plan_rebuilt", "walk_row_tiles"]
        d = {n: info[i] for i, n in enumerate(names)}
        d["walk_waves"] = d["walk_row_tiles"] // 256
        d["walk_row_tiles"] %= 256
        return d


# ---- functions named like the C entry points ------------------------------------------------
def spex_tree_create(**kwargs) -> SpexTree:
    return SpexTree(**kwargs)


def spex_tree_destroy(tree: SpexTree) -> None:
    tree.close()


def spex_tree_fork(tree: SpexTree, parent: int, n_children: int) -> List[int]:
    return tree.fork(parent, n_children)


def spex_tree_append_step(tree: SpexTree, node: int, k, v, k_scales=None, v_scales=None,
                          n_tokens=None) -> None:
    tree.append_step(node, k, v, k_scales, v_scales, n_tokens)


def spex_tree_prune(tree: SpexTree, node: int) -> None:
    tree.prune(node)


def spex_tree_decode_attention(tree: SpexTree, leaves, q_lens, q, sm_scale, out=None, lse=None):
    return tree.decode_attention(leaves, q_lens, q, sm_scale, out, lse)


def spex_tree_decode_attention_static(tree: SpexTree, leaves, q_lens, q, sm_scale, out, lse=None):
    return tree.decode_attention(leaves, q_lens, q, sm_scale, out, lse, want_lse=lse is not None,
                                 static_scratch=True)


def spex_tree_decode_attention_masked(tree: SpexTree, leaves, q_lens, draft_masks, q, sm_scale, out=None,
                                      lse=None):
    return tree.decode_attention(leaves, q_lens, q, sm_scale, out, lse, draft_masks=draft_masks)


def spex_tree_append_tokens_quantize(tree: SpexTree, nodes, k, v, k_scales, v_scales) -> None:
    tree.append_tokens(nodes, k, v, k_scales, v_scales, quantize=True)


# ---- spex_sched.h: argument marshalling only ------------------------------------------------
def _f64(seq) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(seq, dtype=np.float64))


def _dptr(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def spex_sched_rebase_widths(rewards, budget: int, temperature: float) -> List[int]:
    r = _f64(rewards)
    w = np.zeros(len(r), dtype=np.int32)
    _check(lib.spex_sched_rebase_widths(_dptr(r), len(r), int(budget), float(temperature), _ptr(w)))
    return w.tolist()


class SearchTree:
    """Arrays of a DFS / MCTS search tree in the layout spex_search_tree_t points to."""

    def __init__(self, parent, visits, value_sum, state=None, spec_reward=None, c: float = 1.0):
        n = len(parent)
        self.parent = _i32(parent)
        self.visits = np.ascontiguousarray(np.asarray(visits, dtype=np.int64))
        self.value_sum = _f64(value_sum)
        self.state = _i32(state if state is not None else [0] * n)
        self.spec_reward = _f64(spec_reward if spec_reward is not None else [0.0] * n)
        self.view = SearchTreeView(n, _ptr(self.parent), self.visits.ctypes.data_as(C.POINTER(C.c_int64)),
                                   _dptr(self.value_sum), _ptr(self.state), _dptr(self.spec_reward), float(c))


def spex_sched_ucb_select(tree: SearchTree) -> int:
    out = C.c_int32()
    _check(lib.spex_sched_ucb_select(C.byref(tree.view), C.byref(out)))
    return out.value


def spex_sched_dfs_speculate(tree: SearchTree, k: int) -> List[int]:
    sel = np.zeros(max(k, 1), dtype=np.int32)
    n = C.c_int32()
    _check(lib.spex_sched_dfs_speculate(C.byref(tree.view), int(k), _ptr(sel), C.byref(n)))
    return sel[:n.value].tolist()


def spex_sched_allocate_budget(capacity, hit_rate, kv_bytes, param_bytes: float, tau: float, k_total: int):
    c, p, s = _i32(capacity), _f64(hit_rate), _f64(kv_bytes)
    k = np.zeros(len(c), dtype=np.int32)
    scores = np.zeros(len(c), dtype=np.float64)
    _check(lib.spex_sched_allocate_budget(_ptr(c), _dptr(p), _dptr(s), len(c), float(param_bytes), float(tau),
                                          int(k_total), _ptr(k), _dptr(scores)))
    return k.tolist(), scores.tolist()


def spex_sched_early_termination(answer_id, weight, t: int, alpha: float):
    a, w = _i32(answer_id), _f64(weight)
    term, best = C.c_int32(), C.c_int32()
    _check(lib.spex_sched_early_termination(_ptr(a), _dptr(w), len(a), int(t), float(alpha), C.byref(term),
                                            C.byref(best)))
    return bool(term.value), best.value


def spex_tree_path_kv_bytes(tree: SpexTree, node: int) -> float:
    out = C.c_double()
    _check(lib.spex_tree_path_kv_bytes(tree._h, int(node), C.byref(out)))
    return out.value
