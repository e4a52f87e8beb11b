"""Thin ctypes binding over libomnisparse.so (argument marshalling only).

Function names mirror the C ABI in include/omnisparse.h.  torch is used for
device memory and the current HIP stream; every step of the computation runs in
the library's kernels.  There is no CPU fallback: if the shared library is
missing and cannot be built, importing a function raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libomnisparse.so")

OMNI_F32, OMNI_BF16 = 0, 1
(CALL_SCORE_QUERIES, CALL_SELECT_QUERIES, CALL_KV_BUDGET, CALL_SELECT_KV, CALL_SPARSE_ATTN_FWD,
 CALL_SPARSE_ATTN_BWD, CALL_SLIM_DECODE, CALL_DENSE_ATTN_FWD, CALL_DENSE_DECODE, CALL_GROUP_SUBSET,
 CALL_BLOCK_SCORES, CALL_PREFILL_SELECT, CALL_BLOCK_ATTN_FWD, CALL_BLOCK_ATTN_BWD) = range(14)

EXPORTED = [
    "omni_score_queries", "omni_select_queries", "omni_kv_budget", "omni_budget_from_scores", "omni_select_kv",
    "omni_sparse_attn_fwd", "omni_sparse_attn_bwd", "omni_slim_decode", "omni_visual_subset",
    "omni_dense_attn_fwd", "omni_dense_decode", "omni_workspace_bytes", "omni_last_error", "omni_version",
    "omni_profile_enable", "omni_profile_read", "omni_debug_work_list", "omni_debug_copy", "omni_debug_mfma_rate",
    "omni_group_subset", "omni_slim_decode_grouped", "omni_block_scores", "omni_expand_blocks",
    "omni_block_attn_fwd", "omni_block_attn_bwd", "omni_prefill_select_varlen",
    "omni_select_kv_per_head", "omni_sparse_attn_fwd_per_head", "omni_sparse_attn_bwd_per_head",
    "omni_visual_subset_per_head", "omni_prefill_select", "omni_compact_cache", "omni_slim_decode_compact",
    "omni_compact_cache_paged", "omni_slim_decode_paged",
    "omni_group_subset_per_head", "omni_debug_key_split_len",
    "omni_slim_decode_grouped_static", "omni_static_scratch_bytes",
    "omni_sparse_prefill", "omni_sparse_prefill_workspace_bytes", "omni_slim_decode_prepare",
]

PROF_KERNELS = {"attn_fwd": 0, "pack_kv": 1, "clear_out": 2, "pool_q": 3, "probe_lse": 4, "probe_sum": 5,
                "score": 6, "bwd_dkdv": 7, "bwd_dq": 8, "bwd_reduce": 9, "decode": 10, "select": 11}


class LayerDesc(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("n_tokens", C.c_int32), ("vis_begin", C.c_int32), ("vis_end", C.c_int32), ("sink_index", C.c_int32),
        ("causal", C.c_int32), ("dtype", C.c_int32), ("softmax_scale", C.c_float),
        ("q_stride", C.c_int64 * 3), ("kv_stride", C.c_int64 * 3),
    ]


class DecodeDesc(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("cache_capacity", C.c_int32), ("vis_begin", C.c_int32), ("vis_end", C.c_int32), ("dtype", C.c_int32),
        ("softmax_scale", C.c_float), ("tau", C.c_float), ("kv_stride", C.c_int64 * 3),
        ("static_lists", C.c_int32),
    ]


class PagePool(C.Structure):
    _fields_ = [
        ("K", C.c_void_p), ("V", C.c_void_p), ("page_table", C.c_void_p),
        ("n_pages", C.c_int32), ("page_rows", C.c_int32), ("pages_cap", C.c_int32),
    ]


def make_page_pool(Kpool, Vpool, page_table) -> PagePool:
    """Descriptor of a page pool: Kpool / Vpool [n_pages, page_rows, D], page_table [B, Hkv, pages_cap] int32."""
    if not (Kpool.is_contiguous() and Vpool.is_contiguous() and page_table.is_contiguous()):
        raise ValueError("pool tensors and page table must be contiguous")
    if page_table.dtype != torch.int32 or Kpool.shape != Vpool.shape or Kpool.dim() != 3:
        raise ValueError("page_table must be int32; Kpool and Vpool [n_pages, page_rows, head_dim]")
    pool = PagePool()
    pool.K, pool.V, pool.page_table = Kpool.data_ptr(), Vpool.data_ptr(), page_table.data_ptr()
    pool.n_pages, pool.page_rows, pool.pages_cap = Kpool.shape[0], Kpool.shape[1], page_table.shape[-1]
    pool._keep = (Kpool, Vpool, page_table)
    return pool


class OmniError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"omnisparse error {code}: {message}")
        self.code = code
        self.message = message


_lib = None


def load_library(path: str = LIB_PATH) -> C.CDLL:
    """Loads the built library (builds it first if no build exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        from . import build as _build
        _build.build()
    lib = C.CDLL(path)
    vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
    lib.omni_last_error.restype = C.c_char_p
    lib.omni_version.restype = C.c_int
    lib.omni_workspace_bytes.restype = sz
    lib.omni_workspace_bytes.argtypes = [C.c_int, vp, i32]
    lib.omni_score_queries.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp]
    lib.omni_select_queries.argtypes = [vp, vp, C.c_int, f32, vp, vp, vp, sz, vp]
    lib.omni_kv_budget.argtypes = [vp, vp, vp, f32, C.c_int, C.c_int, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.omni_budget_from_scores.argtypes = [vp, vp, f32, C.c_int, vp, vp, vp, vp, vp, sz, vp]
    lib.omni_prefill_select.argtypes = [vp, vp, vp, C.c_int, f32, f32, C.c_int, C.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                        vp, i32, vp, sz, vp]
    lib.omni_sparse_prefill.argtypes = [vp, vp, vp, vp, C.c_int, f32, f32, C.c_int, C.c_int, vp, vp, vp, vp, vp, vp, vp,
                                        vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.omni_sparse_prefill_workspace_bytes.argtypes = [vp, i32, i32]
    lib.omni_sparse_prefill_workspace_bytes.restype = sz
    lib.omni_prefill_select_varlen.argtypes = [vp, vp, vp, vp, vp, vp, C.c_int, f32, f32, C.c_int, C.c_int, vp, vp, vp, vp,
                                               vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.omni_select_kv.argtypes = [vp, vp, vp, i32, vp, vp, sz, vp]
    lib.omni_visual_subset.argtypes = [vp, vp, vp, i32, vp, vp, vp]
    lib.omni_select_kv_per_head.argtypes = lib.omni_select_kv.argtypes
    lib.omni_visual_subset_per_head.argtypes = lib.omni_visual_subset.argtypes
    lib.omni_sparse_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.omni_dense_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.omni_sparse_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, sz, vp]
    lib.omni_sparse_attn_fwd_per_head.argtypes = lib.omni_sparse_attn_fwd.argtypes
    lib.omni_sparse_attn_bwd_per_head.argtypes = lib.omni_sparse_attn_bwd.argtypes
    lib.omni_slim_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.omni_slim_decode_prepare.argtypes = [vp, vp, vp, i32, vp, sz, vp]
    lib.omni_dense_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.omni_group_subset.argtypes = [vp, vp, vp, i32, vp, vp, vp, i32, vp, sz, vp]
    lib.omni_group_subset_per_head.argtypes = lib.omni_group_subset.argtypes
    lib.omni_block_scores.argtypes = [vp, vp, vp, i32, vp, vp, sz, vp]
    lib.omni_expand_blocks.argtypes = [vp, vp, vp, i32, i32, vp, vp, i32, vp]
    lib.omni_block_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, sz, vp]
    lib.omni_block_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.omni_slim_decode_grouped.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.omni_slim_decode_grouped_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp]
    lib.omni_static_scratch_bytes.restype = sz
    lib.omni_static_scratch_bytes.argtypes = []
    lib.omni_compact_cache.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, vp]
    lib.omni_slim_decode_compact.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.omni_compact_cache_paged.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp]
    lib.omni_slim_decode_paged.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.omni_profile_enable.argtypes = [C.c_int]
    lib.omni_debug_copy.argtypes = [vp, vp, sz, vp]
    lib.omni_debug_key_split_len.argtypes = [C.c_int]
    lib.omni_debug_mfma_rate.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.omni_debug_work_list.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, i32, vp, vp]   # same shape: three output arrays
    lib.omni_profile_read.argtypes = [C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_int)]
    for name in EXPORTED:
        fn = getattr(lib, name)
        if name not in ("omni_last_error", "omni_version", "omni_workspace_bytes"):
            fn.restype = C.c_int
    _lib = lib
    return lib


def last_error() -> str:
    return load_library().omni_last_error().decode()


def _check(rc: int):
    if rc != 0:
        raise OmniError(rc, last_error())


def _ptr(t):
    if t is None:
        return None
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return OMNI_BF16
    if t.dtype == torch.float32:
        return OMNI_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def make_layer_desc(Q: torch.Tensor, K: torch.Tensor, vis_begin: int, vis_end: int, sink_index: int = 0,
                    causal: bool = True, softmax_scale: float | None = None) -> LayerDesc:
    B, Hq, N, D = Q.shape
    d = LayerDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim, d.n_tokens = B, Hq, K.shape[1], D, N
    d.vis_begin, d.vis_end, d.sink_index = vis_begin, vis_end, sink_index
    d.causal = 1 if causal else 0
    d.dtype = _dtype_code(Q)
    d.softmax_scale = softmax_scale if softmax_scale is not None else D ** -0.5
    if Q.stride(3) != 1 or K.stride(3) != 1:
        raise ValueError("head_dim must be contiguous")
    d.q_stride = (C.c_int64 * 3)(*Q.stride()[:3])
    d.kv_stride = (C.c_int64 * 3)(*K.stride()[:3])
    return d


def make_decode_desc(q: torch.Tensor, Kcache: torch.Tensor, vis_begin: int, vis_end: int, tau: float,
                     softmax_scale: float | None = None, static_lists: bool = False) -> DecodeDesc:
    B, Hq, D = q.shape
    d = DecodeDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = B, Hq, Kcache.shape[1], D
    d.cache_capacity = Kcache.shape[2]
    d.vis_begin, d.vis_end = vis_begin, vis_end
    d.dtype = _dtype_code(q)
    d.softmax_scale = softmax_scale if softmax_scale is not None else D ** -0.5
    d.tau = tau
    d.kv_stride = (C.c_int64 * 3)(*Kcache.stride()[:3])
    d.static_lists = 1 if static_lists else 0
    return d


def debug_work_list(desc: LayerDesc, q_cnt=None, budget=None, b_cap: int = 1, tile_rows: int = 128, queues: int = 1):
    """Host mirror of the device work list: (item_head[n], item_tile[n], item_cost[n]) in hand-out order, queue after
    queue; with queues > 1 also the end position of every queue."""
    import numpy as np
    lib = load_library()
    cap = desc.batch * desc.n_q_heads * ((desc.n_tokens + 127) // 128)
    head = np.zeros(cap, dtype=np.int32)
    tile = np.zeros(cap, dtype=np.int32)
    cost = np.zeros(cap, dtype=np.int32)
    n = C.c_int32(0)
    qc = None if q_cnt is None else np.ascontiguousarray(q_cnt, dtype=np.int32)
    bd = None if budget is None else np.ascontiguousarray(budget, dtype=np.int32)
    qend = np.zeros(8, dtype=np.int32)
    _check(lib.omni_debug_work_list(C.byref(desc), None if qc is None else qc.ctypes.data,
                                    None if bd is None else bd.ctypes.data, b_cap, tile_rows, queues, head.ctypes.data,
                                    tile.ctypes.data, cost.ctypes.data, cap, C.byref(n), qend.ctypes.data))
    if queues > 1:
        return head[: n.value], tile[: n.value], cost[: n.value], qend
    return head[: n.value], tile[: n.value], cost[: n.value]


def debug_copy(src, dst):
    """Copy src into dst (same byte size, a multiple of 16) with the library's calibration copy kernel."""
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    _check(load_library().omni_debug_copy(_ptr(src), _ptr(dst), nbytes, _stream()))


def debug_key_split_len(tiles: int):
    """Query tiles per share of a split key tile in the backward pass (<= 0: default)."""
    _check(load_library().omni_debug_key_split_len(int(tiles)))


def debug_mfma_rate(random_operands, iters: int = 40000):
    """(TFLOP/s, shader MHz) of register-resident bf16 MFMAs: constant operands (0 / False), pseudo-random ones
    (1 / True), or pseudo-random with the matrix cores idle a third of the time (2)."""
    tf, mhz = C.c_double(0), C.c_double(0)
    _check(load_library().omni_debug_mfma_rate(int(random_operands), iters, C.byref(tf), C.byref(mhz)))
    return tf.value, mhz.value


def profile_enable(on: bool, kernels=None):
    """Kernel timing on (every kernel of PROF_KERNELS, or only the named ones) or off; resets the records."""
    mask = 0
    if on:
        mask = -1 if kernels is None else sum(1 << PROF_KERNELS[k] for k in kernels)
    _check(load_library().omni_profile_enable(mask))


def profile_read(kernel: str):
    """(total milliseconds, launches) recorded for one kernel since profile_enable(True)."""
    ms, n = C.c_float(0), C.c_int(0)
    _check(load_library().omni_profile_read(PROF_KERNELS[kernel], C.byref(ms), C.byref(n)))
    return float(ms.value), int(n.value)


def workspace_bytes(call_id: int, desc, param: int = 0) -> int:
    n = load_library().omni_workspace_bytes(call_id, C.byref(desc), param)
    if n == 0:
        raise OmniError(-1, last_error() or "invalid descriptor")
    return int(n)


class Workspace:
    """Caller-owned scratch buffers, one per call id, grown on demand and reused."""

    def __init__(self, device="cuda"):
        self.device = device
        self.bufs: dict[int, torch.Tensor] = {}

    def get(self, call_id: int, desc, param: int = 0):
        need = workspace_bytes(call_id, desc, param)
        buf = self.bufs.get(call_id)
        if buf is None or buf.numel() < need:
            buf = torch.empty(need, dtype=torch.uint8, device=self.device)
            self.bufs[call_id] = buf
        return buf


_default_ws = None


def default_workspace() -> Workspace:
    global _default_ws
    if _default_ws is None:
        _default_ws = Workspace()
    return _default_ws


# ------------------------------------------------------------------ entry points

def omni_score_queries(desc: LayerDesc, Q, K, probe_keys=None, scores=None, ws: Workspace | None = None):
    lib = load_library()
    ws = ws or default_workspace()
    dev = Q.device
    if probe_keys is None:
        probe_keys = torch.empty(desc.batch, desc.n_kv_heads, 2, desc.head_dim, dtype=torch.float32, device=dev)
    if scores is None:
        scores = torch.empty(desc.batch, desc.n_q_heads, desc.n_tokens, dtype=torch.float32, device=dev)
    buf = ws.get(CALL_SCORE_QUERIES, desc)
    _check(lib.omni_score_queries(C.byref(desc), _ptr(Q), _ptr(K), _ptr(probe_keys), _ptr(scores), _ptr(buf),
                                  buf.numel(), _stream()))
    return probe_keys, scores


def omni_select_queries(desc: LayerDesc, scores, mode: int, param: float, q_idx=None, q_cnt=None,
                        ws: Workspace | None = None):
    lib = load_library()
    ws = ws or default_workspace()
    dev = scores.device
    if q_idx is None:
        q_idx = torch.empty(desc.batch, desc.n_q_heads, desc.n_tokens, dtype=torch.int32, device=dev)
    if q_cnt is None:
        q_cnt = torch.empty(desc.batch, desc.n_q_heads, dtype=torch.int32, device=dev)
    buf = ws.get(CALL_SELECT_QUERIES, desc)
    _check(lib.omni_select_queries(C.byref(desc), _ptr(scores), mode, param, _ptr(q_idx), _ptr(q_cnt), _ptr(buf),
                                   buf.numel(), _stream()))
    return q_idx, q_cnt


@dataclass
class BudgetResult:
    key_scores: torch.Tensor
    kurtosis: torch.Tensor
    flattest: torch.Tensor
    budget: torch.Tensor
    recall: torch.Tensor


def omni_kv_budget(desc: LayerDesc, Q, K, recall_p: float, probe_block: int = 256, budget_mode: int = 0,
                   out: BudgetResult | None = None, budget_host=None, ws: Workspace | None = None) -> BudgetResult:
    lib = load_library()
    ws = ws or default_workspace()
    dev = Q.device
    B, H, N = desc.batch, desc.n_q_heads, desc.n_tokens
    if out is None:
        out = BudgetResult(
            torch.empty(B, H, N, dtype=torch.float32, device=dev), torch.empty(B, H, dtype=torch.float64, device=dev),
            torch.empty(B, dtype=torch.int32, device=dev),
            torch.empty((B, H) if budget_mode == 2 else (B,), dtype=torch.int32, device=dev),
            torch.empty(B, H, dtype=torch.float32, device=dev))
    buf = ws.get(CALL_KV_BUDGET, desc, probe_block)
    _check(lib.omni_kv_budget(C.byref(desc), _ptr(Q), _ptr(K), recall_p, probe_block, budget_mode,
                              _ptr(out.key_scores), _ptr(out.kurtosis), _ptr(out.flattest), _ptr(out.budget),
                              _ptr(out.recall), _ptr(budget_host), _ptr(buf), buf.numel(), _stream()))
    return out


@dataclass
class SelectionResult:
    probe_keys: torch.Tensor
    scores: torch.Tensor
    q_idx: torch.Tensor
    q_cnt: torch.Tensor
    budget: BudgetResult
    kv_idx: torch.Tensor


def omni_prefill_select(desc: LayerDesc, Q, K, q_mode: int, q_param: float, recall_p: float, probe_block: int = 256,
                        budget_mode: int = 0, b_cap: int | None = None, out: SelectionResult | None = None,
                        ws: Workspace | None = None) -> SelectionResult:
    lib = load_library()
    ws = ws or default_workspace()
    dev = Q.device
    B, H, Hkv, N, D = desc.batch, desc.n_q_heads, desc.n_kv_heads, desc.n_tokens, desc.head_dim
    b_cap = N if b_cap is None else b_cap
    f32, i32 = torch.float32, torch.int32
    if out is None:
        bud = BudgetResult(
            torch.empty(B, H, N, dtype=f32, device=dev), torch.empty(B, H, dtype=torch.float64, device=dev),
            torch.empty(B, dtype=i32, device=dev),
            torch.empty((B, H) if budget_mode == 2 else (B,), dtype=i32, device=dev),
            torch.empty(B, H, dtype=f32, device=dev))
        out = SelectionResult(
            torch.empty(B, Hkv, 2, D, dtype=f32, device=dev), torch.empty(B, H, N, dtype=f32, device=dev),
            torch.empty(B, H, N, dtype=i32, device=dev), torch.empty(B, H, dtype=i32, device=dev), bud,
            torch.empty(B, H, b_cap, dtype=i32, device=dev))
    _budget_shape_ok(desc, out.budget.budget, budget_mode == 2)
    if out.kv_idx.shape[-1] != b_cap:
        raise ValueError("kv_idx must be [batch, n_q_heads, b_cap]")
    buf = ws.get(CALL_PREFILL_SELECT, desc, probe_block)
    r = out.budget
    _check(lib.omni_prefill_select(C.byref(desc), _ptr(Q), _ptr(K), q_mode, q_param, recall_p, probe_block, budget_mode,
                                   _ptr(out.probe_keys), _ptr(out.scores), _ptr(out.q_idx), _ptr(out.q_cnt),
                                   _ptr(r.key_scores), _ptr(r.kurtosis), _ptr(r.flattest), _ptr(r.budget),
                                   _ptr(r.recall), _ptr(out.kv_idx), b_cap, _ptr(buf), buf.numel(), _stream()))
    return out


CALL_SPARSE_PREFILL_WS = -1      # key of the binding's workspace pool only; the library sizes this call by a function


def omni_sparse_prefill(desc: LayerDesc, Q, K, V, q_mode: int, q_param: float, recall_p: float, probe_block: int = 256,
                        budget_mode: int = 0, b_cap: int | None = None, out: SelectionResult | None = None, O=None,
                        lse=None, ws: Workspace | None = None):
    """Selection and sparse attention forward of a prefill step in one call: (SelectionResult, O, lse)."""
    lib = load_library()
    ws = ws or default_workspace()
    dev = Q.device
    B, H, Hkv, N, D = desc.batch, desc.n_q_heads, desc.n_kv_heads, desc.n_tokens, desc.head_dim
    b_cap = N if b_cap is None else b_cap
    f32, i32 = torch.float32, torch.int32
    if out is None:
        bud = BudgetResult(
            torch.empty(B, H, N, dtype=f32, device=dev), torch.empty(B, H, dtype=torch.float64, device=dev),
            torch.empty(B, dtype=i32, device=dev),
            torch.empty((B, H) if budget_mode == 2 else (B,), dtype=i32, device=dev),
            torch.empty(B, H, dtype=f32, device=dev))
        out = SelectionResult(
            torch.empty(B, Hkv, 2, D, dtype=f32, device=dev), torch.empty(B, H, N, dtype=f32, device=dev),
            torch.empty(B, H, N, dtype=i32, device=dev), torch.empty(B, H, dtype=i32, device=dev), bud,
            torch.empty(B, H, b_cap, dtype=i32, device=dev))
    _budget_shape_ok(desc, out.budget.budget, budget_mode == 2)
    if out.kv_idx.shape[-1] != b_cap:
        raise ValueError("kv_idx must be [batch, n_q_heads, b_cap]")
    if O is None:
        O = torch.empty_like(Q)
    if lse is None:
        lse = torch.empty(B, H, N, dtype=f32, device=dev)
    need = lib.omni_sparse_prefill_workspace_bytes(C.byref(desc), probe_block, b_cap)
    if need == 0:
        raise OmniError(-1, last_error())
    buf = ws.bufs.get(CALL_SPARSE_PREFILL_WS)
    if buf is None or buf.numel() < need:
        buf = torch.empty(need, dtype=torch.uint8, device=ws.device)
        ws.bufs[CALL_SPARSE_PREFILL_WS] = buf
    r = out.budget
    _check(lib.omni_sparse_prefill(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), q_mode, q_param, recall_p, probe_block,
                                   budget_mode, _ptr(out.probe_keys), _ptr(out.scores), _ptr(out.q_idx), _ptr(out.q_cnt),
                                   _ptr(r.key_scores), _ptr(r.kurtosis), _ptr(r.flattest), _ptr(r.budget),
                                   _ptr(r.recall), _ptr(out.kv_idx), b_cap, _ptr(O), _ptr(lse), _ptr(buf), buf.numel(),
                                   _stream()))
    return out, O, lse


def omni_prefill_select_varlen(desc: LayerDesc, Q, K, seq_tokens, seq_vis_begin, seq_vis_end, q_mode: int, q_param: float,
                               recall_p: float, probe_block: int = 256, budget_mode: int = 0, b_cap: int | None = None,
                               ws: Workspace | None = None) -> SelectionResult:
    """Fused selection of a padded batch of sequences with their own lengths and visual ranges (host int sequences)."""
    lib = load_library()
    ws = ws or default_workspace()
    dev = Q.device
    B, H, Hkv, N, D = desc.batch, desc.n_q_heads, desc.n_kv_heads, desc.n_tokens, desc.head_dim
    b_cap = N if b_cap is None else b_cap
    f32, i32 = torch.float32, torch.int32
    bud = BudgetResult(
        torch.empty(B, H, N, dtype=f32, device=dev), torch.empty(B, H, dtype=torch.float64, device=dev),
        torch.empty(B, dtype=i32, device=dev), torch.empty((B, H) if budget_mode == 2 else (B,), dtype=i32, device=dev),
        torch.empty(B, H, dtype=f32, device=dev))
    out = SelectionResult(
        torch.empty(B, Hkv, 2, D, dtype=f32, device=dev), torch.empty(B, H, N, dtype=f32, device=dev),
        torch.empty(B, H, N, dtype=i32, device=dev), torch.empty(B, H, dtype=i32, device=dev), bud,
        torch.empty(B, H, b_cap, dtype=i32, device=dev))
    arr = lambda x: (C.c_int32 * B)(*[int(v) for v in x])
    n_arr, v0_arr, v1_arr = arr(seq_tokens), arr(seq_vis_begin), arr(seq_vis_end)
    one = LayerDesc.from_buffer_copy(desc)
    one.batch = 1
    buf = ws.get(CALL_PREFILL_SELECT, one, probe_block)
    _check(lib.omni_prefill_select_varlen(C.byref(desc), _ptr(Q), _ptr(K), n_arr, v0_arr, v1_arr, q_mode, q_param, recall_p,
                                          probe_block, budget_mode, _ptr(out.probe_keys), _ptr(out.scores), _ptr(out.q_idx),
                                          _ptr(out.q_cnt), _ptr(bud.key_scores), _ptr(bud.kurtosis), _ptr(bud.flattest),
                                          _ptr(bud.budget), _ptr(bud.recall), _ptr(out.kv_idx), b_cap, _ptr(buf), buf.numel(),
                                          _stream()))
    return out


def omni_budget_from_scores(desc: LayerDesc, key_scores, recall_p: float, budget_mode: int = 0,
                            ws: Workspace | None = None) -> BudgetResult:
    lib = load_library()
    ws = ws or default_workspace()
    dev = key_scores.device
    B, H = desc.batch, desc.n_q_heads
    out = BudgetResult(key_scores, torch.empty(B, H, dtype=torch.float64, device=dev),
                       torch.empty(B, dtype=torch.int32, device=dev),
                       torch.empty((B, H) if budget_mode == 2 else (B,), dtype=torch.int32, device=dev),
                       torch.empty(B, H, dtype=torch.float32, device=dev))
    buf = ws.get(CALL_KV_BUDGET, desc, 256)
    _check(lib.omni_budget_from_scores(C.byref(desc), _ptr(key_scores), recall_p, budget_mode, _ptr(out.kurtosis),
                                       _ptr(out.flattest), _ptr(out.budget), _ptr(out.recall), _ptr(buf), buf.numel(),
                                       _stream()))
    return out


def _budget_shape_ok(desc, budget, per_head: bool):
    want = desc.batch * (desc.n_q_heads if per_head else 1)
    if budget.numel() != want:
        raise ValueError(f"budget has {budget.numel()} entries, this call reads {want}")


def omni_select_kv(desc: LayerDesc, key_scores, budget, b_cap: int, kv_idx=None, ws: Workspace | None = None,
                   _per_head: bool = False):
    lib = load_library()
    _budget_shape_ok(desc, budget, _per_head)
    ws = ws or default_workspace()
    if kv_idx is None:
        kv_idx = torch.empty(desc.batch, desc.n_q_heads, b_cap, dtype=torch.int32, device=key_scores.device)
    buf = ws.get(CALL_SELECT_KV, desc)
    fn = lib.omni_select_kv_per_head if _per_head else lib.omni_select_kv
    _check(fn(C.byref(desc), _ptr(key_scores), _ptr(budget), b_cap, _ptr(kv_idx), _ptr(buf), buf.numel(), _stream()))
    return kv_idx


def omni_select_kv_per_head(desc: LayerDesc, key_scores, budget, b_cap: int, kv_idx=None, ws: Workspace | None = None):
    return omni_select_kv(desc, key_scores, budget, b_cap, kv_idx, ws, _per_head=True)


def omni_visual_subset(desc: LayerDesc, kv_idx, budget, b_cap: int, vis_idx=None, vis_cnt=None,
                       _per_head: bool = False):
    lib = load_library()
    _budget_shape_ok(desc, budget, _per_head)
    dev = kv_idx.device
    if vis_idx is None:
        vis_idx = torch.empty(desc.batch, desc.n_q_heads, b_cap, dtype=torch.int32, device=dev)
    if vis_cnt is None:
        vis_cnt = torch.empty(desc.batch, desc.n_q_heads, dtype=torch.int32, device=dev)
    fn = lib.omni_visual_subset_per_head if _per_head else lib.omni_visual_subset
    _check(fn(C.byref(desc), _ptr(kv_idx), _ptr(budget), b_cap, _ptr(vis_idx), _ptr(vis_cnt), _stream()))
    return vis_idx, vis_cnt


def omni_visual_subset_per_head(desc: LayerDesc, kv_idx, budget, b_cap: int, vis_idx=None, vis_cnt=None):
    return omni_visual_subset(desc, kv_idx, budget, b_cap, vis_idx, vis_cnt, _per_head=True)


def omni_sparse_attn_fwd(desc: LayerDesc, Q, K, V, q_idx, q_cnt, kv_idx, budget, b_cap: int, O=None, lse=None,
                         ws: Workspace | None = None, _per_head: bool = False):
    lib = load_library()
    _budget_shape_ok(desc, budget, _per_head)
    ws = ws or default_workspace()
    if O is None:
        O = torch.empty_like(Q)
    if lse is None:
        lse = torch.empty(desc.batch, desc.n_q_heads, desc.n_tokens, dtype=torch.float32, device=Q.device)
    buf = ws.get(CALL_SPARSE_ATTN_FWD, desc, b_cap)
    fn = lib.omni_sparse_attn_fwd_per_head if _per_head else lib.omni_sparse_attn_fwd
    _check(fn(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(q_idx), _ptr(q_cnt), _ptr(kv_idx), _ptr(budget), b_cap,
              _ptr(O), _ptr(lse), _ptr(buf), buf.numel(), _stream()))
    return O, lse


def omni_sparse_attn_fwd_per_head(desc: LayerDesc, Q, K, V, q_idx, q_cnt, kv_idx, budget, b_cap: int, O=None, lse=None,
                                  ws: Workspace | None = None):
    return omni_sparse_attn_fwd(desc, Q, K, V, q_idx, q_cnt, kv_idx, budget, b_cap, O, lse, ws, _per_head=True)


def omni_dense_attn_fwd(desc: LayerDesc, Q, K, V, O=None, lse=None, ws: Workspace | None = None):
    lib = load_library()
    ws = ws or default_workspace()
    if O is None:
        O = torch.empty_like(Q)
    if lse is None:
        lse = torch.empty(desc.batch, desc.n_q_heads, desc.n_tokens, dtype=torch.float32, device=Q.device)
    buf = ws.get(CALL_DENSE_ATTN_FWD, desc)
    _check(lib.omni_dense_attn_fwd(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(lse), _ptr(buf),
                                   buf.numel(), _stream()))
    return O, lse


def omni_sparse_attn_bwd(desc: LayerDesc, Q, K, V, O, dO, lse, q_idx, q_cnt, kv_idx, budget, b_cap: int,
                         dQ=None, dK=None, dV=None, ws: Workspace | None = None, _per_head: bool = False):
    lib = load_library()
    _budget_shape_ok(desc, budget, _per_head)
    ws = ws or default_workspace()
    if dQ is None:
        dQ = torch.empty_like(Q)
    if dK is None:
        dK = torch.empty_like(K)
    if dV is None:
        dV = torch.empty_like(V)
    buf = ws.get(CALL_SPARSE_ATTN_BWD, desc, b_cap)
    fn = lib.omni_sparse_attn_bwd_per_head if _per_head else lib.omni_sparse_attn_bwd
    _check(fn(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(lse), _ptr(q_idx), _ptr(q_cnt),
              _ptr(kv_idx), _ptr(budget), b_cap, _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(buf), buf.numel(), _stream()))
    return dQ, dK, dV


def omni_sparse_attn_bwd_per_head(desc: LayerDesc, Q, K, V, O, dO, lse, q_idx, q_cnt, kv_idx, budget, b_cap: int,
                                  dQ=None, dK=None, dV=None, ws: Workspace | None = None):
    return omni_sparse_attn_bwd(desc, Q, K, V, O, dO, lse, q_idx, q_cnt, kv_idx, budget, b_cap, dQ, dK, dV, ws,
                                _per_head=True)


def omni_slim_decode(desc: DecodeDesc, q, Kcache, Vcache, ctx_len, probe_keys, vis_idx, vis_cnt, b_cap: int,
                     O=None, active=None, ws: Workspace | None = None):
    lib = load_library()
    ws = ws or default_workspace()
    if O is None:
        O = torch.empty_like(q)
    if active is None:
        active = torch.empty(desc.batch, desc.n_q_heads, dtype=torch.uint8, device=q.device)
    buf = ws.get(CALL_SLIM_DECODE, desc)
    _check(lib.omni_slim_decode(C.byref(desc), _ptr(q), _ptr(Kcache), _ptr(Vcache), _ptr(ctx_len), _ptr(probe_keys),
                                _ptr(vis_idx), _ptr(vis_cnt), b_cap, _ptr(O), _ptr(active), _ptr(buf), buf.numel(),
                                _stream()))
    return O, active


def omni_slim_decode_prepare(desc: DecodeDesc, vis_idx, vis_cnt, b_cap: int, ws: Workspace | None = None):
    """Merge the per-head lists per KV group into the workspace the omni_slim_decode calls with static_lists get."""
    ws = ws or default_workspace()
    buf = ws.get(CALL_SLIM_DECODE, desc)
    _check(load_library().omni_slim_decode_prepare(C.byref(desc), _ptr(vis_idx), _ptr(vis_cnt), b_cap, _ptr(buf),
                                                   buf.numel(), _stream()))


def block_level_desc(desc: LayerDesc, block: int) -> LayerDesc:
    """Descriptor of the block-level score arrays: one "token" per block, all of them "visual"."""
    nb = (desc.n_tokens + block - 1) // block
    d = LayerDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim, d.n_tokens = desc.batch, desc.n_q_heads, desc.n_kv_heads, desc.head_dim, nb
    d.vis_begin, d.vis_end, d.sink_index, d.causal, d.dtype = 0, nb, 0, desc.causal, desc.dtype
    d.softmax_scale = desc.softmax_scale
    D = desc.head_dim
    d.q_stride = (C.c_int64 * 3)(desc.n_q_heads * nb * D, nb * D, D)
    d.kv_stride = (C.c_int64 * 3)(desc.n_kv_heads * nb * D, nb * D, D)
    return d


def omni_block_scores(desc: LayerDesc, Q, K, block: int, ws: Workspace | None = None):
    """Block-level accumulated key scores [B, Hq, n_blocks] f32, summing to n_blocks per head."""
    lib = load_library()
    ws = ws or default_workspace()
    nb = (desc.n_tokens + block - 1) // block
    out = torch.empty(desc.batch, desc.n_q_heads, nb, dtype=torch.float32, device=Q.device)
    buf = ws.get(CALL_BLOCK_SCORES, desc, block)
    _check(lib.omni_block_scores(C.byref(desc), _ptr(Q), _ptr(K), block, _ptr(out), _ptr(buf), buf.numel(), _stream()))
    return out


def omni_expand_blocks(desc: LayerDesc, blk_idx, blk_budget, block: int, kv_idx=None, budget=None):
    """(kv_idx [B,Hq,blk_cap*block] i32, budget [B] i32): token lists of the selected key blocks."""
    lib = load_library()
    blk_cap = blk_idx.shape[-1]
    b_cap = blk_cap * block if kv_idx is None else kv_idx.shape[-1]
    if kv_idx is None:
        kv_idx = torch.empty(desc.batch, desc.n_q_heads, b_cap, dtype=torch.int32, device=blk_idx.device)
    if budget is None:
        budget = torch.empty(desc.batch, dtype=torch.int32, device=blk_idx.device)
    _check(lib.omni_expand_blocks(C.byref(desc), _ptr(blk_idx), _ptr(blk_budget), blk_cap, block, _ptr(kv_idx),
                                  _ptr(budget), b_cap, _stream()))
    return kv_idx, budget


def omni_block_attn_fwd(desc: LayerDesc, Q, K, V, q_idx, q_cnt, blk_idx, blk_budget, block: int, O=None, lse=None,
                        ws: Workspace | None = None):
    """Sparse forward pass on block lists blk_idx [B,Hq,blk_cap] without a gathered K/V copy (bf16, block % 64 == 0)."""
    lib = load_library()
    ws = ws or default_workspace()
    blk_cap = blk_idx.shape[-1]
    if O is None:
        O = torch.empty_like(Q)
    if lse is None:
        lse = torch.empty(desc.batch, desc.n_q_heads, desc.n_tokens, dtype=torch.float32, device=Q.device)
    buf = ws.get(CALL_BLOCK_ATTN_FWD, desc, blk_cap * block)
    _check(lib.omni_block_attn_fwd(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(q_idx), _ptr(q_cnt), _ptr(blk_idx),
                                   _ptr(blk_budget), blk_cap, block, _ptr(O), _ptr(lse), _ptr(buf), buf.numel(),
                                   _stream()))
    return O, lse


def omni_block_attn_bwd(desc: LayerDesc, Q, K, V, O, dO, lse, q_idx, q_cnt, blk_idx, blk_budget, block: int,
                        dQ=None, dK=None, dV=None, ws: Workspace | None = None):
    """Gradients of omni_block_attn_fwd on the same block lists, again without a gathered K/V copy."""
    lib = load_library()
    ws = ws or default_workspace()
    blk_cap = blk_idx.shape[-1]
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    buf = ws.get(CALL_BLOCK_ATTN_BWD, desc, blk_cap * block)
    _check(lib.omni_block_attn_bwd(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(lse), _ptr(q_idx),
                                   _ptr(q_cnt), _ptr(blk_idx), _ptr(blk_budget), blk_cap, block, _ptr(dQ), _ptr(dK),
                                   _ptr(dV), _ptr(buf), buf.numel(), _stream()))
    return dQ, dK, dV


def omni_group_subset(desc: LayerDesc, kv_idx, budget, b_cap: int, u_cap: int | None = None,
                      ws: Workspace | None = None, _per_head: bool = False):
    """(grp_idx [B,Hkv,u_cap] i32, grp_mask [B,Hkv,u_cap] i32 holding the u32 bits, grp_cnt [B,Hkv] i32)."""
    lib = load_library()
    _budget_shape_ok(desc, budget, _per_head)
    ws = ws or default_workspace()
    if u_cap is None:
        u_cap = desc.vis_end - desc.vis_begin
    dev = kv_idx.device
    grp_idx = torch.empty(desc.batch, desc.n_kv_heads, u_cap, dtype=torch.int32, device=dev)
    grp_mask = torch.empty(desc.batch, desc.n_kv_heads, u_cap, dtype=torch.int32, device=dev)
    grp_cnt = torch.empty(desc.batch, desc.n_kv_heads, dtype=torch.int32, device=dev)
    buf = ws.get(CALL_GROUP_SUBSET, desc)
    fn = lib.omni_group_subset_per_head if _per_head else lib.omni_group_subset
    _check(fn(C.byref(desc), _ptr(kv_idx), _ptr(budget), b_cap, _ptr(grp_idx), _ptr(grp_mask), _ptr(grp_cnt), u_cap,
              _ptr(buf), buf.numel(), _stream()))
    return grp_idx, grp_mask, grp_cnt


def omni_group_subset_per_head(desc: LayerDesc, kv_idx, budget, b_cap: int, u_cap: int | None = None,
                               ws: Workspace | None = None):
    return omni_group_subset(desc, kv_idx, budget, b_cap, u_cap, ws, _per_head=True)


def omni_slim_decode_grouped(desc: DecodeDesc, q, Kcache, Vcache, ctx_len, probe_keys, grp_idx, grp_mask, grp_cnt,
                             O=None, active=None, ws: Workspace | None = None):
    lib = load_library()
    ws = ws or default_workspace()
    if O is None:
        O = torch.empty_like(q)
    if active is None:
        active = torch.empty(desc.batch, desc.n_q_heads, dtype=torch.uint8, device=q.device)
    buf = ws.get(CALL_SLIM_DECODE, desc)
    _check(lib.omni_slim_decode_grouped(C.byref(desc), _ptr(q), _ptr(Kcache), _ptr(Vcache), _ptr(ctx_len),
                                        _ptr(probe_keys), _ptr(grp_idx), _ptr(grp_mask), _ptr(grp_cnt),
                                        grp_idx.shape[-1], _ptr(O), _ptr(active), _ptr(buf), buf.numel(), _stream()))
    return O, active


def omni_slim_decode_grouped_static(desc: DecodeDesc, q, Kcache, Vcache, ctx_len, probe_keys, grp_idx, grp_mask, grp_cnt,
                                    O, active):
    """The grouped decode step on the library's built-in scratch buffer: no workspace, and O / active must be given
    (nothing is allocated on this path)."""
    lib = load_library()
    _check(lib.omni_slim_decode_grouped_static(C.byref(desc), _ptr(q), _ptr(Kcache), _ptr(Vcache), _ptr(ctx_len),
                                               _ptr(probe_keys), _ptr(grp_idx), _ptr(grp_mask), _ptr(grp_cnt),
                                               grp_idx.shape[-1], _ptr(O), _ptr(active), _stream()))
    return O, active


def omni_static_scratch_bytes() -> int:
    return int(load_library().omni_static_scratch_bytes())


def omni_compact_cache(desc: DecodeDesc, Kcache, Vcache, grp_idx, grp_cnt, Kcomp=None, Vcomp=None):
    lib = load_library()
    u_cap = grp_idx.shape[-1]
    shape = (desc.batch, desc.n_kv_heads, u_cap, desc.head_dim)
    if Kcomp is None:
        Kcomp = torch.zeros(shape, dtype=Kcache.dtype, device=Kcache.device)
    if Vcomp is None:
        Vcomp = torch.zeros(shape, dtype=Vcache.dtype, device=Vcache.device)
    _check(lib.omni_compact_cache(C.byref(desc), _ptr(Kcache), _ptr(Vcache), _ptr(grp_idx), _ptr(grp_cnt), u_cap,
                                  _ptr(Kcomp), _ptr(Vcomp), _stream()))
    return Kcomp, Vcomp


def omni_slim_decode_compact(desc: DecodeDesc, q, Kcache, Vcache, ctx_len, probe_keys, Kcomp, Vcomp, grp_idx, grp_mask,
                             grp_cnt, O=None, active=None, ws: Workspace | None = None):
    lib = load_library()
    ws = ws or default_workspace()
    if O is None:
        O = torch.empty_like(q)
    if active is None:
        active = torch.empty(desc.batch, desc.n_q_heads, dtype=torch.uint8, device=q.device)
    if tuple(Kcomp.shape) != (desc.batch, desc.n_kv_heads, grp_idx.shape[-1], desc.head_dim) or not Kcomp.is_contiguous():
        raise ValueError("Kcomp / Vcomp must be contiguous [batch, n_kv_heads, u_cap, head_dim]")
    buf = ws.get(CALL_SLIM_DECODE, desc)
    _check(lib.omni_slim_decode_compact(C.byref(desc), _ptr(q), _ptr(Kcache), _ptr(Vcache), _ptr(ctx_len),
                                        _ptr(probe_keys), _ptr(Kcomp), _ptr(Vcomp), _ptr(grp_idx), _ptr(grp_mask),
                                        _ptr(grp_cnt), grp_idx.shape[-1], _ptr(O), _ptr(active), _ptr(buf), buf.numel(),
                                        _stream()))
    return O, active


def omni_compact_cache_paged(desc: DecodeDesc, Kcache, Vcache, grp_idx, grp_cnt, pool: PagePool):
    lib = load_library()
    if pool._keep[0].dtype != Kcache.dtype or pool._keep[0].shape[-1] != desc.head_dim:
        raise ValueError("pool dtype / head_dim differ from the cache's")
    _check(lib.omni_compact_cache_paged(C.byref(desc), _ptr(Kcache), _ptr(Vcache), _ptr(grp_idx), _ptr(grp_cnt),
                                        grp_idx.shape[-1], C.byref(pool), _stream()))


def omni_slim_decode_paged(desc: DecodeDesc, q, Kcache, Vcache, ctx_len, probe_keys, pool: PagePool, grp_idx, grp_mask,
                           grp_cnt, O=None, active=None, ws: Workspace | None = None):
    lib = load_library()
    ws = ws or default_workspace()
    if O is None:
        O = torch.empty_like(q)
    if active is None:
        active = torch.empty(desc.batch, desc.n_q_heads, dtype=torch.uint8, device=q.device)
    if pool._keep[0].dtype != q.dtype or pool._keep[0].shape[-1] != desc.head_dim:
        raise ValueError("pool dtype / head_dim differ from the query's")
    buf = ws.get(CALL_SLIM_DECODE, desc)
    _check(lib.omni_slim_decode_paged(C.byref(desc), _ptr(q), _ptr(Kcache), _ptr(Vcache), _ptr(ctx_len),
                                      _ptr(probe_keys), C.byref(pool), _ptr(grp_idx), _ptr(grp_mask), _ptr(grp_cnt),
                                      grp_idx.shape[-1], _ptr(O), _ptr(active), _ptr(buf), buf.numel(), _stream()))
    return O, active


def omni_dense_decode(desc: DecodeDesc, q, Kcache, Vcache, ctx_len, O=None, ws: Workspace | None = None):
    lib = load_library()
    ws = ws or default_workspace()
    if O is None:
        O = torch.empty_like(q)
    buf = ws.get(CALL_DENSE_DECODE, desc)
    _check(lib.omni_dense_decode(C.byref(desc), _ptr(q), _ptr(Kcache), _ptr(Vcache), _ptr(ctx_len), _ptr(O), _ptr(buf),
                                 buf.numel(), _stream()))
    return O
