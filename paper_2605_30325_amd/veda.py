"""ctypes binding of libveda.so: argument marshalling only.

Every function below maps one-to-one onto the C entry point of the same name in
include/veda.h and does nothing but turn torch tensors into pointers, sizes and the current
HIP stream.  PyTorch provides device memory and streams; all arithmetic runs in the HIP
kernels.  There is no fallback: if the library is missing or a call fails, this raises.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path
from typing import Optional, Sequence, Tuple

import numpy as np
import torch

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libveda.so"

VEDA_OK, VEDA_ERR_INVALID_ARG, VEDA_ERR_UNSUPPORTED, VEDA_ERR_WORKSPACE, VEDA_ERR_HIP = range(5)
VEDA_F32, VEDA_BF16 = 0, 1
VEDA_ACT_IDENTITY, VEDA_ACT_RELU = 0, 1
VEDA_TOKEN_MAJOR, VEDA_CHANNEL_MAJOR = 0, 1
VEDA_OPT_EXACT_LOGIT_SCALE = 0
VEDA_OPT_ATTN_LIST_WALK = 1
VEDA_OPT_FP32_CHAIN_UNIT = 2
VEDA_CHAINS_MATRIX, VEDA_CHAINS_VECTOR = 1, 2

EXPORTS = (
    "veda_plan_create", "veda_plan_destroy", "veda_plan_set_option", "veda_plan_chain_unit", "veda_plan_tiles", "veda_plan_tile_offset",
    "veda_plan_score_offset", "veda_plan_total_tiles", "veda_plan_score_elems",
    "veda_plan_workspace_bytes", "veda_plan_workspace_layout", "veda_tile_layout", "veda_tile_score", "veda_tile_layout_stats",
    "veda_tile_score_stats", "veda_tile_score_closed_form", "veda_tile_select", "veda_plan_fused_workspace_bytes",
    "veda_tile_score_select", "veda_tile_score_select_stats", "veda_tile_score_select_stats_noalloc",
    "veda_sparse_attn_fwd", "veda_sparse_attn_fwd_q_tokens",
    "veda_sparse_attn_fwd_qk_tokens", "veda_tile_heatmap",
    "veda_tile_recall", "veda_output_sqerr", "veda_status_string", "veda_last_error",
)


class VedaError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        super().__init__(f"{where}: status {status}" + (f" ({detail})" if detail else ""))


class veda_problem(C.Structure):
    _fields_ = [("batch", C.c_int32), ("heads", C.c_int32), ("head_dim", C.c_int32),
                ("T", C.c_int32), ("H", C.c_int32), ("W", C.c_int32), ("tile_tokens", C.c_int32),
                ("tile_shape", C.POINTER(C.c_int32)), ("dtype", C.c_int)]


class veda_strides(C.Structure):
    _fields_ = [("b", C.c_int64), ("h", C.c_int64), ("n", C.c_int64)]


class veda_mlp(C.Structure):
    _fields_ = [("in_dim", C.c_int32), ("hidden", C.c_int32), ("out_dim", C.c_int32), ("act", C.c_int),
                ("w1", C.c_void_p), ("b1", C.c_void_p), ("w2", C.c_void_p), ("b2", C.c_void_p)]


class veda_workspace_layout(C.Structure):
    _fields_ = [("stats_q", C.c_int64), ("stats_k", C.c_int64), ("latent_q", C.c_int64), ("latent_k", C.c_int64)]


_lib = None


def load():
    """Load libveda.so (built in-tree by paper_2605_30325_amd.build).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not LIB_PATH.exists():
        raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_2605_30325_amd.build`")
    L = C.CDLL(str(LIB_PATH))
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    L.veda_plan_create.argtypes = [C.POINTER(veda_problem), C.POINTER(vp)]
    L.veda_plan_create.restype = C.c_int
    L.veda_plan_destroy.argtypes = [vp]
    L.veda_plan_destroy.restype = None
    L.veda_plan_set_option.argtypes = [vp, C.c_int, i32]
    L.veda_plan_set_option.restype = C.c_int
    L.veda_plan_chain_unit.argtypes = [vp]
    L.veda_plan_chain_unit.restype = i32
    L.veda_plan_tiles.argtypes = [vp, i32]
    L.veda_plan_tiles.restype = i32
    for name in ("veda_plan_tile_offset", "veda_plan_score_offset"):
        getattr(L, name).argtypes = [vp, i32]
        getattr(L, name).restype = i64
    for name in ("veda_plan_total_tiles", "veda_plan_score_elems"):
        getattr(L, name).argtypes = [vp]
        getattr(L, name).restype = i64
    L.veda_plan_workspace_bytes.argtypes = [vp, C.POINTER(veda_mlp), C.POINTER(veda_mlp)]
    L.veda_plan_workspace_bytes.restype = C.c_size_t
    L.veda_plan_workspace_layout.argtypes = [vp, C.POINTER(veda_mlp), C.POINTER(veda_mlp), C.POINTER(veda_workspace_layout)]
    L.veda_plan_workspace_layout.restype = C.c_int
    L.veda_tile_layout.argtypes = [vp, vp, veda_strides, C.c_int, vp, vp, vp, vp]
    L.veda_tile_layout.restype = C.c_int
    L.veda_tile_score.argtypes = [vp, vp, vp, vp, C.POINTER(veda_mlp), C.POINTER(veda_mlp), C.c_float,
                                  vp, vp, C.c_size_t, vp]
    L.veda_tile_score.restype = C.c_int
    L.veda_tile_layout_stats.argtypes = [vp, vp, veda_strides, vp, vp, vp, vp, vp]
    L.veda_tile_layout_stats.restype = C.c_int
    L.veda_tile_score_stats.argtypes = [vp, vp, vp, C.POINTER(veda_mlp), C.POINTER(veda_mlp), C.c_float, vp, vp,
                                        C.c_size_t, vp]
    L.veda_tile_score_stats.restype = C.c_int
    L.veda_tile_score_closed_form.argtypes = [vp, vp, vp, vp, C.c_float, vp, vp, C.c_size_t, vp]
    L.veda_tile_score_closed_form.restype = C.c_int
    L.veda_tile_select.argtypes = [vp, vp, C.POINTER(i32), vp, vp, vp]
    L.veda_tile_select.restype = C.c_int
    L.veda_plan_fused_workspace_bytes.argtypes = [vp, C.POINTER(veda_mlp), C.POINTER(veda_mlp)]
    L.veda_plan_fused_workspace_bytes.restype = C.c_size_t
    L.veda_tile_score_select.argtypes = [vp, vp, vp, vp, C.POINTER(veda_mlp), C.POINTER(veda_mlp), C.c_float,
                                         C.POINTER(i32), vp, vp, vp, C.c_size_t, vp]
    L.veda_tile_score_select.restype = C.c_int
    L.veda_tile_score_select_stats.argtypes = [vp, vp, vp, C.POINTER(veda_mlp), C.POINTER(veda_mlp), C.c_float,
                                               C.POINTER(i32), vp, vp, vp, C.c_size_t, vp]
    L.veda_tile_score_select_stats.restype = C.c_int
    L.veda_tile_score_select_stats_noalloc.argtypes = [vp, vp, vp, C.POINTER(veda_mlp), C.POINTER(veda_mlp), C.c_float,
                                                       C.POINTER(i32), vp, vp, vp]
    L.veda_tile_score_select_stats_noalloc.restype = C.c_int
    L.veda_sparse_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, C.c_float, vp, veda_strides, vp, vp]
    L.veda_sparse_attn_fwd.restype = C.c_int
    L.veda_sparse_attn_fwd_q_tokens.argtypes = [vp, vp, veda_strides, vp, vp, vp, vp, vp, C.c_float, vp, veda_strides,
                                                vp, vp]
    L.veda_sparse_attn_fwd_q_tokens.restype = C.c_int
    L.veda_sparse_attn_fwd_qk_tokens.argtypes = [vp, vp, veda_strides, vp, veda_strides, vp, vp, vp, vp, C.c_float, vp,
                                                 veda_strides, vp, vp]
    L.veda_sparse_attn_fwd_qk_tokens.restype = C.c_int
    L.veda_tile_heatmap.argtypes = [vp, vp, vp, vp, C.c_float, vp, i64, vp, vp]
    L.veda_tile_heatmap.restype = C.c_int
    L.veda_tile_recall.argtypes = [vp, C.POINTER(i32), vp, vp, vp, vp, C.c_size_t, vp]
    L.veda_tile_recall.restype = C.c_int
    L.veda_output_sqerr.argtypes = [vp, vp, veda_strides, vp, veda_strides, vp, vp, C.c_size_t, vp]
    L.veda_output_sqerr.restype = C.c_int
    L.veda_status_string.argtypes = [C.c_int]
    L.veda_status_string.restype = C.c_char_p
    L.veda_last_error.argtypes = []
    L.veda_last_error.restype = C.c_char_p
    _lib = L
    return L


def _check(status: int, where: str):
    if status != VEDA_OK:
        L = load()
        detail = L.veda_status_string(status).decode()
        if status == VEDA_ERR_HIP:
            detail += ": " + L.veda_last_error().decode()
        raise VedaError(status, where, detail)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _strides(t: torch.Tensor) -> veda_strides:
    assert t.dim() == 4 and t.stride(3) == 1, "expected [batch, heads, N, d] with unit channel stride"
    return veda_strides(t.stride(0), t.stride(1), t.stride(2))


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return VEDA_F32
    if dt == torch.bfloat16:
        return VEDA_BF16
    raise TypeError(f"unsupported dtype {dt}")


class Mlp:
    """Device-resident projection weights as the veda_mlp struct expects them."""

    def __init__(self, w1, b1, w2=None, b2=None, relu: bool = True, device="cuda"):
        def dev(a):
            return None if a is None else torch.as_tensor(np.ascontiguousarray(a, np.float32)).to(device).contiguous()
        self.w1, self.b1, self.w2, self.b2 = dev(w1), dev(b1), dev(w2), dev(b2)
        self.in_dim = int(self.w1.shape[1])
        self.hidden = 0 if self.w2 is None else int(self.w1.shape[2])
        self.out_dim = int(self.w1.shape[2] if self.w2 is None else self.w2.shape[2])
        self.act = VEDA_ACT_RELU if relu else VEDA_ACT_IDENTITY

    def struct(self) -> veda_mlp:
        return veda_mlp(self.in_dim, self.hidden, self.out_dim, self.act,
                        _ptr(self.w1), _ptr(self.b1), _ptr(self.w2), _ptr(self.b2))


class Plan:
    """veda_plan handle plus the sizes callers need to allocate buffers."""

    def __init__(self, batch: int, heads: int, head_dim: int, grid: Sequence[int],
                 tile_shape: np.ndarray, dtype: torch.dtype, tile_tokens: int = 64):
        L = load()
        self._shape = np.ascontiguousarray(tile_shape, np.int32).reshape(-1)
        if self._shape.size != 3 * heads:
            raise VedaError(VEDA_ERR_INVALID_ARG, "Plan", "tile_shape must be [heads, 3]")
        prob = veda_problem(batch, heads, head_dim, int(grid[0]), int(grid[1]), int(grid[2]), tile_tokens,
                            self._shape.ctypes.data_as(C.POINTER(C.c_int32)), _dtype_code(dtype))
        h = C.c_void_p()
        self.handle = None
        _check(L.veda_plan_create(C.byref(prob), C.byref(h)), "veda_plan_create")
        self.handle = h
        self.batch, self.heads, self.head_dim, self.grid, self.dtype = batch, heads, head_dim, tuple(grid), dtype
        self.tile_tokens = int(tile_tokens)        # 64, or 128 (two 64-slot halves per tile)
        self.mask_words = self.tile_tokens // 64   # u64 words of valid_mask per tile
        self.tokens = int(grid[0]) * int(grid[1]) * int(grid[2])
        self.tiles = [int(L.veda_plan_tiles(h, i)) for i in range(heads)]
        self.tile_offset = [int(L.veda_plan_tile_offset(h, i)) for i in range(heads)]
        self.score_offset = [int(L.veda_plan_score_offset(h, i)) for i in range(heads)]
        self.total_tiles = int(L.veda_plan_total_tiles(h))
        self.score_elems = int(L.veda_plan_score_elems(h))

    def set_option(self, option: int, value: int):
        _check(load().veda_plan_set_option(self.handle, option, int(value)), "veda_plan_set_option")

    def chain_unit(self) -> int:
        """VEDA_CHAINS_MATRIX or VEDA_CHAINS_VECTOR: where the plan's next stage-2 call runs its fp32 chains."""
        return int(load().veda_plan_chain_unit(self.handle))

    def workspace_bytes(self, phi_q: Mlp, phi_k: Mlp) -> int:
        return int(load().veda_plan_workspace_bytes(self.handle, C.byref(phi_q.struct()), C.byref(phi_k.struct())))

    def workspace_layout(self, phi_q: Mlp, phi_k: Mlp) -> veda_workspace_layout:
        """Float offsets of the intermediates veda_tile_score leaves in its workspace."""
        lay = veda_workspace_layout()
        _check(load().veda_plan_workspace_layout(self.handle, C.byref(phi_q.struct()), C.byref(phi_k.struct()),
                                                 C.byref(lay)), "veda_plan_workspace_layout")
        return lay

    def close(self):
        if self.handle is not None:
            load().veda_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def veda_tile_layout(plan: Plan, x: torch.Tensor, order: int = VEDA_TOKEN_MAJOR,
                     x_tiled: Optional[torch.Tensor] = None, valid_mask: Optional[torch.Tensor] = None,
                     valid_cnt: Optional[torch.Tensor] = None, want_mask: bool = True):
    """Stage 1.  Returns (x_tiled [batch, total_tiles, tile_tokens*d], valid_mask i64-as-u64
    [total_tiles * tile_tokens/64], valid_cnt i32 [total_tiles])."""
    dev = x.device
    if x_tiled is None:
        x_tiled = torch.empty((plan.batch, plan.total_tiles, plan.tile_tokens * plan.head_dim), dtype=x.dtype,
                              device=dev)
    if want_mask and valid_mask is None:
        valid_mask = torch.empty(plan.total_tiles * plan.mask_words, dtype=torch.int64, device=dev)
    if want_mask and valid_cnt is None:
        valid_cnt = torch.empty(plan.total_tiles, dtype=torch.int32, device=dev)
    _check(load().veda_tile_layout(plan.handle, _ptr(x), _strides(x), order, _ptr(x_tiled), _ptr(valid_mask),
                                   _ptr(valid_cnt), _stream()), "veda_tile_layout")
    return x_tiled, valid_mask, valid_cnt


def veda_tile_score(plan: Plan, q_tiled, k_tiled, valid_mask, phi_q: Mlp, phi_k: Mlp, scale: float,
                    scores: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """Stage 2.  Returns (scores fp32 [batch, score_elems], workspace)."""
    dev = q_tiled.device
    if scores is None:
        scores = torch.empty((plan.batch, plan.score_elems), dtype=torch.float32, device=dev)
    need = plan.workspace_bytes(phi_q, phi_k)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    sq, sk = phi_q.struct(), phi_k.struct()
    _check(load().veda_tile_score(plan.handle, _ptr(q_tiled), _ptr(k_tiled), _ptr(valid_mask), C.byref(sq),
                                  C.byref(sk), C.c_float(scale), _ptr(scores), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream()), "veda_tile_score")
    return scores, workspace


def veda_tile_layout_stats(plan: Plan, x: torch.Tensor, x_tiled: Optional[torch.Tensor] = None,
                           valid_mask: Optional[torch.Tensor] = None, valid_cnt: Optional[torch.Tensor] = None,
                           stats: Optional[torch.Tensor] = None, want_mask: bool = True, want_tiles: bool = True):
    """Stage 1 (token-major) with the TripPool descriptors taken during the gather.
    Returns (x_tiled, valid_mask, valid_cnt, stats fp32 [batch, total_tiles, 3*d]).
    want_tiles=False: descriptors (and masks) only, x_tiled is returned as None."""
    dev = x.device
    if x_tiled is None and want_tiles:
        x_tiled = torch.empty((plan.batch, plan.total_tiles, plan.tile_tokens * plan.head_dim), dtype=x.dtype,
                              device=dev)
    if want_mask and valid_mask is None:
        valid_mask = torch.empty(plan.total_tiles * plan.mask_words, dtype=torch.int64, device=dev)
    if want_mask and valid_cnt is None:
        valid_cnt = torch.empty(plan.total_tiles, dtype=torch.int32, device=dev)
    if stats is None:
        stats = torch.empty((plan.batch, plan.total_tiles, 3 * plan.head_dim), dtype=torch.float32, device=dev)
    _check(load().veda_tile_layout_stats(plan.handle, _ptr(x), _strides(x), _ptr(x_tiled), _ptr(valid_mask),
                                         _ptr(valid_cnt), _ptr(stats), _stream()), "veda_tile_layout_stats")
    return x_tiled, valid_mask, valid_cnt, stats


def veda_tile_score_stats(plan: Plan, stats_q, stats_k, phi_q: Mlp, phi_k: Mlp, scale: float,
                          scores: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """Stage 2 from descriptors.  Returns (scores fp32 [batch, score_elems], workspace holding the latents)."""
    dev = stats_q.device
    if scores is None:
        scores = torch.empty((plan.batch, plan.score_elems), dtype=torch.float32, device=dev)
    sq, sk = phi_q.struct(), phi_k.struct()
    if workspace is None:   # room for the hidden layers too: the faster route of the projections
        need = int(load().veda_plan_workspace_bytes(plan.handle, C.byref(sq), C.byref(sk)))
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    _check(load().veda_tile_score_stats(plan.handle, _ptr(stats_q), _ptr(stats_k), C.byref(sq), C.byref(sk),
                                        C.c_float(scale), _ptr(scores), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream()),
           "veda_tile_score_stats")
    return scores, workspace


def veda_tile_score_closed_form(plan: Plan, q_tiled, k_tiled, valid_mask, lam: float,
                                scores: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """Stage 2 with the weight-free scorer.  Returns (scores fp32 [batch, score_elems], workspace)."""
    dev = q_tiled.device
    if scores is None:
        scores = torch.empty((plan.batch, plan.score_elems), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(plan.batch * plan.total_tiles * 10 * plan.head_dim * 4, dtype=torch.uint8, device=dev)
    _check(load().veda_tile_score_closed_form(plan.handle, _ptr(q_tiled), _ptr(k_tiled), _ptr(valid_mask),
                                              C.c_float(lam), _ptr(scores), _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _stream()),
           "veda_tile_score_closed_form")
    return scores, workspace


def veda_tile_select(plan: Plan, scores, k_per_head: Sequence[int], row_ptr: Optional[torch.Tensor] = None,
                     col_idx: Optional[torch.Tensor] = None):
    """Stage 3.  Returns (row_ptr i32 [batch*total_tiles+1], col_idx i32 [batch*nnz])."""
    k = np.ascontiguousarray(k_per_head, np.int32)
    if k.size != plan.heads:
        raise VedaError(VEDA_ERR_INVALID_ARG, "veda_tile_select", "k_per_head must have one entry per head")
    nnz = int(sum(int(n) * int(kk) for n, kk in zip(plan.tiles, k)))
    dev = scores.device
    if row_ptr is None:
        row_ptr = torch.empty(plan.batch * plan.total_tiles + 1, dtype=torch.int32, device=dev)
    if col_idx is None:
        col_idx = torch.empty(max(1, plan.batch * max(nnz, 0)), dtype=torch.int32, device=dev)
    _check(load().veda_tile_select(plan.handle, _ptr(scores), k.ctypes.data_as(C.POINTER(C.c_int32)),
                                   _ptr(row_ptr), _ptr(col_idx), _stream()), "veda_tile_select")
    return row_ptr, col_idx


def veda_tile_score_select(plan: Plan, phi_q: Mlp, phi_k: Mlp, scale: float, k_per_head: Sequence[int],
                           q_tiled=None, k_tiled=None, valid_mask=None, stats_q=None, stats_k=None,
                           row_ptr: Optional[torch.Tensor] = None, col_idx: Optional[torch.Tensor] = None,
                           workspace: Optional[torch.Tensor] = None):
    """Stages 2 + 3 in one call, from the tiled Q, K (q_tiled, k_tiled, valid_mask) or from their
    descriptors (stats_q, stats_k).  Returns (row_ptr, col_idx, workspace)."""
    k = np.ascontiguousarray(k_per_head, np.int32)
    if k.size != plan.heads:
        raise VedaError(VEDA_ERR_INVALID_ARG, "veda_tile_score_select", "k_per_head must have one entry per head")
    from_stats = stats_q is not None
    dev = (stats_q if from_stats else q_tiled).device
    nnz = int(sum(int(n) * int(kk) for n, kk in zip(plan.tiles, k)))
    if row_ptr is None:
        row_ptr = torch.empty(plan.batch * plan.total_tiles + 1, dtype=torch.int32, device=dev)
    if col_idx is None:
        col_idx = torch.empty(max(1, plan.batch * max(nnz, 0)), dtype=torch.int32, device=dev)
    sq, sk = phi_q.struct(), phi_k.struct()
    if workspace is None:
        need = int(load().veda_plan_fused_workspace_bytes(plan.handle, C.byref(sq), C.byref(sk)))
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    kp = k.ctypes.data_as(C.POINTER(C.c_int32))
    nbytes = workspace.numel() * workspace.element_size()
    if from_stats:
        _check(load().veda_tile_score_select_stats(plan.handle, _ptr(stats_q), _ptr(stats_k), C.byref(sq), C.byref(sk),
                                                   C.c_float(scale), kp, _ptr(row_ptr), _ptr(col_idx), _ptr(workspace),
                                                   nbytes, _stream()), "veda_tile_score_select_stats")
    else:
        _check(load().veda_tile_score_select(plan.handle, _ptr(q_tiled), _ptr(k_tiled), _ptr(valid_mask), C.byref(sq),
                                             C.byref(sk), C.c_float(scale), kp, _ptr(row_ptr), _ptr(col_idx),
                                             _ptr(workspace), nbytes, _stream()), "veda_tile_score_select")
    return row_ptr, col_idx, workspace


NOALLOC_SCRATCH_BYTES = 128 << 20


def veda_tile_score_select_stats_noalloc(plan: Plan, phi_q: Mlp, phi_k: Mlp, scale: float, k_per_head: Sequence[int],
                                         stats_q: torch.Tensor, stats_k: torch.Tensor, row_ptr: torch.Tensor,
                                         col_idx: torch.Tensor):
    """Stages 2 + 3 from descriptors with the library's fixed scratch array: the caller passes every
    input and output, nothing is allocated here or in the library."""
    k = np.ascontiguousarray(k_per_head, np.int32)
    if k.size != plan.heads:
        raise VedaError(VEDA_ERR_INVALID_ARG, "veda_tile_score_select_stats_noalloc",
                        "k_per_head must have one entry per head")
    sq, sk = phi_q.struct(), phi_k.struct()
    status = load().veda_tile_score_select_stats_noalloc(
        plan.handle, _ptr(stats_q), _ptr(stats_k), C.byref(sq), C.byref(sk), C.c_float(scale),
        k.ctypes.data_as(C.POINTER(C.c_int32)), _ptr(row_ptr), _ptr(col_idx), _stream())
    if status == VEDA_ERR_WORKSPACE:
        raise VedaError(status, "veda_tile_score_select_stats_noalloc", load().veda_last_error().decode())
    _check(status, "veda_tile_score_select_stats_noalloc")
    return row_ptr, col_idx


def veda_sparse_attn_fwd(plan: Plan, q_tiled, k_tiled, v_tiled, valid_mask, row_ptr, col_idx,
                         softmax_scale: float, out: Optional[torch.Tensor] = None,
                         lse: Optional[torch.Tensor] = None, want_lse: bool = False,
                         q_tokens: Optional[torch.Tensor] = None, k_tokens: Optional[torch.Tensor] = None):
    """Stage 4.  Returns (out [batch, heads, N, d] in token order, lse or None).
    q_tokens (with q_tiled None): Q in token order [batch, heads, N, d], gathered by the kernel;
    k_tokens (with q_tokens, k_tiled None): K in token order as well."""
    dev = v_tiled.device
    if out is None:
        out = torch.empty((plan.batch, plan.heads, plan.tokens, plan.head_dim), dtype=plan.dtype, device=dev)
    if want_lse and lse is None:
        lse = torch.empty((plan.batch, plan.heads, plan.tokens), dtype=torch.float32, device=dev)
    if q_tokens is not None and k_tokens is not None and q_tiled is None and k_tiled is None:
        _check(load().veda_sparse_attn_fwd_qk_tokens(plan.handle, _ptr(q_tokens), _strides(q_tokens), _ptr(k_tokens),
                                                     _strides(k_tokens), _ptr(v_tiled), _ptr(valid_mask),
                                                     _ptr(row_ptr), _ptr(col_idx), C.c_float(softmax_scale), _ptr(out),
                                                     _strides(out), _ptr(lse), _stream()),
               "veda_sparse_attn_fwd_qk_tokens")
        return out, lse
    if q_tokens is not None and q_tiled is None:
        _check(load().veda_sparse_attn_fwd_q_tokens(plan.handle, _ptr(q_tokens), _strides(q_tokens), _ptr(k_tiled),
                                                    _ptr(v_tiled), _ptr(valid_mask), _ptr(row_ptr), _ptr(col_idx),
                                                    C.c_float(softmax_scale), _ptr(out), _strides(out), _ptr(lse),
                                                    _stream()), "veda_sparse_attn_fwd_q_tokens")
        return out, lse
    _check(load().veda_sparse_attn_fwd(plan.handle, _ptr(q_tiled), _ptr(k_tiled), _ptr(v_tiled),
                                       _ptr(valid_mask), _ptr(row_ptr), _ptr(col_idx), C.c_float(softmax_scale),
                                       _ptr(out), _strides(out), _ptr(lse), _stream()), "veda_sparse_attn_fwd")
    return out, lse


def veda_tile_heatmap(plan: Plan, q_tiled, k_tiled, valid_mask, softmax_scale: float,
                      query_tiles: Optional[torch.Tensor] = None, heat: Optional[torch.Tensor] = None):
    """Target tile scores of full attention: heat fp32 [batch, score_elems] (rows of unlisted query
    tiles are left as they were)."""
    dev = q_tiled.device
    if heat is None:
        heat = torch.zeros((plan.batch, plan.score_elems), dtype=torch.float32, device=dev)
    n_qt = 0 if query_tiles is None else int(query_tiles.numel())
    _check(load().veda_tile_heatmap(plan.handle, _ptr(q_tiled), _ptr(k_tiled), _ptr(valid_mask),
                                    C.c_float(softmax_scale), _ptr(query_tiles), n_qt, _ptr(heat), _stream()),
           "veda_tile_heatmap")
    return heat


def veda_tile_recall(plan: Plan, k_per_head: Sequence[int], col_idx_a, col_idx_b,
                     recall: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """Recall@k of selection a against selection b: fp32 [batch, heads]."""
    k = np.ascontiguousarray(k_per_head, np.int32)
    if k.size != plan.heads:
        raise VedaError(VEDA_ERR_INVALID_ARG, "veda_tile_recall", "k_per_head must have one entry per head")
    dev = col_idx_a.device
    if recall is None:
        recall = torch.empty((plan.batch, plan.heads), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(plan.batch * plan.heads, dtype=torch.int64, device=dev)
    _check(load().veda_tile_recall(plan.handle, k.ctypes.data_as(C.POINTER(C.c_int32)), _ptr(col_idx_a), _ptr(col_idx_b),
                                   _ptr(recall), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                   _stream()), "veda_tile_recall")
    return recall


def veda_output_sqerr(plan: Plan, a: torch.Tensor, b: torch.Tensor, err: Optional[torch.Tensor] = None,
                      workspace: Optional[torch.Tensor] = None):
    """Squared Frobenius distance of two [batch, heads, N, d] tensors per (batch, head): fp64 [batch, heads]."""
    dev = a.device
    if err is None:
        err = torch.empty((plan.batch, plan.heads), dtype=torch.float64, device=dev)
    if workspace is None:
        workspace = torch.empty(plan.batch * plan.heads * 64, dtype=torch.float64, device=dev)
    _check(load().veda_output_sqerr(plan.handle, _ptr(a), _strides(a), _ptr(b), _strides(b), _ptr(err),
                                    _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
           "veda_output_sqerr")
    return err


def veda_attention(plan: Plan, q, k, v, phi_q: Mlp, phi_k: Mlp, k_per_head, score_scale: float,
                   softmax_scale: float, buffers: Optional[dict] = None, fused: bool = False,
                   one_call: bool = False, from_tokens: bool = False):
    """The whole path in call order: layout x3 -> score -> select -> sparse attention.
    fused=True takes the descriptors during the Q and K gathers (veda_tile_layout_stats +
    veda_tile_score_stats); one_call=True runs stages 2 and 3 through veda_tile_score_select*,
    which never writes the score matrix; from_tokens=True (with fused, bf16) writes no
    tiled copy of Q and K: the gathers only take descriptors and masks, and the attention kernel
    gathers the rows of both from token order.  The results are bit-identical whichever way.
    `buffers` (optional dict) is filled on the first call and reused afterwards so that a
    steady-state step allocates nothing."""
    bufs = {} if buffers is None else buffers
    if from_tokens and not fused:
        raise ValueError("from_tokens needs fused=True (the descriptors must come from the gathers)")
    if fused:
        qt, vm, vc, zq = veda_tile_layout_stats(plan, q, bufs.get("qt"), bufs.get("vm"), bufs.get("vc"), bufs.get("zq"),
                                                want_tiles=not from_tokens)
        kt, _, _, zk = veda_tile_layout_stats(plan, k, bufs.get("kt"), stats=bufs.get("zk"), want_mask=False,
                                              want_tiles=not from_tokens)
        bufs.update(zq=zq, zk=zk)
    else:
        qt, vm, vc = veda_tile_layout(plan, q, VEDA_TOKEN_MAJOR, bufs.get("qt"), bufs.get("vm"), bufs.get("vc"))
        kt, _, _ = veda_tile_layout(plan, k, VEDA_TOKEN_MAJOR, bufs.get("kt"), want_mask=False)
    vt, _, _ = veda_tile_layout(plan, v, VEDA_CHANNEL_MAJOR, bufs.get("vt"), want_mask=False)
    if one_call:
        s = None
        if fused:
            rp, ci, ws = veda_tile_score_select(plan, phi_q, phi_k, score_scale, k_per_head, stats_q=zq, stats_k=zk,
                                                row_ptr=bufs.get("rp"), col_idx=bufs.get("ci"), workspace=bufs.get("ws"))
        else:
            rp, ci, ws = veda_tile_score_select(plan, phi_q, phi_k, score_scale, k_per_head, q_tiled=qt, k_tiled=kt,
                                                valid_mask=vm, row_ptr=bufs.get("rp"), col_idx=bufs.get("ci"),
                                                workspace=bufs.get("ws"))
    else:
        if fused:
            s, ws = veda_tile_score_stats(plan, zq, zk, phi_q, phi_k, score_scale, bufs.get("s"), bufs.get("ws"))
        else:
            s, ws = veda_tile_score(plan, qt, kt, vm, phi_q, phi_k, score_scale, bufs.get("s"), bufs.get("ws"))
        rp, ci = veda_tile_select(plan, s, k_per_head, bufs.get("rp"), bufs.get("ci"))
    out, _ = veda_sparse_attn_fwd(plan, qt, kt, vt, vm, rp, ci, softmax_scale, bufs.get("out"),
                                  q_tokens=q if from_tokens else None, k_tokens=k if from_tokens else None)
    bufs.update(qt=qt, kt=kt, vt=vt, vm=vm, vc=vc, s=s, ws=ws, rp=rp, ci=ci, out=out)
    return out, bufs
