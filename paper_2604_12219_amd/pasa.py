"""ctypes binding of the C ABI in ``include/pasa.h``: argument marshalling only.

Tensors are torch tensors on the GPU; the binding passes their device pointers, the current HIP
stream and sizes straight through.  Every step of the forward runs in the HIP kernels.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpasa_hip.so")
_lib = None

EXPORTS = ("pasa_strerror", "pasa_topk_count", "pasa_num_blocks", "pasa_mask_words", "pasa_score_workspace_bytes",
           "pasa_attn_workspace_bytes", "pasa_block_score", "pasa_block_score_with_stats", "pasa_route", "pasa_route_gumbel", "pasa_kv_stats", "pasa_key_prior", "pasa_sparse_attn_fwd",
           "pasa_sparse_attn_fwd_prepared", "pasa_sparse_attn_fwd_static", "pasa_forward", "pasa_forward_workspace_bytes", "pasa_check_selection", "pasa_attn_dense_ref", "pasa_l1_workspace_bytes", "pasa_l1_distance",
           "pasa_budget_schedule", "pasa_mfma_probe")


class PasaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load_library().pasa_strerror(status).decode()
        super().__init__(f"{where}: {msg} (status {status})")


class _CShape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("n", ctypes.c_int32), ("d", ctypes.c_int32),
                ("block", ctypes.c_int32), ("group", ctypes.c_int32),
                ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64),
                ("scale", ctypes.c_float), ("kv_slices", ctypes.c_int32)]


@dataclass
class Shape:
    B: int
    H: int
    n: int
    d: int
    block: int = 64
    group: int = 32
    stride_b: int = 0
    stride_h: int = 0
    stride_n: int = 0
    scale: float = 0.0
    kv_slices: int = 0

    @staticmethod
    def of(x: torch.Tensor, block: int = 64, group: int = 32, scale: float = 0.0, kv_slices: int = 0) -> "Shape":
        if x.dim() != 4 or x.stride(3) != 1:
            raise ValueError("expected a [B, H, n, d] tensor with contiguous last dimension")
        B, H, n, d = x.shape
        return Shape(B, H, n, d, block, group, x.stride(0), x.stride(1), x.stride(2), scale, kv_slices)

    def c(self) -> _CShape:
        return _CShape(self.B, self.H, self.n, self.d, self.block, self.group, self.stride_b, self.stride_h,
                       self.stride_n, self.scale, self.kv_slices)


def lib_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libpasa_hip.so; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2604_12219_amd.build` "
                               "(hipcc, gfx950). There is no CPU fallback.")
        L = ctypes.CDLL(_LIB_PATH)
        vp, sp = ctypes.c_void_p, ctypes.POINTER(_CShape)
        L.pasa_strerror.restype = ctypes.c_char_p
        L.pasa_strerror.argtypes = [ctypes.c_int]
        L.pasa_topk_count.restype = ctypes.c_int32
        L.pasa_topk_count.argtypes = [ctypes.c_int32, ctypes.c_double]
        L.pasa_num_blocks.restype = ctypes.c_int32
        L.pasa_num_blocks.argtypes = [sp]
        L.pasa_mask_words.restype = ctypes.c_int32
        L.pasa_mask_words.argtypes = [ctypes.c_int32]
        L.pasa_score_workspace_bytes.restype = ctypes.c_size_t
        L.pasa_score_workspace_bytes.argtypes = [sp]
        L.pasa_attn_workspace_bytes.restype = ctypes.c_size_t
        L.pasa_attn_workspace_bytes.argtypes = [sp]
        L.pasa_block_score.restype = ctypes.c_int
        L.pasa_block_score.argtypes = [vp, vp, sp, vp, vp, vp, ctypes.c_size_t, vp]
        L.pasa_block_score_with_stats.restype = ctypes.c_int
        L.pasa_block_score_with_stats.argtypes = [vp, sp, vp, vp, vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
        L.pasa_route.restype = ctypes.c_int
        L.pasa_route.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_uint64, ctypes.c_float,
                                 vp, vp, vp]
        L.pasa_route_gumbel.restype = ctypes.c_int
        L.pasa_route_gumbel.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_uint64, ctypes.c_float,
                                 vp, vp, vp]
        L.pasa_mfma_probe.restype = ctypes.c_int
        L.pasa_mfma_probe.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.pasa_sparse_attn_fwd.restype = ctypes.c_int
        L.pasa_sparse_attn_fwd.argtypes = [vp, vp, vp, sp, vp, vp, ctypes.c_int32, vp, vp, vp, ctypes.c_size_t, vp]
        L.pasa_sparse_attn_fwd_prepared.restype = ctypes.c_int
        L.pasa_sparse_attn_fwd_prepared.argtypes = L.pasa_sparse_attn_fwd.argtypes
        L.pasa_sparse_attn_fwd_static.restype = ctypes.c_int
        L.pasa_sparse_attn_fwd_static.argtypes = [vp, vp, vp, sp, vp, vp, ctypes.c_int32, vp, vp, vp]
        L.pasa_forward_workspace_bytes.restype = ctypes.c_size_t
        L.pasa_forward_workspace_bytes.argtypes = [sp, ctypes.c_double]
        L.pasa_forward.restype = ctypes.c_int
        L.pasa_forward.argtypes = [vp, vp, vp, sp, ctypes.c_double, ctypes.c_uint64, ctypes.c_float, vp, vp, vp, ctypes.c_size_t, vp]
        L.pasa_check_selection.restype = ctypes.c_int
        L.pasa_check_selection.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp]
        L.pasa_kv_stats.restype = ctypes.c_int
        L.pasa_kv_stats.argtypes = [vp, vp, sp, vp, ctypes.c_size_t, vp]
        L.pasa_key_prior.restype = ctypes.c_int
        L.pasa_key_prior.argtypes = [vp, vp, sp, ctypes.c_float, vp, vp, ctypes.c_size_t, vp]
        L.pasa_l1_workspace_bytes.restype = ctypes.c_size_t
        L.pasa_l1_workspace_bytes.argtypes = []
        L.pasa_l1_distance.restype = ctypes.c_int
        L.pasa_l1_distance.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, vp, vp, ctypes.c_size_t, vp]
        L.pasa_budget_schedule.restype = ctypes.c_int
        L.pasa_budget_schedule.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                           ctypes.c_double, ctypes.POINTER(ctypes.c_double)]
        L.pasa_attn_dense_ref.restype = ctypes.c_int
        L.pasa_attn_dense_ref.argtypes = [vp, vp, vp, sp, vp, vp, vp, ctypes.c_size_t, vp]
        _lib = L
    return _lib


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _check_extent(shape: "Shape", **tensors):
    """host-side bounds check of the marshalled arguments: the last element the kernels may touch through the strides
    of `shape` (batch B-1, head H-1, token n-1, column d-1; no token >= n is ever read or written) must lie inside
    the tensor's storage"""
    last = (shape.B - 1) * shape.stride_b + (shape.H - 1) * shape.stride_h + (shape.n - 1) * shape.stride_n + shape.d - 1
    for name, t in tensors.items():
        if t is None:
            continue
        if t.dtype != torch.bfloat16:
            raise ValueError(f"{name}: expected bf16, got {t.dtype}")
        room = t.untyped_storage().nbytes() // t.element_size() - t.storage_offset()
        if last >= room:
            raise ValueError(f"{name}: the shape's strides reach element {last} of a storage that holds {room} from the tensor's start")


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, where: str):
    if rc != 0:
        raise PasaError(rc, where)


def topk_count(n_blocks: int, keep_ratio: float) -> int:
    k = load_library().pasa_topk_count(n_blocks, keep_ratio)
    if k < 0:
        raise PasaError(k, "pasa_topk_count")
    return k


def num_blocks(shape: Shape) -> int:
    nb = load_library().pasa_num_blocks(ctypes.byref(shape.c()))
    if nb < 0:
        raise PasaError(nb, "pasa_num_blocks")
    return nb


def mask_words(n_blocks: int) -> int:
    return load_library().pasa_mask_words(n_blocks)


def score_workspace_bytes(shape: Shape) -> int:
    return load_library().pasa_score_workspace_bytes(ctypes.byref(shape.c()))


def attn_workspace_bytes(shape: Shape) -> int:
    return load_library().pasa_attn_workspace_bytes(ctypes.byref(shape.c()))


def _workspace(nbytes: int, device, ws):
    if ws is None:
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    return ws


def block_score(q, k, shape: Shape, key_bias=None, scores=None, ws=None, stats_ws=None):
    """-> scores fp32 [B*H, N_B, N_B].  With stats_ws (the workspace kv_stats() filled for the same k and shape) the
    block-mean keys are taken from there and K is not read (k may be None)."""
    L = load_library()
    nb = num_blocks(shape)
    if scores is None:
        scores = torch.empty((shape.B * shape.H, nb, nb), dtype=torch.float32, device=q.device)
    ws = _workspace(score_workspace_bytes(shape), q.device, ws)
    _check_extent(shape, q=q, k=k)
    if stats_ws is not None:
        _check(L.pasa_block_score_with_stats(_ptr(q), ctypes.byref(shape.c()), _ptr(key_bias), _ptr(scores), _ptr(ws), ws.numel(),
                                             _ptr(stats_ws), stats_ws.numel(), _stream()), "pasa_block_score_with_stats")
        return scores
    _check(L.pasa_block_score(_ptr(q), _ptr(k), ctypes.byref(shape.c()), _ptr(key_bias), _ptr(scores), _ptr(ws),
                              ws.numel(), _stream()), "pasa_block_score")
    return scores


def route(scores, k_sel: int, seed: int, noise_amp: float, idx=None, mask=None, want_mask: bool = True, noise: str = "uniform"):
    """-> (idx int32 [BH, N_B, k_sel] ascending, mask int32-typed bitmap [BH, N_B, ceil(N_B/32)] or None)
    noise: "uniform" (bias in [-noise_amp, noise_amp), bit-reproducible) or "gumbel" (Gumbel(0, noise_amp) bias)"""
    if noise not in ("uniform", "gumbel"):
        raise ValueError(f"unknown routing noise {noise!r}")
    L = load_library()
    BH, nb, _ = scores.shape
    if idx is None:
        idx = torch.empty((BH, nb, max(k_sel, 1)), dtype=torch.int32, device=scores.device)
    if mask is None and want_mask:
        mask = torch.empty((BH, nb, (nb + 31) // 32), dtype=torch.int32, device=scores.device)
    fn = L.pasa_route if noise == "uniform" else L.pasa_route_gumbel
    _check(fn(_ptr(scores), BH, nb, k_sel, seed & (2**64 - 1), noise_amp, _ptr(idx), _ptr(mask), _stream()), "pasa_route")
    return idx, mask


def check_selection(idx, mask, n_blocks: int, k_sel: int, n_bad=None):
    """number of rows whose index list / bitmap row is not a valid selection of k_sel blocks -> int32 device scalar.
    idx [BH, N_B, k_sel] or None, mask [BH, N_B, ceil(N_B/32)] or None"""
    t = idx if idx is not None else mask
    if n_bad is None:
        n_bad = torch.empty(1, dtype=torch.int32, device=t.device)
    _check(load_library().pasa_check_selection(_ptr(idx), _ptr(mask), t.shape[0], n_blocks, k_sel, _ptr(n_bad), _stream()),
           "pasa_check_selection")
    return n_bad


def kv_stats(k, v, shape: Shape, ws=None):
    """fills (and returns) the attention workspace with the key/value block statistics"""
    L = load_library()
    ws = _workspace(attn_workspace_bytes(shape), k.device, ws)
    _check_extent(shape, k=k, v=v)
    _check(L.pasa_kv_stats(_ptr(k), _ptr(v), ctypes.byref(shape.c()), _ptr(ws), ws.numel(), _stream()), "pasa_kv_stats")
    return ws


def key_prior(k, v, shape: Shape, ws, eps: float = 1e-6, beta=None):
    """covariance-aware routing prior beta [B*H, N_B]; ``ws`` must hold kv_stats() of the same k, v, shape"""
    L = load_library()
    if beta is None:
        beta = torch.empty((shape.B * shape.H, num_blocks(shape)), dtype=torch.float32, device=k.device)
    _check(L.pasa_key_prior(_ptr(k), _ptr(v), ctypes.byref(shape.c()), eps, _ptr(beta), _ptr(ws), ws.numel(), _stream()),
           "pasa_key_prior")
    return beta


def l1_distance(a, b, out=None, ws=None):
    """mean |a - b| of two contiguous bf16 or fp32 device tensors of equal size -> fp32 device scalar"""
    L = load_library()
    if a.dtype != b.dtype or a.numel() != b.numel() or not (a.is_contiguous() and b.is_contiguous()):
        raise ValueError("l1_distance needs two contiguous tensors of the same dtype and size")
    dtype = {torch.bfloat16: 0, torch.float32: 1}.get(a.dtype)
    if dtype is None:
        raise ValueError("l1_distance supports bf16 and fp32")
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=a.device)
    ws = _workspace(int(L.pasa_l1_workspace_bytes()), a.device, ws)
    _check(L.pasa_l1_distance(_ptr(a), _ptr(b), a.numel(), dtype, _ptr(out), _ptr(ws), ws.numel(), _stream()),
           "pasa_l1_distance")
    return out


def budget_schedule(l1, rho: float, dense_fraction: float = 0.2):
    """per-step keep ratios rho_t [n_steps] from calibration signals l1 [n_prompts, n_steps] (host data)"""
    import numpy as np
    L = load_library()
    l1 = np.ascontiguousarray(np.atleast_2d(np.asarray(l1, dtype=np.float64)))
    n_prompts, n_steps = l1.shape
    out = np.empty(n_steps, dtype=np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    _check(L.pasa_budget_schedule(l1.ctypes.data_as(dp), n_prompts, n_steps, float(rho), float(dense_fraction),
                                  out.ctypes.data_as(dp)), "pasa_budget_schedule")
    return out


def sparse_attn_fwd(q, k, v, shape: Shape, idx, mask, out=None, lse=None, ws=None, want_lse: bool = False,
                    prepared: bool = False, k_sel: int | None = None):
    """prepared=True: ``ws`` already holds kv_stats() of the same k, v, shape; run the attention kernel alone.
    One of idx and mask may be None (with idx None pass k_sel)."""
    L = load_library()
    if prepared and ws is None:
        raise ValueError("prepared=True needs the workspace kv_stats() filled")
    if out is None:
        out = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty((shape.B * shape.H, shape.n), dtype=torch.float32, device=q.device)
    ws = _workspace(attn_workspace_bytes(shape), q.device, ws)
    _check_extent(shape, q=q, k=k, v=v, out=out)
    fn = L.pasa_sparse_attn_fwd_prepared if prepared else L.pasa_sparse_attn_fwd
    k_sel = idx.shape[-1] if idx is not None else int(k_sel)
    _check(fn(_ptr(q), _ptr(k), _ptr(v), ctypes.byref(shape.c()), _ptr(idx), _ptr(mask), k_sel, _ptr(out),
              _ptr(lse), _ptr(ws), ws.numel(), _stream()), "pasa_sparse_attn_fwd")
    return (out, lse) if want_lse else out


STATIC_SCRATCH_BYTES = 64 << 20  # PASA_STATIC_SCRATCH_BYTES of pasa.h


def sparse_attn_fwd_static(q, k, v, shape: Shape, idx, mask, out, lse=None):
    """pasa_sparse_attn_fwd_static: the caller passes inputs and outputs only; nothing is allocated, here or in the library"""
    _check_extent(shape, q=q, k=k, v=v, out=out)
    _check(load_library().pasa_sparse_attn_fwd_static(_ptr(q), _ptr(k), _ptr(v), ctypes.byref(shape.c()), _ptr(idx), _ptr(mask),
                                                      idx.shape[-1], _ptr(out), _ptr(lse), _stream()),
           "pasa_sparse_attn_fwd_static")
    return out


def attn_dense_ref(q, k, v, shape: Shape, out=None, lse=None, ws=None, want_lse: bool = False):
    L = load_library()
    if out is None:
        out = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty((shape.B * shape.H, shape.n), dtype=torch.float32, device=q.device)
    ws = _workspace(attn_workspace_bytes(shape), q.device, ws)
    _check_extent(shape, q=q, k=k, v=v, out=out)
    _check(L.pasa_attn_dense_ref(_ptr(q), _ptr(k), _ptr(v), ctypes.byref(shape.c()), _ptr(out), _ptr(lse), _ptr(ws),
                                 ws.numel(), _stream()), "pasa_attn_dense_ref")
    return (out, lse) if want_lse else out


def forward(q, k, v, keep_ratio: float, seed: int, noise_amp: float, block: int = 64, group: int = 32,
            scale: float = 0.0, buffers: dict | None = None):
    """The whole hot path: score -> route -> statistics + piecewise attention. Returns (out, idx).

    ``buffers`` (optional dict) caches every intermediate and workspace between calls.
    """
    shape = Shape.of(q, block=block, group=group, scale=scale)
    nb = num_blocks(shape)
    k_sel = topk_count(nb, keep_ratio)
    b = buffers if buffers is not None else {}
    key = (tuple(q.shape), block, group, k_sel)
    if b.get("key") != key:
        b.clear()
        b["key"] = key
        b["scores"] = torch.empty((shape.B * shape.H, nb, nb), dtype=torch.float32, device=q.device)
        b["idx"] = torch.empty((shape.B * shape.H, nb, k_sel), dtype=torch.int32, device=q.device)
        b["mask"] = torch.empty((shape.B * shape.H, nb, (nb + 31) // 32), dtype=torch.int32, device=q.device)
        b["ws_score"] = torch.empty(score_workspace_bytes(shape), dtype=torch.uint8, device=q.device)
        b["ws_attn"] = torch.empty(attn_workspace_bytes(shape), dtype=torch.uint8, device=q.device)
        b["out"] = torch.empty_like(q)
    block_score(q, k, shape, scores=b["scores"], ws=b["ws_score"])
    route(b["scores"], k_sel, seed, noise_amp, idx=b["idx"], mask=b["mask"])
    sparse_attn_fwd(q, k, v, shape, b["idx"], b["mask"], out=b["out"], ws=b["ws_attn"])
    return b["out"], b["idx"]


def forward_single_call(q, k, v, shape: Shape, keep_ratio: float, seed: int, noise_amp: float, out=None, lse=None, ws=None,
                        want_lse: bool = False):
    """pasa_forward: the whole path in one library call, every intermediate inside one workspace"""
    L = load_library()
    nbytes = int(L.pasa_forward_workspace_bytes(ctypes.byref(shape.c()), float(keep_ratio)))
    if nbytes == 0:
        raise PasaError(-1, "pasa_forward_workspace_bytes")
    ws = _workspace(nbytes, q.device, ws)
    if out is None:
        out = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty((shape.B * shape.H, shape.n), dtype=torch.float32, device=q.device)
    _check_extent(shape, q=q, k=k, v=v, out=out)
    _check(L.pasa_forward(_ptr(q), _ptr(k), _ptr(v), ctypes.byref(shape.c()), float(keep_ratio), seed & (2**64 - 1), noise_amp,
                          _ptr(out), _ptr(lse), _ptr(ws), ws.numel(), _stream()), "pasa_forward")
    return (out, lse) if want_lse else out


def mfma_probe(workgroups: int = 4096, iterations: int = 4096, reps: int = 3, random_operands: bool = False) -> float:
    """TFLOP/s of a loop of nothing but bf16 MFMAs on this device (a measurement aid, see pasa.h); with
    random_operands the operands are N(0,1)-like, which costs power and therefore clock"""
    L = load_library()
    sink = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda")
    flops = ctypes.c_double(0.0)
    rnd = 1 if random_operands else 0
    _check(L.pasa_mfma_probe(workgroups, iterations, rnd, _ptr(sink), ctypes.byref(flops), _stream()), "pasa_mfma_probe")
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        _check(L.pasa_mfma_probe(workgroups, iterations, rnd, _ptr(sink), ctypes.byref(flops), _stream()), "pasa_mfma_probe")
    e1.record()
    torch.cuda.synchronize()
    return flops.value * reps / (e0.elapsed_time(e1) * 1e-3) / 1e12
