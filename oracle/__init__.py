"""Python face of the fp64 CPU oracle (``pasa_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
``cpu_baseline`` leg.  Nothing in the product package may import this module, and this module
imports nothing from the product package.

Every function takes and returns numpy arrays (float64 unless stated); tensors are laid out
``[BH, n, d]`` with ``BH`` = batch*heads flattened.  The arithmetic lives in the C file; this module
only marshals arguments.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pasa_oracle.c")
_LIB = os.path.join(_HERE, "libpasa_oracle.so")

_f64p = ctypes.POINTER(ctypes.c_double)
_f32p = ctypes.POINTER(ctypes.c_float)
_i32p = ctypes.POINTER(ctypes.c_int32)
_u32p = ctypes.POINTER(ctypes.c_uint32)
_i64 = ctypes.c_int64


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (no HIP involved). Returns the path of the shared object."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build_oracle())
        L = _lib
        L.oracle_num_threads.restype = ctypes.c_int32
        L.oracle_topk_count.restype = ctypes.c_int32
        L.oracle_topk_count.argtypes = [ctypes.c_int32, ctypes.c_double]
        L.oracle_philox4x32_10.restype = None
        L.oracle_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        L.oracle_noise_unit.restype = ctypes.c_float
        L.oracle_noise_unit.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32]
        L.oracle_block_mean.restype = None
        L.oracle_block_mean.argtypes = [_f64p, _i64, _i64, _i64, _i64, _f64p]
        L.oracle_block_scores.restype = None
        L.oracle_block_scores.argtypes = [_f64p, _f64p, _i64, _i64, _i64, _i64, ctypes.c_double, _f64p, _f64p]
        L.oracle_route.restype = None
        L.oracle_route.argtypes = [_f32p, _i64, _i64, _i64, ctypes.c_uint64, ctypes.c_float, _i32p, _i32p, _f32p]
        L.oracle_kv_stats.restype = None
        L.oracle_kv_stats.argtypes = [_f64p, _f64p, _i64, _i64, _i64, _i64, _i64, _f64p, _f64p, _f64p, _f64p]
        L.oracle_dense_attention.restype = None
        L.oracle_dense_attention.argtypes = [_f64p, _f64p, _f64p, _i64, _i64, _i64, ctypes.c_double, _i32p, _i64, _f64p, _f64p]
        L.oracle_pasa_attention.restype = None
        L.oracle_pasa_attention.argtypes = [_f64p, _f64p, _f64p, _i64, _i64, _i64, _i64, _i64, ctypes.c_double,
                                            _i32p, _i64, ctypes.c_int32, _i32p, _i64, _f64p, _f64p, _f64p, _f64p]
        L.oracle_lemma1.restype = None
        L.oracle_lemma1.argtypes = [_f64p, _f64p, _f64p, _f64p, _i64, _i64, _i64, _i32p, _i64, _f64p]
    return _lib


def _p(a, ptr):
    return None if a is None else a.ctypes.data_as(ptr)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _bhnd(x):
    x = _c(x, np.float64)
    if x.ndim != 3:
        raise ValueError("expected a [BH, n, d] array")
    return x


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def n_blocks(n: int, block: int) -> int:
    return (n + block - 1) // block


def topk_count(n_blocks_: int, keep_ratio: float) -> int:
    return int(_load().oracle_topk_count(int(n_blocks_), float(keep_ratio)))


def philox4x32_10(ctr, key):
    c = _c(ctr, np.uint32)
    k = _c(key, np.uint32)
    out = np.empty(4, np.uint32)
    _load().oracle_philox4x32_10(_p(c, _u32p), _p(k, _u32p), _p(out, _u32p))
    return out


def noise_unit(seed: int, bh: int, i: int, j: int) -> float:
    return float(_load().oracle_noise_unit(int(seed), int(bh), int(i), int(j)))


def block_mean(x, block: int):
    x = _bhnd(x)
    BH, n, d = x.shape
    out = np.empty((BH, n_blocks(n, block), d), np.float64)
    _load().oracle_block_mean(_p(x, _f64p), BH, n, d, block, _p(out, _f64p))
    return out


def block_scores(q, k, block: int, scale: float | None = None, key_bias=None):
    q, k = _bhnd(q), _bhnd(k)
    BH, n, d = q.shape
    NB = n_blocks(n, block)
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    kb = None if key_bias is None else _c(key_bias, np.float64)
    out = np.empty((BH, NB, NB), np.float64)
    _load().oracle_block_scores(_p(q, _f64p), _p(k, _f64p), BH, n, d, block, float(scale), _p(kb, _f64p), _p(out, _f64p))
    return out


def route(scores_f32, k: int, seed: int, amp: float, bh_ids=None, return_noisy: bool = False):
    """scores_f32 [BH, NB, NB] float32 -> idx [BH, NB, k] int32 ascending (and the noisy scores)."""
    s = _c(scores_f32, np.float32)
    BH, NB, NB2 = s.shape
    assert NB == NB2
    ids = None if bh_ids is None else _c(bh_ids, np.int32)
    idx = np.empty((BH, NB, k), np.int32)
    noisy = np.empty_like(s) if return_noisy else None
    _load().oracle_route(_p(s, _f32p), BH, NB, int(k), int(seed) & (2**64 - 1), float(amp), _p(ids, _i32p), _p(idx, _i32p), _p(noisy, _f32p))
    return (idx, noisy) if return_noisy else idx

def _philox4x32_10_np(c0, c1, c2, c3, k0, k1):
    """Philox4x32-10 (Salmon et al., "Parallel random numbers: as easy as 1, 2, 3") on numpy arrays of counters;
    written out in 64-bit integer arithmetic, independently of the C routine above (a pin compares the two)."""
    M0, M1, W0, W1, MASK = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85, 0xFFFFFFFF
    c0, c1, c2, c3 = (np.asarray(c, np.uint64) & np.uint64(MASK) for c in np.broadcast_arrays(c0, c1, c2, c3))
    k0, k1 = int(k0) & MASK, int(k1) & MASK
    for _ in range(10):
        p0 = np.uint64(M0) * c0
        p1 = np.uint64(M1) * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & np.uint64(MASK)
        hi1, lo1 = p1 >> np.uint64(32), p1 & np.uint64(MASK)
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
        k0, k1 = (k0 + W0) & MASK, (k1 + W1) & MASK
    return c0, c1, c2, c3


def route_gumbel(scores_f32, k: int, seed: int, temperature: float, bh_ids=None, return_noisy: bool = False):
    """Routing with a Gumbel-distributed selection bias (Sec. "Stochastic Routing" fixes no distribution; this is
    the Gumbel-top-k variant): r = s + temperature * g, g = -log(-log(u)), u = ((x >> 9) + 0.5) 2^-23 with x the
    Philox word of (bh, i, j) exactly as in route(); the k largest r per row (ties: smaller j), ascending.
    fp64 after the binary32 scores.  -> idx [BH, NB, k] int32 (and r)."""
    s = _c(scores_f32, np.float32).astype(np.float64)
    BH, NB, NB2 = s.shape
    assert NB == NB2 and 1 <= k <= NB
    seed = int(seed) & (2**64 - 1)
    bh = np.arange(BH) if bh_ids is None else np.asarray(bh_ids)
    j = np.arange(NB)
    words = _philox4x32_10_np((j >> 2)[None, None, :], np.arange(NB)[None, :, None], bh[:, None, None], 0,
                              seed & 0xFFFFFFFF, seed >> 32)
    x = np.choose((j & 3)[None, None, :], words)  # word j & 3 of the call that serves blocks 4(j>>2) .. +3
    u = ((x >> np.uint64(9)).astype(np.float64) + 0.5) * 2.0**-23
    r = s + float(temperature) * -np.log(-np.log(u))
    order = np.lexsort((np.broadcast_to(j, r.shape), -r), axis=-1)  # larger r first, then smaller j
    idx = np.sort(order[..., :k], axis=-1).astype(np.int32)
    return (idx, r) if return_noisy else idx


def kv_stats(k, v, block: int, group: int, want_hj: bool = False):
    """Returns dict(kbar, vs, hg[, hj]); hg is None when group <= 0."""
    k, v = _bhnd(k), _bhnd(v)
    BH, n, d = k.shape
    NB = n_blocks(n, block)
    NG = (NB + group - 1) // group if group > 0 else 0
    kbar = np.empty((BH, NB, d), np.float64)
    vs = np.empty((BH, NB, d), np.float64)
    hj = np.empty((BH, NB, d, d), np.float64) if want_hj else None
    hg = np.empty((BH, NG, d, d), np.float64) if NG else None
    _load().oracle_kv_stats(_p(k, _f64p), _p(v, _f64p), BH, n, d, block, group, _p(kbar, _f64p), _p(vs, _f64p), _p(hj, _f64p), _p(hg, _f64p))
    return dict(kbar=kbar, vs=vs, hj=hj, hg=hg)


def key_prior(k, v, block: int, group: int, eps: float = 1e-6):
    """Covariance-aware routing prior, the second term of Eq.8, for every key block:
    beta[bh, j] = log(||H_j - Hg_{g(j)}||_F + eps), H_j as in Eq.5, Hg the mean of H_j over the group of
    `group` consecutive blocks that contains j (Eq.12; group >= N_B: the global mean of Eq.6), Frobenius
    norm, no logit scale.  Written out from oracle_kv_stats' H_j and Hg."""
    assert group > 0
    st = kv_stats(k, v, block, group, want_hj=True)
    hj, hg = st["hj"], st["hg"]
    BH, NB = hj.shape[:2]
    g_eff = min(group, NB)
    beta = np.empty((BH, NB), np.float64)
    for bh in range(BH):
        for j in range(NB):
            diff = hj[bh, j] - hg[bh, j // g_eff]
            beta[bh, j] = np.log(np.sqrt((diff * diff).sum()) + eps)
    return beta


def l1_distance(a, b) -> float:
    """mean absolute difference of two arrays (the calibration signal of Sec. "Curvature-Aware Dynamic
    Budgeting": distance between the velocity fields of consecutive steps), in float64"""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.abs(a - b).sum() / a.size)


def budget_schedule(l1, rho: float, dense_fraction: float = 0.2):
    """Eq.9-11: l1 [n_prompts, n_steps] -> rho_t [n_steps].  The first floor(dense_fraction*n_steps + 0.5)
    steps are dense (rho_t = 1); on the others l_t is the prompt average, lbar its mean over those steps,
    alpha_t = l_t / lbar, rho_t = rho * alpha_t, capped at 1."""
    l1 = np.atleast_2d(np.asarray(l1, np.float64))
    n_steps = l1.shape[1]
    n_dense = min(n_steps, int(math.floor(dense_fraction * n_steps + 0.5)))
    out = np.ones(n_steps, np.float64)
    if n_dense < n_steps:
        lt = l1[:, n_dense:].mean(axis=0)
        lbar = lt.mean()
        alpha = lt / lbar
        out[n_dense:] = np.minimum(1.0, rho * alpha)
    return out


def dense_attention(q, k, v, scale: float | None = None, q_rows=None, return_lse: bool = False):
    q, k, v = _bhnd(q), _bhnd(k), _bhnd(v)
    BH, n, d = q.shape
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    rows = None if q_rows is None else _c(q_rows, np.int32)
    nr = n if rows is None else len(rows)
    o = np.empty((BH, nr, d), np.float64)
    lse = np.empty((BH, nr), np.float64)
    _load().oracle_dense_attention(_p(q, _f64p), _p(k, _f64p), _p(v, _f64p), BH, n, d, float(scale), _p(rows, _i32p), nr, _p(o, _f64p), _p(lse, _f64p))
    return (o, lse) if return_lse else o


def pasa_attention(q, k, v, idx, block: int, group: int = 32, scale: float | None = None, terms: int = 3,
                   q_blocks=None, return_all: bool = False):
    """PASA piecewise attention for the routing ``idx`` [BH, NB, k].

    Returns O [BH, n, d] (rows outside ``q_blocks`` are NaN), or a dict with o, lse, parts, wsum.
    """
    q, k, v = _bhnd(q), _bhnd(k), _bhnd(v)
    BH, n, d = q.shape
    NB = n_blocks(n, block)
    idx = _c(idx, np.int32)
    assert idx.shape[:2] == (BH, NB), (idx.shape, BH, NB)
    ksel = idx.shape[2]
    assert idx.min() >= 0 and idx.max() < NB
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    qb = None if q_blocks is None else _c(q_blocks, np.int32)
    nqb = 0 if qb is None else len(qb)
    o = np.full((BH, n, d), np.nan, np.float64)
    lse = np.full((BH, n), np.nan, np.float64)
    parts = np.full((BH, n, 3, d), np.nan, np.float64) if return_all else None
    wsum = np.full((BH, n, 2), np.nan, np.float64) if return_all else None
    _load().oracle_pasa_attention(_p(q, _f64p), _p(k, _f64p), _p(v, _f64p), BH, n, d, block, int(group), float(scale),
                                  _p(idx, _i32p), ksel, int(terms), _p(qb, _i32p), nqb,
                                  _p(o, _f64p), _p(lse, _f64p), _p(parts, _f64p), _p(wsum, _f64p))
    if return_all:
        return dict(o=o, lse=lse, parts=parts, wsum=wsum)
    return o


def lemma1(q_scaled, kbar, hj, hg, group: int, sel_idx):
    """(||R||_F, bound) of Lemma 1 for one scaled query row and one head's statistics."""
    qs = _c(q_scaled, np.float64)
    kbar, hj, hg = _c(kbar, np.float64), _c(hj, np.float64), _c(hg, np.float64)
    NB, d = kbar.shape
    sel = _c(sel_idx, np.int32)
    out = np.empty(2, np.float64)
    _load().oracle_lemma1(_p(qs, _f64p), _p(kbar, _f64p), _p(hj, _f64p), _p(hg, _f64p), NB, d, int(group), _p(sel, _i32p), len(sel), _p(out, _f64p))
    return float(out[0]), float(out[1])
