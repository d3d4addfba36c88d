"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds NO arithmetic of the attention method: it only manufactures Q, K, V tensors with
the shapes and the "smooth video signal + noise" structure of the video-DiT workloads the paper
evaluates on (Wan 2.1 1.3B/480p and 14B/720p token grids).  Real activations need model weights and
prompts that are not available, so these tensors stand in for them.

Recipe (per head, token grid ``(F, Hh, Ww)`` flattened frame-major, then row, then column):
  field_qk, field_v = Gaussian-smoothed white noise over (F, Hh, Ww), sigma = 2 tokens per axis,
                      reflect boundary, rescaled to unit standard deviation (one field per channel);
  Q = a*N(0,1) + field_qk,  K = a*N(0,1) + field_qk (independent whites, shared field),
  V = a*N(0,1) + field_v,   all rounded to bf16.
Each head draws from its own generator seeded by (seed, head), so a subset of heads can be produced
without producing the others (on the same device type: CPU and GPU generators differ, which is fine
because both sides of any comparison always receive the same tensor).
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    grid: tuple  # (frames, rows, cols) of latent tokens
    heads: int
    d: int
    block: int
    keep_ratio: float
    batch: int = 1
    seed: int = 0

    @property
    def n(self) -> int:
        return self.grid[0] * self.grid[1] * self.grid[2]

    @property
    def n_blocks(self) -> int:
        return (self.n + self.block - 1) // self.block


WORKLOADS = {
    # a CPU oracle finishes this one in seconds
    "tiny": Workload("tiny", (4, 16, 16), heads=2, d=64, block=64, keep_ratio=0.25),
    # Wan 2.1 1.3B at 480p: 21 latent frames x 30 x 52 patches
    "wan1.3b-480p": Workload("wan1.3b-480p", (21, 30, 52), heads=12, d=128, block=64, keep_ratio=0.20),
    # Wan 2.1 14B at 720p: 21 latent frames x 45 x 80 patches = 75,600 tokens
    "wan14b-720p": Workload("wan14b-720p", (21, 45, 80), heads=40, d=128, block=64, keep_ratio=0.15),
    # the paper's second model family, HunyuanVideo 13B at 720p.  The paper gives no shapes for it; these are assumed from
    # the public model description (24 heads of 128; 129 frames -> 33 latent frames x 45 x 80 patches, video tokens only)
    "hunyuan13b-720p": Workload("hunyuan13b-720p", (33, 45, 80), heads=24, d=128, block=64, keep_ratio=0.15),
    # long video: 41 latent frames at the 720p grid, coarse blocks, very sparse
    "long-video": Workload("long-video", (41, 45, 80), heads=40, d=128, block=128, keep_ratio=0.05),
    # the same token count with 64-token blocks: 2307 key blocks, i.e. selection bitmaps of more than 64 words (two heads
    # only: a parity case, not a benchmark)
    "long-video-b64": Workload("long-video-b64", (41, 45, 80), heads=2, d=128, block=64, keep_ratio=0.03),
}


def budget_schedule_keep_ratio(step: int, n_steps: int = 50) -> float:
    """keep ratio of denoising step ``step`` in the budget-schedule workload (a bump around t=0.3)."""
    t = step / n_steps
    return 0.1 + 0.3 * math.exp(-(((t - 0.3) / 0.1) ** 2))


def budget_schedule_noise_amplitude(step: int, n_steps: int = 50) -> float:
    """white-noise amplitude ``a`` of the inputs at ``step``: linear from 1.0 down to 0.2."""
    return 1.0 - 0.8 * step / (n_steps - 1)


def _smoothing_matrix(length: int, sigma: float, device, dtype) -> torch.Tensor:
    """[length, length] matrix applying a truncated Gaussian filter with reflect boundary."""
    radius = max(1, int(4.0 * sigma + 0.5))
    taps = torch.arange(-radius, radius + 1, dtype=torch.float64)
    w = torch.exp(-0.5 * (taps / sigma) ** 2)
    w = w / w.sum()
    m = torch.zeros(length, length, dtype=torch.float64)
    period = 2 * length
    for out in range(length):
        for t, wt in zip(range(-radius, radius + 1), w.tolist()):
            src = (out + t) % period
            if src >= length:
                src = period - 1 - src  # mirror: (d c b a | a b c d | d c b a)
            m[out, src] += wt
    return m.to(device=device, dtype=dtype)


def _smooth_field(gen: torch.Generator, grid, d: int, sigma: float, device) -> torch.Tensor:
    f, h, w = grid
    x = torch.randn((f, h, w, d), generator=gen, device=device, dtype=torch.float32)
    x = torch.einsum("af,fhwd->ahwd", _smoothing_matrix(f, sigma, device, x.dtype), x)
    x = torch.einsum("bh,fhwd->fbwd", _smoothing_matrix(h, sigma, device, x.dtype), x)
    x = torch.einsum("cw,fhwd->fhcd", _smoothing_matrix(w, sigma, device, x.dtype), x)
    x = x / x.std()
    return x.reshape(f * h * w, d)


def _head_generator(seed: int, head: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1_000_003 + int(head) * 7919 + 12345) & 0x7FFFFFFFFFFFFFFF)
    return g


def make_qkv(grid, heads, d: int, seed: int = 0, noise_amplitude: float = 1.0, sigma: float = 2.0,
             device="cpu", batch: int = 1):
    """Q, K, V as bf16 tensors ``[batch, len(heads), n, d]``.

    ``heads`` is an int (heads 0..heads-1) or an explicit list of head ids (batch b, head h draws
    from stream ``b * 4096 + h``).
    """
    head_ids = list(range(heads)) if isinstance(heads, int) else list(heads)
    n = grid[0] * grid[1] * grid[2]
    dev = torch.device(device)
    q = torch.empty((batch, len(head_ids), n, d), dtype=torch.bfloat16, device=dev)
    k = torch.empty_like(q)
    v = torch.empty_like(q)
    for b in range(batch):
        for slot, h in enumerate(head_ids):
            gen = _head_generator(seed, b * 4096 + h, dev)
            f_qk = _smooth_field(gen, grid, d, sigma, dev)
            f_v = _smooth_field(gen, grid, d, sigma, dev)
            for dst, field in ((q, f_qk), (k, f_qk), (v, f_v)):
                white = torch.randn((n, d), generator=gen, device=dev, dtype=torch.float32)
                dst[b, slot] = (noise_amplitude * white + field).to(torch.bfloat16)
    return q, k, v


def make_workload_qkv(w: Workload, device="cpu", heads=None, noise_amplitude: float = 1.0, seed=None):
    return make_qkv(w.grid, w.heads if heads is None else heads, w.d, seed=w.seed if seed is None else seed,
                    noise_amplitude=noise_amplitude, device=device, batch=w.batch)
