"""GPU tests of the boundary's safety net: validation of caller-built selections, attention from index lists alone,
and guard bands -- every output and workspace sits between sentinel-filled bands that must come back untouched, every
input between NaN-filled bands that must not leak into a result."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from _util import assert_close, to_f64

pytestmark = pytest.mark.gpu

GUARD = 4096  # bytes on either side


@pytest.fixture(scope="module")
def P():
    import paper_2604_12219_amd as P
    assert torch.cuda.is_available(), "these tests need the MI355X"
    P.load_library()
    return P


def _routed(P, grid=(5, 21, 13), heads=2, d=128, block=64, keep=0.2, seed=9):
    q, k, v = workloads.make_qkv(grid, heads, d, seed=seed, device="cuda")
    shape = P.Shape.of(q, block=block, group=32)
    nb = P.num_blocks(shape)
    k_sel = P.topk_count(nb, keep)
    scores = P.block_score(q, k, shape)
    idx, mask = P.route(scores, k_sel, seed, 0.2)
    return q, k, v, shape, nb, k_sel, idx, mask


def test_check_selection_passes_routing_output_and_counts_each_kind_of_corruption(P):
    q, k, v, shape, nb, k_sel, idx, mask = _routed(P)
    assert nb == 22 and k_sel == 4
    assert P.check_selection(idx, mask, nb, k_sel).item() == 0
    assert P.check_selection(idx, None, nb, k_sel).item() == 0
    assert P.check_selection(None, mask, nb, k_sel).item() == 0

    def corrupted(fn):
        i2, m2 = idx.clone(), mask.clone()
        fn(i2, m2)
        return i2, m2

    def out_of_range(i, m): i[0, 3, 2] = nb
    def negative(i, m): i[1, 0, 0] = -1
    def descending(i, m): i[0, 5, 1], i[0, 5, 2] = i[0, 5, 2].item(), i[0, 5, 1].item()
    def duplicate(i, m): i[1, 7, 1] = i[1, 7, 0]
    def extra_bit(i, m):  # a fifth block in the bitmap
        free = next(j for j in range(nb) if j not in i[0, 9].tolist())
        m[0, 9, free >> 5] |= 1 << (free & 31)
    def missing_bit(i, m):
        j = i[1, 11, 0].item()
        m[1, 11, j >> 5] &= ~(1 << (j & 31))
    def beyond_end(i, m): m[0, 2, 0] |= 1 << 25  # block 25 of 22 does not exist
    def other_block(i, m):  # same population count, different set
        j = i[1, 20, 3].item()
        free = next(x for x in range(nb) if x not in i[1, 20].tolist())
        m[1, 20, 0] = (m[1, 20, 0] & ~(1 << j)) | (1 << free)

    kinds = [out_of_range, negative, descending, duplicate, extra_bit, missing_bit, beyond_end, other_block]
    for fn in kinds:
        i2, m2 = corrupted(fn)
        assert P.check_selection(i2, m2, nb, k_sel).item() == 1, fn.__name__
    i2, m2 = idx.clone(), mask.clone()
    for fn in kinds:  # all at once, each in a row of its own
        fn(i2, m2)
    assert P.check_selection(i2, m2, nb, k_sel).item() == len(kinds)
    assert P.check_selection(i2, None, nb, k_sel).item() == 4   # what the lists alone show
    assert P.check_selection(None, m2, nb, k_sel).item() == 3   # what the bitmap alone shows (extra, missing, beyond the end)
    # twice in a row into the same counter: it is reset by the call
    n_bad = torch.full((1,), 77, dtype=torch.int32, device="cuda")
    P.check_selection(idx, mask, nb, k_sel, n_bad=n_bad)
    assert n_bad.item() == 0


@pytest.mark.parametrize("grid,d,block", [((5, 21, 13), 128, 64), ((9, 20, 23), 64, 128), ((12, 30, 33), 128, 64)])
def test_attention_from_index_lists_alone_and_from_the_bitmap_alone(P, grid, d, block):
    """a caller with its own index lists passes no bitmap (one is built from the lists); a caller with a bitmap passes no lists"""
    q, k, v, shape, nb, k_sel, idx, mask = _routed(P, grid=grid, d=d, block=block, keep=0.15)
    want, want_lse = P.sparse_attn_fwd(q, k, v, shape, idx, mask, want_lse=True)
    from_idx, lse_i = P.sparse_attn_fwd(q, k, v, shape, idx, None, want_lse=True)
    from_mask, lse_m = P.sparse_attn_fwd(q, k, v, shape, None, mask, want_lse=True, k_sel=k_sel)
    torch.cuda.synchronize()
    assert torch.equal(from_idx, want) and torch.equal(from_mask, want)
    assert torch.equal(lse_i, want_lse) and torch.equal(lse_m, want_lse)
    ref = oracle.pasa_attention(to_f64(q), to_f64(k), to_f64(v), idx.cpu().numpy(), block, group=32)
    assert_close(to_f64(from_idx), ref, what="index lists alone")


def _banded(nbytes_or_shape, dtype, fill):
    """a tensor of the given shape in the middle of a larger allocation whose bands on both sides hold `fill`"""
    shape = tuple(nbytes_or_shape) if not isinstance(nbytes_or_shape, int) else (nbytes_or_shape,)
    esz = torch.empty((), dtype=dtype).element_size()
    n = int(np.prod(shape))
    pad = GUARD // esz
    lead = (256 // esz)  # keeps the payload 256-byte aligned
    pad = (pad + lead - 1) // lead * lead
    whole = torch.full((pad + n + pad,), fill, dtype=dtype, device="cuda")
    return whole, whole[pad:pad + n].view(shape)


def _bands_intact(whole, payload, fill):
    esz = whole.element_size()
    start = (payload.data_ptr() - whole.data_ptr()) // esz
    lo, hi = whole[:start], whole[start + payload.numel():]
    if isinstance(fill, float) and fill != fill:
        return bool(torch.isnan(lo).all() and torch.isnan(hi).all())
    return bool((lo == fill).all() and (hi == fill).all())


@pytest.mark.parametrize("grid,d,block,group", [((5, 21, 13), 128, 64, 32), ((9, 20, 23), 64, 128, 32), ((9, 20, 23), 128, 64, 8),
                                                ((1, 9, 11), 128, 64, 32)])
def test_nothing_is_written_outside_the_buffers_and_nothing_outside_the_inputs_is_used(P, grid, d, block, group):
    heads = 2
    q0, k0, v0 = workloads.make_qkv(grid, heads, d, seed=17, device="cuda")
    nan = float("nan")
    ins = []
    for t in (q0, k0, v0):  # inputs between NaN bands: a row read from outside and used would poison the result
        whole, view = _banded(t.shape, torch.bfloat16, nan)
        view.copy_(t)
        ins.append((whole, view))
    q, k, v = (x[1] for x in ins)
    shape = P.Shape.of(q, block=block, group=group)
    nb = P.num_blocks(shape)
    k_sel = P.topk_count(nb, 0.25)
    bh = heads
    bufs = {
        "scores": _banded((bh, nb, nb), torch.float32, nan),
        "idx": _banded((bh, nb, k_sel), torch.int32, -7),
        "mask": _banded((bh, nb, P.mask_words(nb)), torch.int32, -7),
        "ws_score": _banded(P.score_workspace_bytes(shape), torch.uint8, 0xA5),
        "ws_attn": _banded(P.attn_workspace_bytes(shape), torch.uint8, 0xA5),
        "out": _banded(q.shape, torch.bfloat16, nan),
        "lse": _banded((bh, shape.n), torch.float32, nan),
        "dense": _banded(q.shape, torch.bfloat16, nan),
        "beta": _banded((bh, nb), torch.float32, nan),
        "n_bad": _banded((1,), torch.int32, -7),
    }
    b = {name: view for name, (_, view) in bufs.items()}
    b["ws_attn"].fill_(0xFF)  # NaN patterns inside the workspace too: stale contents must never be consumed
    P.block_score(q, k, shape, scores=b["scores"], ws=b["ws_score"])
    P.route(b["scores"], k_sel, 5, 0.2, idx=b["idx"], mask=b["mask"])
    P.check_selection(b["idx"], b["mask"], nb, k_sel, n_bad=b["n_bad"])
    P.sparse_attn_fwd(q, k, v, shape, b["idx"], b["mask"], out=b["out"], lse=b["lse"], ws=b["ws_attn"])
    P.key_prior(k, v, shape, b["ws_attn"], beta=b["beta"])
    P.attn_dense_ref(q, k, v, shape, out=b["dense"], ws=b["ws_attn"])
    torch.cuda.synchronize()
    for name, (whole, view) in bufs.items():
        fill = {"idx": -7, "mask": -7, "n_bad": -7, "ws_score": 0xA5, "ws_attn": 0xA5}.get(name, nan)
        assert _bands_intact(whole, view, fill), f"{name}: guard band overwritten"
    for whole, view in ins:
        assert _bands_intact(whole, view, nan)
    assert b["n_bad"].item() == 0
    for name in ("scores", "out", "lse", "dense", "beta"):
        assert torch.isfinite(b[name].float()).all(), f"{name}: non-finite values (something outside the inputs was used)"
    ref = oracle.pasa_attention(to_f64(q0), to_f64(k0), to_f64(v0), b["idx"].cpu().numpy(), block, group=group)
    assert_close(to_f64(b["out"]), ref, what="guarded sparse")
    assert_close(to_f64(b["dense"]), oracle.dense_attention(to_f64(q0), to_f64(k0), to_f64(v0)), what="guarded dense")
