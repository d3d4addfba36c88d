"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by element,
on the same seeded inputs.  Sizes span several tiles and ragged tails."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from _util import assert_close, to_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2604_12219_amd as P
    assert torch.cuda.is_available(), "these tests need the MI355X"
    P.load_library()
    return P


def _inputs(grid, heads, d, seed=0, batch=1):
    return workloads.make_qkv(grid, heads, d, seed=seed, device="cuda", batch=batch)


# ------------------------------------------------------------------------------------------------
# dense reference kernel (Eq.1)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("grid,heads,d", [((4, 16, 16), 2, 64), ((3, 11, 13), 2, 128), ((1, 5, 7), 1, 128),
                                          ((2, 16, 16), 3, 128)])
def test_dense_matches_oracle(P, grid, heads, d):
    q, k, v = _inputs(grid, heads, d)
    shape = P.Shape.of(q)
    out, lse = P.attn_dense_ref(q, k, v, shape, want_lse=True)
    torch.cuda.synchronize()
    ref, ref_lse = oracle.dense_attention(to_f64(q), to_f64(k), to_f64(v), return_lse=True)
    assert_close(to_f64(out), ref, what=f"dense {grid} d={d}")
    np.testing.assert_allclose(lse.cpu().numpy(), ref_lse, atol=2e-2)


def test_dense_respects_strides_and_scale(P):
    q, k, v = _inputs((2, 9, 10), 2, 128)
    B, H, n, d = q.shape
    big = torch.zeros((3, B, n, H, d + 8), dtype=torch.bfloat16, device="cuda")  # [which, B, n, H, d+pad]
    for i, t in enumerate((q, k, v)):
        big[i, :, :, :, :d] = t.permute(0, 2, 1, 3)
    qs, ks, vs = (big[i, :, :, :, :d].permute(0, 2, 1, 3) for i in range(3))  # [B,H,n,d] views, n-stride H*(d+8)
    shape = P.Shape.of(qs, scale=0.11)
    out = torch.zeros_like(big[0])[:, :, :, :d].permute(0, 2, 1, 3)
    P.attn_dense_ref(qs, ks, vs, shape, out=out)
    torch.cuda.synchronize()
    ref = oracle.dense_attention(to_f64(q), to_f64(k), to_f64(v), scale=0.11)
    assert_close(to_f64(out), ref, what="strided dense")


# ------------------------------------------------------------------------------------------------
# stage 1: scores
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("grid,d,block", [((4, 16, 16), 64, 64), ((3, 21, 13), 128, 64), ((3, 21, 13), 128, 128)])
def test_block_scores_match_oracle(P, grid, d, block):
    q, k, _ = _inputs(grid, 2, d)
    shape = P.Shape.of(q, block=block)
    nb = P.num_blocks(shape)
    bias = torch.randn((2, nb), device="cuda", generator=torch.Generator("cuda").manual_seed(1))
    s0 = P.block_score(q, k, shape)
    s1 = P.block_score(q, k, shape, key_bias=bias)
    torch.cuda.synchronize()
    ref = oracle.block_scores(to_f64(q), to_f64(k), block)
    tol = 1e-3 * np.abs(ref).max()
    np.testing.assert_allclose(s0.cpu().numpy(), ref, atol=tol, rtol=0)
    np.testing.assert_allclose(s1.cpu().numpy(), ref + bias.cpu().numpy()[:, None, :], atol=tol, rtol=0)


@pytest.mark.parametrize("grid,d,block,group", [((4, 16, 16), 64, 64, 32), ((3, 21, 13), 128, 64, 32), ((3, 21, 13), 128, 128, 8),
                                                ((9, 20, 23), 128, 64, 64), ((9, 20, 23), 64, 64, 1000), ((1, 5, 7), 128, 64, 32)])
def test_block_scores_from_the_statistics_workspace(P, grid, d, block, group):
    """pasa_block_score_with_stats: the block-mean keys come from pasa_kv_stats' workspace, K is not read again"""
    q, k, v = _inputs(grid, 2, d, seed=3)
    shape = P.Shape.of(q, block=block, group=group)
    nb = P.num_blocks(shape)
    bias = torch.randn((2, nb), device="cuda", generator=torch.Generator("cuda").manual_seed(2))
    ws = P.kv_stats(k, v, shape)
    s0 = P.block_score(q, None, shape, stats_ws=ws)
    s1 = P.block_score(q, None, shape, key_bias=bias, stats_ws=ws)
    plain = P.block_score(q, k, shape)
    torch.cuda.synchronize()
    ref = oracle.block_scores(to_f64(q), to_f64(k), block)
    tol = 1e-3 * np.abs(ref).max()
    np.testing.assert_allclose(s0.cpu().numpy(), ref, atol=tol, rtol=0)
    np.testing.assert_allclose(s1.cpu().numpy(), ref + bias.cpu().numpy()[:, None, :], atol=tol, rtol=0)
    # the two routes to the scores differ only by the summation order of the key means
    np.testing.assert_allclose(s0.cpu().numpy(), plain.cpu().numpy(), atol=2e-5 * np.abs(ref).max(), rtol=0)
    # the statistics workspace still serves the attention kernel afterwards
    k_sel = P.topk_count(nb, 0.3)
    idx, mask = P.route(s0, k_sel, 5, 0.1)
    out = P.sparse_attn_fwd(q, k, v, shape, idx, mask, ws=ws, prepared=True)
    torch.cuda.synchronize()
    res = oracle.pasa_attention(to_f64(q), to_f64(k), to_f64(v), idx.cpu().numpy(), block, group=group)
    assert_close(to_f64(out), res, what="attention after scoring from the statistics")
    with pytest.raises(P.PasaError):  # approximation off: the statistics call leaves no key means
        P.block_score(q, None, P.Shape.of(q, block=block, group=0), stats_ws=ws)


@pytest.mark.parametrize("grid,d,block,group", [((4, 16, 16), 64, 64, 32), ((5, 21, 13), 128, 64, 8),
                                                ((9, 20, 23), 128, 64, 32), ((9, 20, 23), 128, 64, 64),
                                                ((9, 20, 23), 128, 64, 1000), ((9, 20, 23), 128, 128, 32),
                                                ((9, 20, 23), 64, 64, 1)])
def test_key_prior_matches_oracle_and_feeds_the_scores(P, grid, d, block, group):
    """covariance-aware routing prior (Eq.8): beta against the oracle, then scores with it as key bias"""
    q, k, v = _inputs(grid, 2, d, seed=5)
    shape = P.Shape.of(q, block=block, group=group)
    ws = P.kv_stats(k, v, shape)
    beta = P.key_prior(k, v, shape, ws, eps=1e-6)
    torch.cuda.synchronize()
    ref = oracle.key_prior(to_f64(k), to_f64(v), block, group, eps=1e-6)
    if group == 1:  # every block is its own group: the norm is rounding noise, only "tiny" can be compared
        assert np.all(beta.cpu().numpy() < np.log(1e-2)) and np.all(ref < np.log(1e-5))
    else:
        np.testing.assert_allclose(beta.cpu().numpy(), ref, atol=2e-3, rtol=0)
    s = P.block_score(q, k, shape, key_bias=beta)
    torch.cuda.synchronize()
    want = oracle.block_scores(to_f64(q), to_f64(k), block) + beta.cpu().numpy().astype(np.float64)[:, None, :]
    np.testing.assert_allclose(s.cpu().numpy(), want, atol=1e-3 * np.abs(want).max(), rtol=0)


# ------------------------------------------------------------------------------------------------
# stage 2: routing is bit-exact against the oracle fed the GPU's scores
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("nb,k_sel,amp", [(16, 4, 0.0), (16, 4, 0.5), (67, 9, 1.0), (130, 130, 0.3), (515, 77, 2.0),
                                          (1182, 177, 0.7), (64, 1, 0.1), (1000, 150, 0.3), (1500, 1500, 0.1),
                                          (2000, 3, 0.2), (4096, 300, 0.5)])
def test_routing_bit_exact(P, nb, k_sel, amp):
    g = torch.Generator("cuda").manual_seed(nb)
    scores = torch.randn((3, nb, nb), device="cuda", generator=g)
    scores[0, 0, : nb // 2] = 0.25  # ties
    scores[1, 1, :] = -1.5          # a fully tied row
    scores[2, 0, 0] = -0.0
    seed = 0x1234_5678_9ABC_DEF0 + nb
    idx, mask = P.route(scores, k_sel, seed, amp)
    torch.cuda.synchronize()
    want = oracle.route(scores.cpu().numpy(), k_sel, seed, amp)
    np.testing.assert_array_equal(idx.cpu().numpy(), want)
    words = mask.cpu().numpy().view(np.uint32)
    bits = np.zeros((3, nb, words.shape[-1] * 32), bool)
    for h in range(3):
        for i in range(nb):
            bits[h, i, want[h, i]] = True
    packed = np.packbits(bits.reshape(3, nb, -1, 32), axis=-1, bitorder="little").view(np.uint32)[..., 0]
    np.testing.assert_array_equal(words, packed)


@pytest.mark.parametrize("nb,k_sel,tau", [(16, 4, 0.0), (67, 9, 1.0), (515, 77, 0.3), (1182, 177, 0.125)])
def test_gumbel_routing_matches_oracle_up_to_the_rounding_of_the_logarithms(P, nb, k_sel, tau):
    """Relaxed parity: the oracle takes the two logarithms in fp64, the kernel in binary32, so a block may differ
    only if its perturbed logit lies within rounding distance of the k-th largest of its row."""
    g = torch.Generator("cuda").manual_seed(nb)
    scores = torch.randn((3, nb, nb), device="cuda", generator=g)
    seed = 0x0FED_CBA9_8765_4321 + nb
    idx, mask = P.route(scores, k_sel, seed, tau, noise="gumbel")
    torch.cuda.synchronize()
    got = idx.cpu().numpy()
    want, r = oracle.route_gumbel(scores.cpu().numpy(), k_sel, seed, tau, return_noisy=True)
    assert (np.diff(got, axis=-1) > 0).all() and got.min() >= 0 and got.max() < nb  # k distinct blocks, ascending
    bits = (mask.cpu().numpy().view(np.uint32)[..., None] >> np.arange(32, dtype=np.uint32)) & 1
    sel = np.zeros((3, nb, nb), bool)
    np.put_along_axis(sel, got.astype(np.int64), True, axis=-1)
    np.testing.assert_array_equal(bits.reshape(3, nb, -1)[..., :nb].astype(bool), sel)
    # |g| <= 17 for this grid of u; binary32 logarithms and the fused multiply-add: a few ulp of the largest term
    delta = 64 * 2.0**-24 * (np.abs(r).max() + 17 * tau)
    kth = np.sort(r, axis=-1)[..., nb - k_sel][..., None]
    want_sel = np.zeros_like(sel)
    np.put_along_axis(want_sel, want.astype(np.int64), True, axis=-1)
    differ = sel != want_sel
    assert (np.abs(r - kth)[differ] <= delta).all()
    assert differ.mean() < 1e-3
    if tau == 0.0:
        assert not differ.any()



def test_routing_on_real_scores_and_determinism(P):
    q, k, _ = _inputs((4, 16, 16), 2, 64)
    shape = P.Shape.of(q)
    scores = P.block_score(q, k, shape)
    idx, mask = P.route(scores, 4, 99, 0.4)
    idx2, mask2 = P.route(scores, 4, 99, 0.4)
    idx3, _ = P.route(scores, 4, 100, 0.4)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(mask, mask2)
    assert not torch.equal(idx, idx3)
    np.testing.assert_array_equal(idx.cpu().numpy(), oracle.route(scores.cpu().numpy(), 4, 99, 0.4))


# ------------------------------------------------------------------------------------------------
# stages 3+4: piecewise attention
# ------------------------------------------------------------------------------------------------
def _run_sparse(P, q, k, v, block, group, keep, seed=3, amp=0.3, kv_slices=0):
    shape = P.Shape.of(q, block=block, group=group, kv_slices=kv_slices)
    nb = P.num_blocks(shape)
    k_sel = P.topk_count(nb, keep)
    scores = P.block_score(q, k, shape)
    idx, mask = P.route(scores, k_sel, seed, amp)
    out, lse = P.sparse_attn_fwd(q, k, v, shape, idx, mask, want_lse=True)
    torch.cuda.synchronize()
    return out, lse, idx


CASES = [
    # grid, heads, d, block, group, keep
    ((4, 16, 16), 2, 64, 64, 32, 0.25),     # the tiny workload
    ((4, 16, 16), 2, 128, 64, 32, 0.25),
    ((5, 21, 13), 2, 128, 64, 32, 0.2),     # n=1365: 22 blocks, tail of 21 tokens
    ((9, 20, 23), 1, 128, 64, 32, 0.15),    # n=4140: 65 blocks (3 chunks, last group 1 block), tail 44
    ((9, 20, 23), 1, 128, 128, 32, 0.1),    # block 128: 33 blocks, tail 44 (< 64: second half-tile empty)
    ((9, 20, 23), 1, 128, 64, 0, 0.15),     # approximation off
    ((9, 20, 23), 1, 128, 64, 1000, 0.15),  # one global matrix (Eq.6/Eq.7)
    ((9, 20, 23), 1, 128, 64, 64, 0.15),    # 64 blocks per group
    ((9, 20, 23), 1, 128, 64, 8, 0.15),     # small groups
    ((9, 20, 23), 1, 128, 64, 1, 0.05),     # per-block first-order term (Eq.13)
    ((9, 20, 23), 1, 64, 128, 32, 0.1),
    ((1, 5, 7), 1, 128, 64, 32, 1.0),       # n=35: shorter than one tile
    ((1, 9, 11), 2, 64, 64, 32, 0.5),       # n=99: two blocks, the second one ragged; one block each selected
    ((2, 16, 16), 1, 128, 64, 32, 0.3),     # n=512: no ragged tile at all
    ((1, 9, 11), 1, 128, 128, 32, 1.0),     # n=99 with 128-token blocks: a single block, its second tile ragged
    ((12, 30, 33), 1, 128, 64, 32, 0.1),    # n=11880: 186 blocks = 6 chunks (5 of them whole), tail of 40 tokens
    ((12, 30, 32), 1, 64, 64, 64, 0.1),     # n=11520: 180 blocks, groups of two chunks, head dimension 64
    ((12, 30, 32), 1, 128, 128, 32, 0.1),   # 90 blocks of 128 tokens: 3 chunks
]


@pytest.mark.parametrize("block", [64, 128])
@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 127, 128, 129, 191, 192, 193, 257, 320])
def test_sequence_lengths_around_tile_and_block_boundaries(P, n, block):
    """every length around a multiple of 64 and of 128, dense and sparse (one of two, or two of three blocks kept)"""
    q, k, v = _inputs((1, 1, n), 1, 128, seed=n)
    shape = P.Shape.of(q, block=block, group=32)
    out = P.attn_dense_ref(q, k, v, shape)
    torch.cuda.synchronize()
    assert_close(to_f64(out), oracle.dense_attention(to_f64(q), to_f64(k), to_f64(v)), what=f"dense n={n}")
    out, lse, idx = _run_sparse(P, q, k, v, block, 32, 0.6)
    res = oracle.pasa_attention(to_f64(q), to_f64(k), to_f64(v), idx.cpu().numpy(), block, group=32, return_all=True)
    assert_close(to_f64(out), res["o"], what=f"sparse n={n} b={block}")
    np.testing.assert_allclose(lse.cpu().numpy(), res["lse"], atol=2e-2)


def test_sparse_path_respects_strides_batch_and_scale(P):
    """Q, K, V and O as views of token-major storage [B, n, H, d + pad] (what a transformer block hands over),
    batch 2, a non-default logit scale: every stage reads through the strides of the shape"""
    q, k, v = _inputs((5, 21, 13), 3, 128, seed=13, batch=2)
    B, H, n, d = q.shape
    big = torch.zeros((4, B, n, H, d + 8), dtype=torch.bfloat16, device="cuda")
    for i, t in enumerate((q, k, v)):
        big[i, :, :, :, :d] = t.permute(0, 2, 1, 3)
    qs, ks, vs, out = (big[i, :, :, :, :d].permute(0, 2, 1, 3) for i in range(4))
    scale = 0.07
    shape = P.Shape.of(qs, block=64, group=32, scale=scale)
    nb = P.num_blocks(shape)
    k_sel = P.topk_count(nb, 0.2)
    scores = P.block_score(qs, ks, shape)
    idx, mask = P.route(scores, k_sel, 77, 0.2)
    P.sparse_attn_fwd(qs, ks, vs, shape, idx, mask, out=out)
    torch.cuda.synchronize()
    ref_scores = oracle.block_scores(to_f64(q), to_f64(k), 64, scale=scale)
    np.testing.assert_allclose(scores.cpu().numpy(), ref_scores, atol=1e-3 * np.abs(ref_scores).max(), rtol=0)
    np.testing.assert_array_equal(idx.cpu().numpy(), oracle.route(scores.cpu().numpy(), k_sel, 77, 0.2))
    res = oracle.pasa_attention(to_f64(q), to_f64(k), to_f64(v), idx.cpu().numpy(), 64, group=32, scale=scale)
    assert_close(to_f64(out), res, what="strided sparse path")
    assert torch.all(big[3, :, :, :, d:] == 0)  # the padding between rows was not written


@pytest.mark.parametrize("grid,heads,d,block,group,keep", CASES)
def test_sparse_matches_oracle(P, grid, heads, d, block, group, keep):
    q, k, v = _inputs(grid, heads, d, seed=7)
    out, lse, idx = _run_sparse(P, q, k, v, block, group, keep)
    res = oracle.pasa_attention(to_f64(q), to_f64(k), to_f64(v), idx.cpu().numpy(), block, group=group,
                                return_all=True)
    assert_close(to_f64(out), res["o"], what=f"sparse {grid} d={d} b={block} G={group}")
    np.testing.assert_allclose(lse.cpu().numpy(), res["lse"], atol=2e-2)


SLICED_CASES = [
    # grid, d, block, group, keep, kv_slices   (needs at least kv_slices chunks of 32 key blocks)
    ((8, 45, 46), 128, 64, 32, 0.15, 8),    # n=16,560: 259 blocks (tail 48), 9 chunks over 8 slices
    ((8, 45, 46), 128, 64, 0, 0.02, 8),     # approximation off, very sparse: some slices hold no selected block
    ((12, 40, 46), 64, 64, 32, 0.1, 8),     # d = 64
    ((16, 40, 52), 128, 64, 32, 0.05, 16),  # n=33,280: 520 blocks, 17 chunks over 16 slices (two rounds per XCD)
    ((16, 40, 52), 128, 128, 32, 0.1, 8),   # block 128: 260 blocks, 9 chunks
]


@pytest.mark.parametrize("grid,d,block,group,keep,kv_slices", SLICED_CASES)
def test_key_range_slicing_matches_oracle_and_unsliced_kernel(P, grid, d, block, group, keep, kv_slices):
    q, k, v = _inputs(grid, 1, d, seed=13)
    out, lse, idx = _run_sparse(P, q, k, v, block, group, keep, kv_slices=kv_slices)
    out1, lse1, idx1 = _run_sparse(P, q, k, v, block, group, keep, kv_slices=1)
    assert torch.equal(idx, idx1)
    # same arithmetic up to summation order and one bf16 rounding
    a, b = out.float(), out1.float()
    assert (a - b).abs().max().item() <= 2e-2 * b.abs().max().item()
    assert (a - b).abs().mean().item() <= 1e-3 * b.abs().mean().item()
    np.testing.assert_allclose(lse.cpu().numpy(), lse1.cpu().numpy(), atol=1e-3)
    res = oracle.pasa_attention(to_f64(q), to_f64(k), to_f64(v), idx.cpu().numpy(), block, group=group,
                                return_all=True)
    assert_close(to_f64(out), res["o"], what=f"sliced {grid} d={d} b={block} G={group} S={kv_slices}")
    np.testing.assert_allclose(lse.cpu().numpy(), res["lse"], atol=2e-2)


def test_keep_everything_equals_dense_kernel_and_oracle(P):
    q, k, v = _inputs((5, 21, 13), 2, 128, seed=2)
    out, _, idx = _run_sparse(P, q, k, v, 64, 32, 1.0)
    assert idx.shape[-1] == 22
    ref = oracle.dense_attention(to_f64(q), to_f64(k), to_f64(v))
    assert_close(to_f64(out), ref, what="keep=1")
    dense = P.attn_dense_ref(q, k, v, P.Shape.of(q))
    torch.cuda.synchronize()
    assert_close(to_f64(out), to_f64(dense).astype(np.float64), what="keep=1 vs dense kernel")


def test_batch_and_heads_are_independent_and_results_are_deterministic(P):
    q, k, v = _inputs((3, 16, 16), 3, 128, seed=11, batch=2)
    out, _, idx = _run_sparse(P, q, k, v, 64, 32, 0.25)
    out2, _, idx2 = _run_sparse(P, q, k, v, 64, 32, 0.25)
    assert torch.equal(out, out2) and torch.equal(idx, idx2)  # bitwise run-to-run
    # batch 1, head 2 alone (routing noise is keyed by bh, so feed the same routing rows)
    shape1 = P.Shape.of(q[1:2, 2:3], block=64, group=32)
    bh = 1 * 3 + 2
    nb = idx.shape[1]
    mask = torch.zeros((1, nb, (nb + 31) // 32), dtype=torch.int32, device="cuda")
    words = np.zeros((nb, (nb + 31) // 32), np.uint32)
    for i, row in enumerate(idx[bh].cpu().numpy()):
        for j in row:
            words[i, j >> 5] |= np.uint32(1) << np.uint32(j & 31)
    mask[0] = torch.from_numpy(words.view(np.int32)).cuda()
    single = P.sparse_attn_fwd(q[1:2, 2:3], k[1:2, 2:3], v[1:2, 2:3], shape1, idx[bh:bh + 1].contiguous(), mask)
    torch.cuda.synchronize()
    assert torch.equal(single[0, 0], out[1, 2])
    ref = oracle.pasa_attention(to_f64(q), to_f64(k), to_f64(v), idx.cpu().numpy(), 64, group=32)
    assert_close(to_f64(out), ref, what="batch=2")


@pytest.mark.parametrize("grid,d,block,group,keep", [((4, 16, 16), 64, 64, 32, 0.25), ((9, 20, 23), 128, 64, 32, 0.15),
                                                     ((9, 20, 23), 128, 128, 8, 0.3), ((5, 21, 13), 128, 64, 0, 0.2)])
def test_single_call_forward_equals_the_stage_calls(P, grid, d, block, group, keep):
    """pasa_forward against the four stage entry points (bit for bit: the same kernels in the same order) and the oracle"""
    q, k, v = _inputs(grid, 2, d, seed=31)
    shape = P.Shape.of(q, block=block, group=group)
    nb = P.num_blocks(shape)
    k_sel = P.topk_count(nb, keep)
    out, lse = P.forward_single_call(q, k, v, shape, keep, 123, 0.2, want_lse=True)
    ws = P.kv_stats(k, v, shape)
    scores = P.block_score(q, None, shape, stats_ws=ws) if group > 0 else P.block_score(q, k, shape)
    idx, mask = P.route(scores, k_sel, 123, 0.2)
    want, want_lse = P.sparse_attn_fwd(q, k, v, shape, idx, mask, ws=ws, prepared=True, want_lse=True)
    torch.cuda.synchronize()
    assert torch.equal(out, want) and torch.equal(lse, want_lse)
    ref = oracle.pasa_attention(to_f64(q), to_f64(k), to_f64(v), idx.cpu().numpy(), block, group=group)
    assert_close(to_f64(out), ref, what="pasa_forward")


def test_forward_convenience_wrapper(P):
    q, k, v = _inputs((4, 16, 16), 2, 64)
    out, idx = P.forward(q, k, v, keep_ratio=0.25, seed=5, noise_amp=0.2)
    torch.cuda.synchronize()
    ref = oracle.pasa_attention(to_f64(q), to_f64(k), to_f64(v), idx.cpu().numpy(), 64, group=32)
    assert_close(to_f64(out), ref, what="forward()")


# ------------------------------------------------------------------------------------------------
# calibration signal of the curvature-aware budget: mean L1 distance of two tensors
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,dtype", [(1, torch.float32), (7, torch.bfloat16), (4096, torch.bfloat16), (1000003, torch.float32),
                                     (16 * 21 * 45 * 80 + 5, torch.bfloat16), (64 * 1024 * 1024, torch.bfloat16)])
def test_l1_distance_matches_oracle_and_is_deterministic(P, n, dtype):
    g = torch.Generator("cuda").manual_seed(n % 1000)
    a = torch.randn(n, device="cuda", generator=g).to(dtype)
    b = (a.float() + 0.3 * torch.randn(n, device="cuda", generator=g)).to(dtype)
    got = P.l1_distance(a, b)
    again = P.l1_distance(a, b)
    torch.cuda.synchronize()
    want = oracle.l1_distance(a.float().cpu().numpy(), b.float().cpu().numpy())
    assert abs(got.item() - want) <= 2e-6 * want + 1e-12
    assert got.item() == again.item()
    assert P.l1_distance(a, a).item() == 0.0


# ------------------------------------------------------------------------------------------------
# the whole path on a side stream and inside a HIP graph (launch-bound serving loops capture it)
# ------------------------------------------------------------------------------------------------
def test_forward_on_a_side_stream_and_in_a_graph_replays_identically(P):
    q, k, v = _inputs((9, 20, 23), 2, 128, seed=21)
    shape = P.Shape.of(q, block=64, group=32)
    nb = P.num_blocks(shape)
    k_sel = P.topk_count(nb, 0.15)
    scores = torch.empty((2, nb, nb), dtype=torch.float32, device="cuda")
    idx = torch.empty((2, nb, k_sel), dtype=torch.int32, device="cuda")
    mask = torch.empty((2, nb, P.mask_words(nb)), dtype=torch.int32, device="cuda")
    ws_s = torch.empty(P.score_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    ws_a = torch.empty(P.attn_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(q)

    def run():
        P.block_score(q, k, shape, scores=scores, ws=ws_s)
        P.route(scores, k_sel, 99, 0.125, idx=idx, mask=mask)
        P.sparse_attn_fwd(q, k, v, shape, idx, mask, out=out, ws=ws_a)

    run()
    torch.cuda.synchronize()
    eager = out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        out.zero_()
        run()
    side.synchronize()
    assert torch.equal(out, eager)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for _ in range(3):
        out.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager)
        (out.float().sum()).item()  # eager work between the replays


# ------------------------------------------------------------------------------------------------
# the method-variant tables (group sizes, routing noise, selection-count histogram) on the tiny workload
# ------------------------------------------------------------------------------------------------
def _table_rows(text):
    rows = [[c.strip() for c in line.strip().strip("|").split("|")] for line in text.splitlines() if line.startswith("|")]
    return [r for r in rows if not set("".join(r)) <= set("-")]  # without the separator rows


def test_sweep_tables_on_the_tiny_workload(P, capsys):
    import paper_2604_12219_amd.sweeps as sweeps
    sweeps.selection_histogram("tiny", 6, 1.0)  # a bias as large as the logit spread of this small workload
    rows = _table_rows(capsys.readouterr().out)
    assert [r[0] for r in rows[1:]] == ["deterministic", "stochastic, uniform bias", "stochastic, Gumbel bias"]
    pct = lambda s: float(s.rstrip("%"))
    for r in rows[1:]:
        assert abs(pct(r[1]) + pct(r[2]) + pct(r[3]) + pct(r[4]) - 100.0) < 0.5   # the four classes partition the pairs
        assert abs(pct(r[1]) + pct(r[5]) - 100.0) < 0.2                           # never + ever = all
    det, sto = rows[1], rows[2]
    assert pct(sto[5]) > pct(det[5])          # the seeded bias spreads the exact computation over more pairs ...
    assert float(sto[6]) < float(det[6])      # ... each of which is selected in fewer steps
    sweeps.sweep_noise("tiny")
    rows = _table_rows(capsys.readouterr().out)
    changed = [pct(r[1]) for r in rows[1:]]
    assert changed[0] == 0.0 and all(a <= b + 1e-9 for a, b in zip(changed, changed[1:])) and changed[-1] > 5.0
    sweeps.sweep_groups("tiny", 0.125, 1.0)
    rows = _table_rows(capsys.readouterr().out)
    assert [r[0] for r in rows[1:]] == ["0 (drop)", "1 (per block)", "16 (global)"] or rows[1][0] == "0 (drop)"
    errs = {r[0]: float(r[5]) for r in rows[1:]}
    assert errs["0 (drop)"] > errs["1 (per block)"]  # the approximation of the unselected blocks pays


# ------------------------------------------------------------------------------------------------
# seeded random configurations: shapes, strides, block and group sizes, keep ratios drawn at random
# ------------------------------------------------------------------------------------------------
def _random_config(rng):
    d = int(rng.choice([64, 128]))
    block = int(rng.choice([64, 128]))
    n = int(rng.integers(1, 2600))
    nb = (n + block - 1) // block
    group = int(rng.choice([0, 1, 2, 4, 8, 16, 32, 64, 10_000]))
    keep = float(rng.choice([0.02, 0.1, 0.25, 0.5, 0.9, 1.0]))
    heads, batch = int(rng.integers(1, 4)), int(rng.integers(1, 3))
    token_major = bool(rng.integers(0, 2))
    scale = float(rng.choice([0.0, 0.05, 0.2]))
    return dict(d=d, block=block, n=n, nb=nb, group=group, keep=keep, heads=heads, batch=batch, token_major=token_major, scale=scale)


@pytest.mark.parametrize("case", range(24))
def test_random_configurations_against_oracle(P, case):
    rng = np.random.default_rng(1000 + case)
    c = _random_config(rng)
    q, k, v = workloads.make_qkv((1, 1, c["n"]), c["heads"], c["d"], seed=case, device="cuda", batch=c["batch"])
    if c["token_major"]:
        q, k, v = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (q, k, v))
    shape = P.Shape.of(q, block=c["block"], group=c["group"], scale=c["scale"])
    k_sel = P.topk_count(c["nb"], c["keep"])
    scale = c["scale"] if c["scale"] > 0 else None
    ws = P.kv_stats(k, v, shape)
    scores = P.block_score(q, None, shape, stats_ws=ws) if c["group"] > 0 else P.block_score(q, k, shape)
    idx, mask = P.route(scores, k_sel, 7 * case + 1, 0.3)
    out, lse = P.sparse_attn_fwd(q, k, v, shape, idx, mask, want_lse=True)
    dense = P.attn_dense_ref(q, k, v, shape)
    torch.cuda.synchronize()
    what = f"case {case}: {c}"
    assert P.check_selection(idx, mask, c["nb"], k_sel).item() == 0, what
    ref_scores = oracle.block_scores(to_f64(q), to_f64(k), c["block"], scale=scale)
    np.testing.assert_allclose(scores.cpu().numpy(), ref_scores, atol=1e-3 * max(np.abs(ref_scores).max(), 1e-3), rtol=0, err_msg=what)
    np.testing.assert_array_equal(idx.cpu().numpy(), oracle.route(scores.cpu().numpy(), k_sel, 7 * case + 1, 0.3), err_msg=what)
    res = oracle.pasa_attention(to_f64(q), to_f64(k), to_f64(v), idx.cpu().numpy(), c["block"], group=c["group"], scale=scale,
                                return_all=True)
    assert_close(to_f64(out), res["o"], what=what)
    np.testing.assert_allclose(lse.cpu().numpy(), res["lse"], atol=2e-2, err_msg=what)
    assert_close(to_f64(dense), oracle.dense_attention(to_f64(q), to_f64(k), to_f64(v), scale=scale), what="dense, " + what)
