"""GPU parity at the full workload sizes, in the launch configuration bench.py times (all heads at
once): sampled query blocks of sampled heads are compared with the oracle one by one; routing is
compared bit for bit on those heads."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from _util import assert_close, to_f64

pytestmark = pytest.mark.gpu

NOISE_AMP = 0.125  # the benchmark's setting


@pytest.fixture(scope="module")
def P():
    import paper_2604_12219_amd as P
    assert torch.cuda.is_available(), "these tests need the MI355X"
    P.load_library()
    return P


def _sample_blocks(nb, rng, extra=4):
    fixed = {0, 1, nb // 2, nb // 2 + 1, nb - 2, nb - 1}  # both members of the first, a middle and the last pair; ragged tail
    fixed |= set(int(x) for x in rng.choice(nb, extra, replace=False))
    return sorted(fixed)


@pytest.mark.parametrize("name,heads_checked", [("wan1.3b-480p", (0, 11)), ("wan14b-720p", (0, 39)), ("long-video", (17,)),
                                                ("long-video-b64", (1,)), ("hunyuan13b-720p", (23,))])
def test_full_size_workload_sampled_against_oracle(P, name, heads_checked):
    w = workloads.WORKLOADS[name]
    q, k, v = workloads.make_workload_qkv(w, device="cuda")
    shape = P.Shape.of(q, block=w.block, group=32)
    nb = P.num_blocks(shape)
    k_sel = P.topk_count(nb, w.keep_ratio)
    assert (nb, k_sel) == {"wan1.3b-480p": (512, 102), "wan14b-720p": (1182, 177), "long-video": (1154, 58),
                             "long-video-b64": (2307, 69), "hunyuan13b-720p": (1857, 279)}[name]
    scores = P.block_score(q, k, shape)
    idx, mask = P.route(scores, k_sel, w.seed, NOISE_AMP)
    out, lse = P.sparse_attn_fwd(q, k, v, shape, idx, mask, want_lse=True)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    for h in heads_checked:
        qh, kh, vh = (to_f64(t[:, h:h + 1]) for t in (q, k, v))
        # stage 1: scores of this head
        ref_scores = oracle.block_scores(qh, kh, w.block)
        got_scores = scores[h:h + 1].cpu().numpy()
        np.testing.assert_allclose(got_scores, ref_scores, atol=1e-3 * np.abs(ref_scores).max(), rtol=0)
        # stage 2: routing, bit for bit, from the GPU's scores
        want_idx = oracle.route(got_scores, k_sel, w.seed, NOISE_AMP, bh_ids=[h])
        np.testing.assert_array_equal(idx[h:h + 1].cpu().numpy(), want_idx)
        # for information: the oracle routing on its OWN fp64 scores (rounded to binary32) -- rows whose selection
        # differs from the GPU's do so because a score within rounding distance of the k-th largest fell on the other side
        own_idx = oracle.route(ref_scores.astype(np.float32), k_sel, w.seed, NOISE_AMP, bh_ids=[h])
        rows_differ = float(np.mean(np.any(own_idx != want_idx, axis=-1)))
        print(f"{name} head {h}: {rows_differ:.2%} of the routing rows differ when the oracle routes on its own scores")
        assert rows_differ < 0.01
        # stages 3+4 on sampled query blocks
        blocks = _sample_blocks(nb, rng)
        res = oracle.pasa_attention(qh, kh, vh, want_idx, w.block, group=32, q_blocks=blocks, return_all=True)
        rows = np.concatenate([np.arange(j * w.block, min((j + 1) * w.block, w.n)) for j in blocks])
        assert_close(to_f64(out[:, h:h + 1]), res["o"], rows=rows, what=f"{name} head {h}")
        np.testing.assert_allclose(lse[h].cpu().numpy()[rows], res["lse"][0, rows], atol=2e-2)
        np.testing.assert_allclose(res["wsum"][0, rows].sum(-1), 1.0, atol=1e-12)
    # rows past the end do not exist; nothing else to check there.  Run-to-run determinism at full size:
    out2 = P.sparse_attn_fwd(q, k, v, shape, idx, mask)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


def test_full_size_dense_reference_sampled_against_oracle(P):
    w = workloads.WORKLOADS["wan14b-720p"]
    q, k, v = workloads.make_workload_qkv(w, device="cuda", heads=[3, 4])
    shape = P.Shape.of(q, block=w.block)
    out, lse = P.attn_dense_ref(q, k, v, shape, want_lse=True)
    torch.cuda.synchronize()
    rows = np.concatenate([np.arange(0, 40), np.arange(37_000, 37_040), np.arange(w.n - 40, w.n)]).astype(np.int32)
    ref, ref_lse = oracle.dense_attention(to_f64(q), to_f64(k), to_f64(v), q_rows=rows, return_lse=True)
    got = to_f64(out)[:, rows]
    assert_close(got, ref, what="dense 75,600 tokens")
    np.testing.assert_allclose(lse.cpu().numpy()[:, rows], ref_lse, atol=2e-2)


@pytest.mark.parametrize("name,head", [("wan14b-720p", 20), ("long-video", 33), ("wan1.3b-480p", 7)])
def test_whole_head_of_a_full_size_workload_against_oracle(P, name, head):
    """Every query block of one head in the middle of the launch, all heads launched as bench.py launches them: covers
    every slot of the kernel's workgroup-id decode for that head and the ragged last query tile (two 64-token query
    blocks per workgroup at the 14B and 480p shapes, one 128-token block at the long-video shape).  Routing bit for
    bit, output and lse row by row."""
    w = workloads.WORKLOADS[name]
    q, k, v = workloads.make_workload_qkv(w, device="cuda")
    shape = P.Shape.of(q, block=w.block, group=32)
    nb = P.num_blocks(shape)
    k_sel = P.topk_count(nb, w.keep_ratio)
    scores = P.block_score(q, k, shape)
    idx, mask = P.route(scores, k_sel, w.seed, NOISE_AMP)
    out, lse = P.sparse_attn_fwd(q, k, v, shape, idx, mask, want_lse=True)
    torch.cuda.synchronize()
    qh, kh, vh = (to_f64(t[:, head:head + 1]) for t in (q, k, v))
    got_scores = scores[head:head + 1].cpu().numpy()
    want_idx = oracle.route(got_scores, k_sel, w.seed, NOISE_AMP, bh_ids=[head])
    np.testing.assert_array_equal(idx[head:head + 1].cpu().numpy(), want_idx)
    res = oracle.pasa_attention(qh, kh, vh, want_idx, w.block, group=32, return_all=True)
    got = to_f64(out[:, head:head + 1])
    assert_close(got, res["o"], what=f"{name} whole head {head}")
    np.testing.assert_allclose(lse[head].cpu().numpy(), res["lse"][0], atol=2e-2)
    # no query tile is off by more than the others: the per-tile errors stay within the same bounds
    err = np.abs(got[0] - res["o"][0])
    scale = np.abs(res["o"][0]).max()
    per_tile = [err[t:t + 128].max() / scale for t in range(0, w.n, 128)]
    assert max(per_tile) <= 2e-2, (int(np.argmax(per_tile)), max(per_tile))


BUDGET_STEPS = (0, 7, 14, 15, 21, 28, 35, 42, 49)  # every 7th step, the peak of the schedule (15) and its last step


def test_budget_schedule_runs_with_runtime_k(P):
    """keep ratio and noise amplitude change per denoising step, nothing is recompiled or re-allocated: the buffers are
    allocated once for the largest k of the schedule and every step runs in them"""
    w = workloads.WORKLOADS["wan1.3b-480p"]
    heads = [0, 1]
    nb = w.n_blocks
    ks = [P.topk_count(nb, workloads.budget_schedule_keep_ratio(s)) for s in range(50)]
    assert min(ks) == 51 and max(ks) == 205 and ks[0] == 51 and ks[15] == 205 and ks[49] == 51
    k_max = max(ks)
    scores = torch.empty((len(heads), nb, nb), dtype=torch.float32, device="cuda")
    idx_buf = torch.empty(len(heads) * nb * k_max, dtype=torch.int32, device="cuda")
    mask = torch.empty((len(heads), nb, P.mask_words(nb)), dtype=torch.int32, device="cuda")
    ws_score = ws_attn = out = None
    for step in BUDGET_STEPS:
        amp_in = workloads.budget_schedule_noise_amplitude(step)
        q, k, v = workloads.make_workload_qkv(w, device="cuda", heads=heads, noise_amplitude=amp_in, seed=w.seed + step)
        shape = P.Shape.of(q, block=w.block, group=32)
        k_sel = ks[step]
        if ws_score is None:
            ws_score = torch.empty(P.score_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
            ws_attn = torch.empty(P.attn_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
            out = torch.empty_like(q)
        idx = idx_buf[: len(heads) * nb * k_sel].view(len(heads), nb, k_sel)
        P.block_score(q, k, shape, scores=scores, ws=ws_score)
        P.route(scores, k_sel, w.seed + step, NOISE_AMP, idx=idx, mask=mask)
        P.sparse_attn_fwd(q, k, v, shape, idx, mask, out=out, ws=ws_attn)
        torch.cuda.synchronize()
        want_idx = oracle.route(scores[:1].cpu().numpy(), k_sel, w.seed + step, NOISE_AMP, bh_ids=[0])
        np.testing.assert_array_equal(idx[:1].cpu().numpy(), want_idx)
        blocks = [0, 257, nb - 1]
        res = oracle.pasa_attention(to_f64(q[:, :1]), to_f64(k[:, :1]), to_f64(v[:, :1]), want_idx, w.block,
                                    group=32, q_blocks=blocks)
        rows = np.concatenate([np.arange(j * w.block, min((j + 1) * w.block, w.n)) for j in blocks])
        assert_close(to_f64(out[:, :1]), res, rows=rows, what=f"budget step {step}")


def test_full_size_key_prior_of_one_head_against_oracle(P):
    """covariance-aware routing prior at the Wan-14B 720p shape: every block of one head, and the timing printed"""
    w = workloads.WORKLOADS["wan14b-720p"]
    q, k, v = workloads.make_workload_qkv(w, device="cuda")
    shape = P.Shape.of(q, block=w.block, group=32)
    ws = P.kv_stats(k, v, shape)
    beta = P.key_prior(k, v, shape, ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(3):
        P.key_prior(k, v, shape, ws, beta=beta)
    e1.record()
    torch.cuda.synchronize()
    print(f"pasa_key_prior at wan14b-720p: {e0.elapsed_time(e1) / 3:.3f} ms")
    head = 23
    ref = oracle.key_prior(to_f64(k[:, head:head + 1]), to_f64(v[:, head:head + 1]), w.block, 32)
    np.testing.assert_allclose(beta.cpu().numpy()[head], ref[0], atol=2e-3, rtol=0)
