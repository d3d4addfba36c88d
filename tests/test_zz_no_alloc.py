"""pasa_sparse_attn_fwd_static, the entry point that allocates nothing, against pasa_sparse_attn_fwd through the
C ABI: two calls in a row on the same GPU, the second on a smaller input (the static scratch keeps the first
call's contents), each compared with the workspace-taking entry point and with the oracle."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import workloads
from _util import assert_close, to_f64

pytestmark = pytest.mark.gpu


def _case(P, grid, heads, d, block, group, keep, seed):
    q, k, v = workloads.make_qkv(grid, heads, d, seed=seed, device="cuda")
    shape = P.Shape.of(q, block=block, group=group)
    nb = P.num_blocks(shape)
    k_sel = P.topk_count(nb, keep)
    scores = P.block_score(q, k, shape)
    idx, mask = P.route(scores, k_sel, seed, 0.1)
    return q, k, v, shape, idx, mask


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    import paper_2604_12219_amd as P
    assert torch.cuda.is_available(), "this test needs the MI355X"
    L = P.load_library()
    # first a case of several tiles per head with a ragged tail, then a smaller one of another head dimension
    cases = [_case(P, (9, 20, 23), 3, 128, 64, 32, 0.2, 3), _case(P, (4, 16, 16), 2, 64, 64, 32, 0.25, 4)]
    assert P.attn_workspace_bytes(cases[0][3]) > P.attn_workspace_bytes(cases[1][3])
    for q, k, v, shape, idx, mask in cases:
        assert P.attn_workspace_bytes(shape) <= P.STATIC_SCRATCH_BYTES
        want, want_lse = P.sparse_attn_fwd(q, k, v, shape, idx, mask, want_lse=True)
        out = torch.full_like(q, float("nan"))
        lse = torch.full((shape.B * shape.H, shape.n), float("nan"), dtype=torch.float32, device="cuda")
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        rc = L.pasa_sparse_attn_fwd_static(ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(k.data_ptr()), ctypes.c_void_p(v.data_ptr()),
                                           ctypes.byref(shape.c()), ctypes.c_void_p(idx.data_ptr()), ctypes.c_void_p(mask.data_ptr()),
                                           idx.shape[-1], ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(lse.data_ptr()), stream)
        assert rc == 0, L.pasa_strerror(rc)
        torch.cuda.synchronize()
        # same kernels, same inputs, fixed summation order: the two entry points agree to the last bit ...
        assert torch.equal(out, want) and torch.equal(lse, want_lse)
        # ... and with the oracle within the tolerance of every parity test
        ref = oracle.pasa_attention(to_f64(q), to_f64(k), to_f64(v), idx.cpu().numpy(), shape.block, group=shape.group, return_all=True)
        assert_close(to_f64(out), ref["o"], what="static scratch")
        np.testing.assert_allclose(lse.cpu().numpy(), ref["lse"], atol=2e-2)
    # the binding's wrapper takes the same route
    q, k, v, shape, idx, mask = cases[0]
    out = P.sparse_attn_fwd_static(q, k, v, shape, idx, mask, torch.empty_like(q))
    torch.cuda.synchronize()
    assert torch.equal(out, P.sparse_attn_fwd(q, k, v, shape, idx, mask))
