"""The seeded input generator: shapes, determinism, structure. CPU only."""
import torch

import workloads


def test_shapes_of_the_named_workloads():
    w = workloads.WORKLOADS
    assert (w["tiny"].n, w["tiny"].n_blocks) == (1024, 16)
    assert (w["wan1.3b-480p"].n, w["wan1.3b-480p"].n_blocks) == (32760, 512)
    assert (w["wan14b-720p"].n, w["wan14b-720p"].n_blocks) == (75600, 1182)  # 75,600 tokens at 720p
    assert (w["long-video"].n, w["long-video"].n_blocks) == (147600, 1154)


def test_generator_is_seeded_per_head_and_bf16():
    q, k, v = workloads.make_qkv((3, 6, 8), 3, 16, seed=5)
    assert q.shape == (1, 3, 144, 16) and q.dtype == torch.bfloat16
    q2, k2, v2 = workloads.make_qkv((3, 6, 8), [2], 16, seed=5)
    assert torch.equal(q2[0, 0], q[0, 2]) and torch.equal(k2[0, 0], k[0, 2]) and torch.equal(v2[0, 0], v[0, 2])
    q3, _, _ = workloads.make_qkv((3, 6, 8), 3, 16, seed=6)
    assert not torch.equal(q3, q)


def test_q_and_k_share_a_smooth_field():
    q, k, v = workloads.make_qkv((4, 16, 16), 1, 32, seed=0)
    qf, kf, vf = q.float()[0, 0], k.float()[0, 0], v.float()[0, 0]
    # unit white noise + unit-variance field => variance about 2
    assert 1.6 < qf.var().item() < 2.4
    corr_qk = (qf * kf).mean().item()
    corr_qv = (qf * vf).mean().item()
    assert corr_qk > 0.7 and abs(corr_qv) < 0.15
    # neighbouring tokens along a row are correlated through the field
    assert (qf[:-1] * qf[1:]).mean().item() > 0.5


def test_budget_schedule_curves():
    ks = [workloads.budget_schedule_keep_ratio(s) for s in range(50)]
    assert abs(max(ks) - 0.4) < 1e-12 and ks.index(max(ks)) == 15
    assert min(ks) >= 0.1 and ks[49] < 0.1001
    assert workloads.budget_schedule_noise_amplitude(0) == 1.0
    assert abs(workloads.budget_schedule_noise_amplitude(49) - 0.2) < 1e-12
