"""The C ABI without a GPU: the library loads, exports every symbol the header declares, and its
host-side helpers and argument validation behave as documented (validation happens before any
launch, so these calls never touch a device)."""
import ctypes
import os
import re

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pasa.h")


@pytest.fixture(scope="module")
def P():
    import paper_2604_12219_amd as P
    if not os.path.exists(P.lib_path()):
        from paper_2604_12219_amd.build import build
        build()
    P.load_library()
    return P


def declared_symbols():
    text = open(HEADER).read()
    return sorted(set(re.findall(r"PASA_API\s+[\w\s\*]+?\b(pasa_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported(P):
    names = declared_symbols()
    assert {"pasa_block_score", "pasa_route", "pasa_route_gumbel", "pasa_sparse_attn_fwd", "pasa_attn_dense_ref", "pasa_kv_stats",
            "pasa_sparse_attn_fwd_prepared", "pasa_topk_count", "pasa_strerror"} <= set(names)
    lib = ctypes.CDLL(P.lib_path())
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in pasa.h but not exported"
    from paper_2604_12219_amd.pasa import EXPORTS
    assert set(EXPORTS) == set(names)
    # ... and nothing else is: the dynamic symbol table holds exactly the declared entry points
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", P.lib_path()], capture_output=True, text=True, check=True).stdout
    exported = {l.split()[-1] for l in out.splitlines() if " T " in l and l.split()[-1].startswith("pasa_")}
    assert exported == set(names), exported ^ set(names)


def test_product_has_no_cpu_fallback_and_does_not_import_the_oracle():
    src = ""
    pkg = os.path.join(ROOT, "paper_2604_12219_amd")
    for f in os.listdir(pkg):
        if f.endswith(".py"):
            src += open(os.path.join(pkg, f)).read()
    assert "import oracle" not in src and "from oracle" not in src
    assert "There is no CPU fallback" in src


def test_topk_count_matches_the_oracle_rule_and_rejects_bad_ratios(P):
    for nb in (1, 7, 16, 512, 1182, 1154):
        for keep in (1e-6, 0.05, 0.15, 0.2, 0.25, 0.5, 0.999, 1.0):
            assert P.topk_count(nb, keep) == oracle.topk_count(nb, keep)
    for bad in (0.0, -0.1, 1.0001, float("nan")):
        with pytest.raises(P.PasaError):
            P.topk_count(100, bad)
    with pytest.raises(P.PasaError):
        P.topk_count(0, 0.5)


def _shape(P, **kw):
    base = dict(B=1, H=2, n=8192, d=128, block=64, group=32, stride_n=128)
    base.update(kw)
    base.setdefault("stride_h", max(base["n"], 1) * base["stride_n"])
    base.setdefault("stride_b", base["H"] * base["stride_h"])
    return P.Shape(**base)


def test_shape_helpers_and_workspace_sizes(P):
    s = _shape(P)
    assert P.num_blocks(s) == 128 and P.mask_words(16) == 1 and P.mask_words(1182) == 37
    assert P.num_blocks(_shape(P, n=1000)) == 16  # ragged tail
    assert P.score_workspace_bytes(s) >= 2 * 2 * 128 * 128 * 4
    assert P.attn_workspace_bytes(_shape(P, group=4096)) > 0  # at least N_B blocks per group: one global matrix
    assert P.attn_workspace_bytes(s) > 0
    assert P.attn_workspace_bytes(_shape(P, group=0)) > 0
    # invalid shapes report 0 bytes
    assert P.attn_workspace_bytes(_shape(P, d=96)) == 0
    assert P.attn_workspace_bytes(_shape(P, group=48)) == 0
    assert P.attn_workspace_bytes(_shape(P, kv_slices=3)) == 0
    assert P.score_workspace_bytes(_shape(P, block=32)) == 0


def test_argument_validation_returns_before_any_launch(P):
    L = P.load_library()
    good = _shape(P).c()
    fake = ctypes.c_void_p(0x1000)  # 16-byte aligned, never dereferenced: every call below fails validation first
    big = ctypes.c_size_t(1 << 40)
    EINVAL, EUNSUPPORTED, EWORKSPACE, EALIGN = -1, -2, -3, -4

    def score(shape, q=fake, k=fake, out=fake, ws=fake, nbytes=big):
        return L.pasa_block_score(q, k, ctypes.byref(shape), None, out, ws, nbytes, None)

    assert score(good, q=None) == EINVAL
    assert score(good, out=None) == EINVAL
    assert score(good, nbytes=ctypes.c_size_t(16)) == EWORKSPACE
    assert score(good, q=ctypes.c_void_p(0x1004)) == EALIGN
    assert score(_shape(P, d=96).c()) == EUNSUPPORTED
    assert score(_shape(P, block=256).c()) == EUNSUPPORTED
    assert score(_shape(P, n=0).c()) == EINVAL
    assert score(_shape(P, stride_n=100).c()) == EINVAL
    assert score(_shape(P, stride_n=132).c()) == EALIGN
    assert score(_shape(P, scale=-1.0).c()) == EINVAL

    def route(scores=fake, bh=2, nb=16, k=4, amp=0.1, idx=fake):
        return L.pasa_route(scores, bh, nb, k, 7, ctypes.c_float(amp), idx, None, None)


    assert route(scores=None) == EINVAL
    assert route(k=0) == EINVAL and route(k=17) == EINVAL
    assert route(amp=-1.0) == EINVAL and route(amp=float("inf")) == EINVAL
    assert route(nb=1 << 20, k=4) == EUNSUPPORTED
    assert L.pasa_route_gumbel(None, 2, 16, 4, 7, ctypes.c_float(0.5), fake, None, None) == EINVAL
    assert L.pasa_route_gumbel(fake, 2, 16, 0, 7, ctypes.c_float(0.5), fake, None, None) == EINVAL
    assert L.pasa_route_gumbel(fake, 2, 16, 4, 7, ctypes.c_float(-0.5), fake, None, None) == EINVAL
    assert L.pasa_route_gumbel(fake, 2, 1 << 20, 4, 7, ctypes.c_float(0.5), fake, None, None) == EUNSUPPORTED

    def sparse(shape, q=fake, idx=fake, mask=fake, k=4, out=ctypes.c_void_p(0x2000), ws=fake, nbytes=big):
        return L.pasa_sparse_attn_fwd(q, fake, fake, ctypes.byref(shape), idx, mask, k, out, None, ws, nbytes, None)

    assert sparse(good, idx=None, mask=None) == EINVAL  # one of the two may be missing, not both
    assert sparse(good, idx=ctypes.c_void_p(0x1002)) == EALIGN
    assert sparse(good, k=0) == EINVAL and sparse(good, k=129) == EINVAL
    assert sparse(good, out=fake) == EINVAL  # output aliases an input
    assert sparse(good, nbytes=ctypes.c_size_t(0)) == EWORKSPACE
    assert sparse(_shape(P, group=48).c()) == EUNSUPPORTED
    assert sparse(_shape(P, group=-1).c()) == EINVAL
    assert sparse(_shape(P, kv_slices=12).c()) == EUNSUPPORTED
    # size limits of the approximation pass: more than 65,535 groups (one block per group on a long sequence)
    assert sparse(_shape(P, n=70_000 * 64, group=1).c()) == EUNSUPPORTED
    assert P.attn_workspace_bytes(_shape(P, n=70_000 * 64, group=32)) > 0  # 70,000 blocks in groups of 32 are within the limits
    assert sparse(_shape(P, H=65_535, n=16_000_000).c()) == EUNSUPPORTED  # workgroup count beyond 32 bits

    def check(idx=fake, mask=fake, bh=2, nb=16, k=4, n_bad=fake):
        return L.pasa_check_selection(idx, mask, bh, nb, k, n_bad, None)

    assert check(idx=None, mask=None) == EINVAL and check(n_bad=None) == EINVAL
    assert check(k=0) == EINVAL and check(k=17) == EINVAL and check(bh=0) == EINVAL
    assert check(idx=ctypes.c_void_p(0x1002)) == EALIGN
    assert L.pasa_attn_dense_ref(fake, fake, fake, ctypes.byref(good), None, None, fake, big, None) == EINVAL
    assert L.pasa_kv_stats(None, fake, ctypes.byref(good), fake, big, None) == EINVAL
    # the entry point that allocates nothing: shapes beyond its static scratch are refused on the host
    ESCRATCH = -6

    def static(shape, q=fake, idx=fake, k=4, out=ctypes.c_void_p(0x2000)):
        return L.pasa_sparse_attn_fwd_static(q, fake, fake, ctypes.byref(shape), idx, fake, k, out, None, None)

    wan14b = _shape(P, H=40, n=75_600).c()
    assert P.attn_workspace_bytes(_shape(P, H=40, n=75_600)) > P.STATIC_SCRATCH_BYTES
    assert static(wan14b) == ESCRATCH
    assert P.attn_workspace_bytes(_shape(P, H=12, n=32_760)) <= P.STATIC_SCRATCH_BYTES  # the 480p shape fits
    assert static(good, q=None) == EINVAL and static(good, k=0) == EINVAL and static(good, k=129) == EINVAL
    assert static(_shape(P, group=48).c()) == EUNSUPPORTED and static(_shape(P, d=96).c()) == EUNSUPPORTED
    assert b"static" in L.pasa_strerror(ESCRATCH)
    # the whole forward in one call
    fwd_bytes = L.pasa_forward_workspace_bytes
    assert fwd_bytes(ctypes.byref(good), 0.15) > P.attn_workspace_bytes(_shape(P)) + P.score_workspace_bytes(_shape(P))
    assert fwd_bytes(ctypes.byref(good), 0.0) == 0 and fwd_bytes(ctypes.byref(good), 1.5) == 0
    assert fwd_bytes(ctypes.byref(_shape(P, d=96).c()), 0.15) == 0

    def forward(shape, keep=0.15, q=fake, out=ctypes.c_void_p(0x2000), ws=fake, nbytes=big):
        return L.pasa_forward(q, fake, fake, ctypes.byref(shape), ctypes.c_double(keep), 7, ctypes.c_float(0.1), out, None, ws, nbytes, None)

    assert forward(good, keep=0.0) == EINVAL and forward(good, keep=float("nan")) == EINVAL
    assert forward(good, q=None) == EINVAL and forward(good, ws=None) == EINVAL
    assert forward(good, nbytes=ctypes.c_size_t(1024)) == EWORKSPACE
    assert forward(_shape(P, group=48).c()) == EUNSUPPORTED
    assert forward(_shape(P, n=5000 * 64).c()) == EUNSUPPORTED  # more key blocks than the routing kernel takes
    for code in (0, -1, -2, -3, -4, -5, -6, -99):
        assert isinstance(L.pasa_strerror(code), bytes) and len(L.pasa_strerror(code)) > 0


def test_binding_raises_a_clear_error_when_the_library_is_missing(P, monkeypatch):
    import paper_2604_12219_amd.pasa as mod
    monkeypatch.setattr(mod, "_lib", None)
    monkeypatch.setattr(mod, "_LIB_PATH", "/nonexistent/libpasa_hip.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        mod.load_library()


def test_generated_mfma_sequences_are_up_to_date():
    """pasa_mfma_pipes.hpp is written by gen_mfma_pipes.py; the committed header must be what the generator emits"""
    import importlib.util
    csrc = os.path.join(ROOT, "paper_2604_12219_amd", "csrc")
    spec = importlib.util.spec_from_file_location("gen_mfma_pipes", os.path.join(csrc, "gen_mfma_pipes.py"))
    gen = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(gen)
    with open(os.path.join(csrc, "pasa_mfma_pipes.hpp")) as f:
        assert f.read() == gen.gen()


def test_sweeps_module_imports_without_a_gpu():
    import paper_2604_12219_amd.sweeps as sweeps
    assert callable(sweeps.main) and callable(sweeps.sweep_groups) and callable(sweeps.selection_histogram)


def test_budget_schedule_host_function_matches_oracle_and_rejects_bad_input():
    """pasa_budget_schedule is host-only: checked here without a GPU (Eq.9-11)"""
    import numpy as np
    import paper_2604_12219_amd as P
    g = np.random.default_rng(5)
    for n_prompts, n_steps, rho, dense in ((10, 50, 0.15, 0.2), (1, 7, 0.5, 0.0), (3, 33, 0.9, 0.3), (2, 5, 0.2, 1.0)):
        l1 = g.uniform(0.1, 2.0, size=(n_prompts, n_steps))
        np.testing.assert_allclose(P.budget_schedule(l1, rho, dense), oracle.budget_schedule(l1, rho, dense), rtol=1e-13)
    for bad in (dict(l1=[[1.0, -1.0]], rho=0.5), dict(l1=[[0.0, 0.0]], rho=0.5, dense_fraction=0.0), dict(l1=[[1.0, 2.0]], rho=0.0),
                dict(l1=[[1.0, float("nan")]], rho=0.5, dense_fraction=0.0), dict(l1=[[1.0, 2.0]], rho=0.5, dense_fraction=1.5)):
        with pytest.raises(P.PasaError):
            P.budget_schedule(**bad)
    # the schedule drives pasa_topk_count step by step
    r = P.budget_schedule(g.uniform(0.5, 1.5, size=(10, 50)), 0.15)
    ks = [P.topk_count(1182, x) for x in r]
    assert ks[:10] == [1182] * 10 and all(1 <= k <= 1182 for k in ks) and abs(sum(ks[10:]) - 0.15 * 1182 * 40) < 40


def test_binding_checks_that_the_strides_stay_inside_the_tensors():
    """host-side bounds check of the binding: a shape whose strides reach beyond a tensor's storage is refused before
    any library call (CPU tensors will do: the check never touches the data)"""
    import torch
    import paper_2604_12219_amd.pasa as mod
    q = torch.zeros((1, 2, 100, 64), dtype=torch.bfloat16)
    shape = mod.Shape.of(q)
    mod._check_extent(shape, q=q, k=q, v=None)  # fits exactly
    longer = mod.Shape(1, 2, 101, 64, 64, 32, shape.stride_b, shape.stride_h, shape.stride_n)
    with pytest.raises(ValueError, match="reach element"):
        mod._check_extent(longer, q=q)
    view = q[:, :, 10:]  # a view that starts later in the same storage has less room
    with pytest.raises(ValueError, match="reach element"):
        mod._check_extent(shape, q=view)
    mod._check_extent(mod.Shape.of(view), q=view)
    with pytest.raises(ValueError, match="bf16"):
        mod._check_extent(shape, q=q.float())


def test_header_is_plain_c(tmp_path):
    """include/pasa.h compiles as C99 with no HIP header in sight, and a C program links against the library by name"""
    import subprocess
    src = tmp_path / "use_pasa.c"
    src.write_text('#include "pasa.h"\n#include <stdio.h>\n'
                   'int main(void) { pasa_shape_t s = {1, 2, 1000, 128, 64, 32, 256000, 128000, 128, 0.0f, 0};\n'
                   '  printf("%d %d %zu %s\\n", pasa_num_blocks(&s), pasa_topk_count(16, 0.25), pasa_attn_workspace_bytes(&s) > 0 ? (size_t)1 : (size_t)0,'
                   ' pasa_strerror(PASA_ESCRATCH));\n  return 0; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc, str(src)], check=True)
    import paper_2604_12219_amd as P
    exe = tmp_path / "use_pasa"
    libdir = os.path.dirname(P.lib_path())
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-l:libpasa_hip.so", f"-Wl,-rpath,{libdir}"],
                   check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split(maxsplit=3)
    assert out[:3] == ["16", "4", "1"] and "static" in out[3]
