"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its
host-side logic (budgets, compaction plan, argument validation) agrees with the oracle.
No device work is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle as orc
import paper_2601_04359_amd as pk
from paper_2601_04359_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.lib_path()):
        from paper_2601_04359_amd.build import build_library
        build_library()
    return binding.lib()


def test_every_declared_symbol_is_exported(L):
    with open(os.path.join(ROOT, "include", "packcache.h")) as f:
        header = f.read()
    names = set(re.findall(r"\b(pc_[a-z0-9_]+)\s*\(", header))
    assert {"pc_budget", "pc_rope3d", "pc_rebase", "pc_score", "pc_compact", "pc_frame_attn", "pc_compact_plan",
            "pc_strerror", "pc_last_error_detail", "pc_version", "pc_score_workspace_bytes",
            "pc_compact_workspace_bytes", "pc_frame_attn_workspace_bytes"} <= names
    for n in names:
        assert hasattr(L, n), n
    assert pk.pc_version() >= 100
    assert pk.pc_strerror(0) == "ok" and "NULL" in pk.pc_strerror(-1)


@pytest.mark.parametrize("gamma", [0.5, 0.7, 0.85, 0.95, 1.0, 0.3333333333333333, 1e-3])
@pytest.mark.parametrize("N,n_past,b_min", [(64, 4, 8), (4032, 47, 512), (4032, 23, 0), (4096, 60, 1), (7, 3, 0)])
def test_budget_pow_matches_oracle(L, gamma, N, n_past, b_min):
    assert pk.pc_budget(pk.PC_BUDGET_POW, N, n_past, gamma, b_min) == orc.budget_pow(N, n_past, gamma, b_min)


def test_budget_pow_config_values(L):
    assert pk.pc_budget(pk.PC_BUDGET_POW, 64, 4, 0.7, 8) == [44, 31, 21, 15]
    assert sum(pk.pc_budget(pk.PC_BUDGET_POW, 4032, 47, 0.85, 512)) == 37512
    assert pk.pc_budget(pk.PC_BUDGET_POW, 4096, 12, 0.5, 0) == [4096 >> d for d in range(1, 13)]
    assert pk.pc_budget(pk.PC_BUDGET_POW, 100, 0, 0.5, 0) == []


@pytest.mark.parametrize("rho", [0.5, 0.7, 0.85, 0.95, 1.0])
@pytest.mark.parametrize("w", [1, 2, 3, 12, 47])
@pytest.mark.parametrize("q_min", [0, 100, 512, 3000])
def test_budget_norm_and_half_match_oracle(L, rho, w, q_min):
    assert pk.pc_budget(pk.PC_BUDGET_NORM, 4084, w, rho, q_min) == orc.budget_norm(4084, w, rho, q_min)
    assert pk.pc_budget(pk.PC_BUDGET_HALF, 4084, w, 0.0, q_min) == orc.budget_half(4084, w, q_min)
    assert pk.pc_budget(pk.PC_BUDGET_SLIDE, 4084, w) == orc.budget_slide(4084, w)


def test_budgets_match_oracle_on_random_parameters(L):
    """Exact integer budgets for random decay factors (arbitrary doubles, not only short decimals),
    frame sizes, window lengths and quotas: the library's big-integer arithmetic against the
    oracle's rationals; and the invariants of Eq. 8 (fixed-budget rules add up to B_one)."""
    rng = np.random.default_rng(2024)
    for _ in range(400):
        N, w = int(rng.integers(1, 9000)), int(rng.integers(0, 100))
        gamma = float(rng.choice([rng.uniform(1e-3, 1.0), 1.0, 0.5, rng.uniform(0.9, 1.0)]))
        q = int(rng.choice([0, rng.integers(0, 50), rng.integers(0, N + 1)]))
        assert pk.pc_budget(pk.PC_BUDGET_POW, N, w, gamma, q) == orc.budget_pow(N, w, gamma, q), (N, w, gamma, q)
        norm = pk.pc_budget(pk.PC_BUDGET_NORM, N, w, gamma, q)
        half = pk.pc_budget(pk.PC_BUDGET_HALF, N, w, 0.0, q)
        assert norm == orc.budget_norm(N, w, gamma, q), (N, w, gamma, q)
        assert half == orc.budget_half(N, w, q), (N, w, q)
        if w > 0:
            assert sum(norm) == N and sum(half) == N
            assert all(a >= b for a, b in zip(norm, norm[1:])) and all(a >= b for a, b in zip(half, half[1:]))


def test_budget_half_series_from_the_paper(L):
    assert pk.pc_budget(pk.PC_BUDGET_HALF, 4096, 4) == [2048, 1024, 512, 512]
    assert pk.pc_budget(pk.PC_BUDGET_HALF, 4096, 1) == [4096]


def test_budget_errors(L):
    for args in [(9, 10, 2, 0.5, 0), (0, -1, 2, 0.5, 0), (0, 10, -2, 0.5, 0), (0, 10, 2, 0.0, 0),
                 (0, 10, 2, 1.5, 0), (1, 10, 2, -0.1, 0), (0, 10, 2, 0.5, -1)]:
        with pytest.raises(pk.PackCacheError) as e:
            pk.pc_budget(*args)
        assert e.value.status == -5
    assert L.pc_budget(0, 10, 2, 0.5, 0, None) == -1
    assert b"budget_out" in L.pc_last_error_detail()


def test_compact_plan_matches_oracle(L):
    w = synth.config1()
    b = pk.pc_budget(pk.PC_BUDGET_POW, w.n_frame, w.n_past, w.gamma, w.b_min)
    budgets = pk.segment_budgets(w.segments, b)
    assert budgets == [16, 64, 15, 21, 31, 44]
    segs, nk = pk.pc_compact_plan(w.segments, budgets)
    assert segs == orc.packed_segments(w.segments, budgets) and nk == 191
    # budget above the segment length is clamped, zero budget empties the segment
    segs, nk = pk.pc_compact_plan(w.segments, [0, 0, 1000, 0, 5, 64])
    assert [s[1] for s in segs] == [16, 64, 64, 0, 5, 64] and nk == 213


def test_compact_plan_errors(L):
    with pytest.raises(pk.PackCacheError) as e:
        pk.pc_compact_plan([(0, 4, 0, 0), (5, 4, 2, 1)], [4, 4])        # gap in the table
    assert e.value.status == -2
    with pytest.raises(pk.PackCacheError) as e:
        pk.pc_compact_plan([(0, 4, 2, 0)], [-1])
    assert e.value.status == -5
    with pytest.raises(pk.PackCacheError) as e:
        pk.pc_compact_plan([(0, 4, 7, 0)], [1])                          # unknown kind
    assert e.value.status == -2


def test_argument_validation_returns_before_any_device_work(L):
    one = C.c_void_p(16)   # non-NULL dummy; every call below must fail before touching it
    # dtype
    assert L.pc_frame_attn(one, one, one, 5, 2, 1, 4, 4, 128, 512, 512, 512, 0.1, one, None, None, 0, None) == -3
    # Hq not a multiple of Hkv
    assert L.pc_frame_attn(one, one, one, 1, 3, 2, 4, 4, 128, 512, 512, 512, 0.1, one, None, None, 0, None) == -2
    # empty key set
    assert L.pc_frame_attn(one, one, one, 1, 2, 1, 4, 0, 128, 512, 512, 512, 0.1, one, None, None, 0, None) == -2
    # NULL tensor
    assert L.pc_frame_attn(None, one, one, 1, 2, 1, 4, 4, 128, 512, 512, 512, 0.1, one, None, None, 0, None) == -1
    # bf16 tier is D = 128 only
    assert L.pc_frame_attn(one, one, one, 1, 2, 1, 4, 4, 64, 256, 256, 256, 0.1, one, None, None, 0, None) == -4
    # stride too small
    assert L.pc_frame_attn(one, one, one, 1, 2, 1, 4, 4, 128, 8, 512, 512, 0.1, one, None, None, 0, None) == -2
    # rope: sections must add up to D
    assert L.pc_rope3d(one, 1, 1, 4, 128, 512, one, 32, 48, 40, 1e4, 1.0, None) == -2
    assert L.pc_rope3d(one, 1, 1, 4, 128, 512, one, 32, 48, 48, 1e4, 0.0, None) == -2      # out_scale must be > 0
    assert L.pc_rope3d(None, 1, 1, 4, 128, 512, one, 32, 48, 48, 1e4, 1.0, None) == -1
    # rebase: sections must add up to D; a temporal section that is not whole 16-byte chunks; NULL
    assert L.pc_rebase(one, 1, 1, 128, 512, one, 1, 12, 0, 4, 4, 32, 48, 40, 1e4, None) == -2
    assert L.pc_rebase(one, 1, 1, 128, 512, one, 1, 12, 0, 4, 4, 20, 60, 48, 1e4, None) == -4
    assert L.pc_rebase(None, 1, 1, 128, 512, one, 1, 12, 0, 4, 4, 32, 48, 48, 1e4, None) == -1
    assert L.pc_rebase(one, 1, 1, 128, 512, one, 2, 12, 0, 4, 4, 32, 48, 48, 1e4, None) == -2   # Hsel > Hkv
    assert L.pc_rebase(None, 1, 1, 128, 512, None, 1, 12, 0, 0, 4, 32, 48, 48, 1e4, None) == 0   # nothing to do
    # score: workspace missing / too small
    need = L.pc_score_workspace_bytes(4, 2, 8, 100, 0)
    assert need > 0
    assert L.pc_score(one, one, 1, 4, 2, 8, 100, 128, 1024, 12800, None, 0.1, None, 0, one, 100, 0, 0, 0, None, 0, None) == -6
    assert L.pc_score(one, one, 1, 4, 2, 8, 100, 128, 1024, 12800, None, 0.1, None, 0, one, 100, 0, 0, 0, one, need - 1, None) == -6
    # key range: empty, reversed or past the end
    for kb, ke in ((5, 5), (7, 3), (0, 101), (-1, 10), (100, 0)):
        assert L.pc_score(one, one, 1, 4, 2, 8, 100, 128, 1024, 12800, None, 0.1, None, 0, one, 100, 0, kb, ke, one, need, None) == -2
    # compact: too many segments; partial aliasing of outputs
    seg = (binding.pc_segment * 2)(binding.pc_segment(0, 4, 0, 0), binding.pc_segment(4, 8, 2, 1))
    bud = (C.c_int32 * 2)(4, 3)
    assert L.pc_compact(one, one, one, 1, 1, 128, 4096, 0, one, 0, seg, 500, bud, 0, one, one, one, 4096, 0,
                        None, 0, None, None, one, 1 << 20, None) == -2
    two = C.c_void_p(4096)
    assert L.pc_compact(one, one, one, 1, 1, 128, 4096, 36, one, 12, seg, 2, bud, 0, one, two, one, 4096, 36,
                        None, 0, None, None, one, 1 << 20, None) == -2
    assert b"alias" in L.pc_last_error_detail()


def test_binding_raises_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "lib_path", lambda: str(tmp_path / "libpackcache.so"))
    with pytest.raises(FileNotFoundError):
        binding.pc_version()


def test_masked_budgets_match_the_oracle():
    w = synth.midsize()
    rng = np.random.default_rng(0)
    valid = (rng.random(w.Nk) < 0.3).astype(np.uint8)
    for gamma, b_min in ((0.85, 32), (0.5, 0), (1.0, 0)):
        budgets = pk.segment_budgets(w.segments, orc.budget_pow(w.n_frame, w.n_past, gamma, b_min))
        assert pk.pc_masked_budgets(w.segments, budgets, valid) == orc.masked_budgets(w.segments, budgets, valid)
    with pytest.raises(pk.PackCacheError):
        pk.pc_masked_budgets(w.segments, [-1] * len(w.segments), valid)


def test_batched_compaction_and_mask_argument_checks(L):
    one, two = C.c_void_p(4096), C.c_void_p(8192)
    seg = (binding.pc_segment * 2)(binding.pc_segment(0, 4, 0, 0), binding.pc_segment(4, 8, 2, 1))
    bud = (C.c_int32 * 2)(4, 3)
    ws = L.pc_compact_batch_workspace_bytes(3, 2, 12, 0)
    assert ws >= L.pc_compact_workspace_bytes(2, 12, 0) > 0
    assert L.pc_compact_batch_workspace_bytes(0, 2, 12, 0) == 0

    def call(n_layers, kv_l, pos_l, sc_l, in_place=True, hkv=2):
        Ko = one if in_place else two
        return L.pc_compact_batch(n_layers, one, one, one, 1, hkv, 128, 12 * 128, kv_l, 36, pos_l, one, 12, sc_l,
                                  seg, 2, bud, 0, Ko, Ko, Ko, 12 * 128, kv_l, 36, pos_l, None, 0, 0, None, None,
                                  one, 1 << 24, None)
    # a layer stride smaller than one layer of K / pos / score
    assert call(3, 2 * 12 * 128 - 8, 72, 24) == -2
    assert call(3, 2 * 12 * 128, 71, 24) == -2
    assert call(3, 2 * 12 * 128, 72, 23) == -2
    # zero layers; too many (layer, head) pairs for the in-place tickets
    assert call(0, 0, 0, 0) == -2
    assert call(129, 2 * 12 * 128, 72, 24) == -4
    assert b"pairs" in L.pc_last_error_detail()
    # mask: NULL pointers, short stride; empty input is fine
    assert L.pc_mask_scores(None, 2, 10, 10, one, None) == -1
    assert L.pc_mask_scores(one, 2, 10, 9, one, None) == -2
    assert L.pc_mask_scores(None, 0, 10, 10, None, None) == 0
    assert L.pc_masked_budgets(seg, 2, bud, None, bud) == -1
    # status of a workspace that does not exist
    assert L.pc_compact_status(None, None) == -1
    assert L.pc_strerror(-8) not in (None, L.pc_strerror(-7))


def test_static_scratch_entry_rejects_oversized_requests_before_any_device_work(L):
    # pc_compact_static: the request is sized on the host and refused before the device is touched
    assert L.pc_compact_static_capacity() == 4 << 20
    assert L.pc_compact_workspace_bytes(4, 193_792, 0) <= L.pc_compact_static_capacity()
    one = C.c_void_p(4096)
    n = 400_000
    assert L.pc_compact_workspace_bytes(8, n, 0) > L.pc_compact_static_capacity()
    seg = (binding.pc_segment * 1)(binding.pc_segment(0, n, 1, 0))
    bud = (C.c_int32 * 1)(n)
    rc = L.pc_compact_static(one, one, one, 1, 8, 128, n * 128, n * 3, one, n, seg, 1, bud, 0, one, one, one,
                             n * 128, n * 3, None, 0, None, None, None)
    assert rc == -6 and b"scratch" in L.pc_last_error_detail()
    # malformed table: refused as a shape error, also before any device work
    assert L.pc_compact_static(one, one, one, 1, 0, 128, 0, 0, one, 0, seg, 1, bud, 0, one, one, one, 0, 0, None,
                               0, None, None, None) == -2


def test_fold_helpers_are_the_constants_the_header_names():
    import math
    assert pk.PC_SCALE_FOLDED == math.log(2.0)
    # what the kernels test for: float(ln 2) * float(log2 e), rounded to fp32, is exactly 1
    assert C.c_float(C.c_float(pk.PC_SCALE_FOLDED).value * C.c_float(1.4426950408889634).value).value == 1.0
    for s in (128 ** -0.5, 64 ** -0.5, 0.3):
        assert abs(pk.folded_q_scale(s) - s / math.log(2.0)) <= 1e-15 * s
    src = open(os.path.join(ROOT, "include", "packcache.h")).read()
    assert "#define PC_SCALE_FOLDED 0.693147180559945309f" in src


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout.strip() == ""
