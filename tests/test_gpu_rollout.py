"""GPU parity of the rolling cache (several frame steps of one layer, cache kept packed in
place) against the oracle's rolling rollout, step by step, on identical input bits: the
oracle's rotated keys and queries are what the device reads, so segment tables, carried
positions and moved rows must match bit for bit and the attention outputs within the bf16
bars (max |err| <= 2e-2, mean |err| <= 2e-3)."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_2601_04359_amd as pk
from paper_2601_04359_amd import synth
from paper_2601_04359_amd.rollout import RollingLayer

from test_gpu_parity import DEV, LN2, dev, host, q_fold

pytestmark = pytest.mark.gpu


def _rotated(case, q_scale=1.0):
    rnd = orc.round_to_bf16
    aK = rnd(orc.rope3d(case.anchor_K, case.anchor_pos, case.sections, case.base))
    frames = [(rnd(orc.rope3d(K, p, case.sections, case.base)), V, p) for K, V, p in case.frames]
    queries = [rnd(orc.rope3d(Q, p, case.sections, case.base) * q_scale)
               for Q, p in zip(case.queries, case.query_pos)]
    return aK, frames, queries


def _budget_fn(mode, case, gamma, b_min):
    n = case.n_frame
    return {"pow": lambda w: orc.budget_pow(n, w, gamma, b_min),
            "norm": lambda w: orc.budget_norm(n, w, gamma, b_min),
            "half": lambda w: orc.budget_half(n, w, b_min),
            "slide": lambda w: orc.budget_slide(n, w),
            "dense": lambda w: [n] * w}[mode]


def _insert(layer, K, V, p, kind, frame):
    n = K.shape[1]
    k, v, pp = layer.reserve(n)
    k.copy_(dev(K.astype(np.float32), "bf16"))
    v.copy_(dev(V, "bf16"))
    pp.copy_(dev(np.broadcast_to(p[None], (pp.shape[0], n, 3)).copy(), None))
    layer.commit(n, kind, frame)


# fold: the queries carry scale * log2(e) and the calls get ln 2 as their scale (the kernels' shorter loops)
@pytest.mark.parametrize("mode,gamma,b_min,share,fold", [
    ("pow", 0.85, 32, False, False), ("pow", 0.6, 16, False, False), ("norm", 0.7, 20, False, False),
    ("half", 1.0, 30, False, False), ("half", 1.0, 60, False, False), ("slide", 1.0, 0, False, False),
    ("dense", 1.0, 0, False, False), ("pow", 0.85, 32, True, False), ("half", 1.0, 60, True, False),
    ("pow", 0.85, 32, False, True), ("norm", 0.7, 20, True, True), ("dense", 1.0, 0, False, True)])
def test_rolling_layer_matches_oracle(mode, gamma, b_min, share, fold):
    case = synth.rolling_case(seed=11, n_steps=6)
    aK, frames, queries = _rotated(case, q_fold(case.scale) if fold else 1.0)
    want = orc.rolling_rollout(aK, case.anchor_V, case.anchor_pos, case.anchor_segments, frames, queries,
                               LN2 if fold else case.scale, _budget_fn(mode, case, gamma, b_min),
                               score_rows=case.score_rows, share_heads=share)
    n = case.n_frame
    layer = RollingLayer(case.Hq, case.Hkv, case.D, case.anchor_K.shape[1] + len(frames) * n, n, case.scale,
                         mode=mode, gamma=gamma, b_min=b_min, n_score=case.score_rows.size,
                         sections=case.sections, base=case.base, device=DEV, share_heads=share, fold_scale=fold)
    assert np.array_equal(host(layer.q_rows), case.score_rows)
    for (start, length, kind, frame) in case.anchor_segments:
        _insert(layer, aK[:, start:start + length], case.anchor_V[:, start:start + length],
                case.anchor_pos[start:start + length], kind, frame)
    for i, Q in enumerate(queries):
        if i >= 1:
            Kf, Vf, pf = frames[i - 1]
            _insert(layer, Kf, Vf, pf, pk.PC_SEG_FRAME, i)
        O = layer.step(dev(Q.astype(np.float32), "bf16"))
        w = want[i]
        assert layer.segments == w["segments"], (mode, i)
        nk = layer.nk
        assert nk == w["K"].shape[1]
        assert np.array_equal(host(layer.pos[:, :nk]), w["pos"]), f"step {i + 1}: kept set differs"
        assert np.array_equal(host(layer.K[:, :nk]).astype(np.float64), w["K"])
        assert np.array_equal(host(layer.V[:, :nk]).astype(np.float64), w["V"])
        err = np.abs(host(O).astype(np.float64) - w["O"])
        assert err.max() <= 2e-2 and err.mean() <= 2e-3, (mode, i, err.max(), err.mean())
    if mode == "slide":   # only the newest frame survives, older segments are empty
        assert [s[1] for s in layer.segments if s[2] == pk.PC_SEG_FRAME] == [0] * (len(frames) - 2) + [n]


@pytest.mark.parametrize("mode,gamma,b_min,share,fold", [("pow", 0.85, 32, False, False), ("half", 1.0, 40, True, True)])
def test_rolling_layer_with_the_steps_own_frame_in_the_cache(mode, gamma, b_min, share, fold):
    """The frame being generated is in the cache as an always-kept SELF segment (Eq. 2: attention
    inside a frame is bidirectional) and becomes the newest past frame at the next step by a
    table edit; against the oracle's rollout with include_self."""
    case = synth.rolling_case(seed=17, n_steps=5)
    aK, frames, queries = _rotated(case, q_fold(case.scale) if fold else 1.0)
    want = orc.rolling_rollout(aK, case.anchor_V, case.anchor_pos, case.anchor_segments, frames, queries,
                               LN2 if fold else case.scale, _budget_fn(mode, case, gamma, b_min),
                               score_rows=case.score_rows, share_heads=share, include_self=True)
    n = case.n_frame
    layer = RollingLayer(case.Hq, case.Hkv, case.D, case.anchor_K.shape[1] + (len(frames) + 1) * n, n, case.scale,
                         mode=mode, gamma=gamma, b_min=b_min, n_score=case.score_rows.size,
                         sections=case.sections, base=case.base, device=DEV, share_heads=share, fold_scale=fold)
    for (start, length, kind, frame) in case.anchor_segments:
        _insert(layer, aK[:, start:start + length], case.anchor_V[:, start:start + length],
                case.anchor_pos[start:start + length], kind, frame)
    for i, Q in enumerate(queries):
        layer.promote_self()
        Kf, Vf, pf = frames[i]
        _insert(layer, Kf, Vf, pf, pk.PC_SEG_SELF, i + 1)
        O = layer.step(dev(Q.astype(np.float32), "bf16"))
        w = want[i]
        assert layer.segments == w["segments"], (mode, i)
        nk = layer.nk
        assert nk == w["K"].shape[1] and layer.segments[-1] == (nk - n, n, pk.PC_SEG_SELF, i + 1)
        assert np.array_equal(host(layer.pos[:, :nk]), w["pos"]), f"step {i + 1}: kept set differs"
        assert np.array_equal(host(layer.K[:, :nk]).astype(np.float64), w["K"])
        assert np.array_equal(host(layer.V[:, :nk]).astype(np.float64), w["V"])
        err = np.abs(host(O).astype(np.float64) - w["O"])
        assert err.max() <= 2e-2 and err.mean() <= 2e-3, (mode, i, err.max(), err.mean())


def test_rotation_on_insert_equals_standalone_rotation():
    case = synth.rolling_case(seed=3, n_steps=2)
    n = case.n_frame
    layer = RollingLayer(case.Hq, case.Hkv, case.D, 2 * n, n, case.scale, n_score=64, device=DEV)
    K, V, p = case.frames[0]
    k, v, pp = layer.reserve(n)
    k.copy_(dev(K, "bf16"))
    v.copy_(dev(V, "bf16"))
    pd = dev(p, None)
    pp.copy_(pd[None].expand(layer.Hkv, n, 3))
    layer.commit(n, pk.PC_SEG_FRAME, 1, rotate_with=pd)
    ref = dev(K, "bf16")
    pk.pc_rope3d(ref, pd, case.sections, case.base)
    assert torch.equal(layer.K[:, :n], ref) and layer.nk == n and layer.segments == [(0, n, pk.PC_SEG_FRAME, 1)]


def test_attend_then_refresh_with_its_lse_keeps_the_same_rows():
    # iterative decoding: first pass on the un-packed cache, its LSE feeds the scoring
    case = synth.rolling_case(seed=11, n_steps=3)
    aK, frames, queries = _rotated(case)
    n = case.n_frame
    mk = lambda: RollingLayer(case.Hq, case.Hkv, case.D, case.anchor_K.shape[1] + 3 * n, n, case.scale, mode="pow",
                              gamma=0.85, b_min=32, n_score=case.score_rows.size, sections=case.sections,
                              device=DEV)
    a, b = mk(), mk()
    for lay in (a, b):
        for (start, length, kind, frame) in case.anchor_segments:
            _insert(lay, aK[:, start:start + length], case.anchor_V[:, start:start + length],
                    case.anchor_pos[start:start + length], kind, frame)
    lse = torch.empty((case.Hq, n), dtype=torch.float32, device=DEV)
    for i, Q in enumerate(queries):
        if i >= 1:
            for lay in (a, b):
                _insert(lay, *frames[i - 1], pk.PC_SEG_FRAME, i)
        Qd = dev(Q.astype(np.float32), "bf16")
        Oa = a.step(Qd)
        b.attend(Qd, lse=lse)
        b.refresh(Qd, lse=lse)
        Ob = b.attend(Qd)
        assert a.segments == b.segments
        # the two scorings differ by the LSE's fp32 rounding: same kept rows on this seed
        assert torch.equal(a.pos[:, :a.nk], b.pos[:, :b.nk]) and torch.equal(a.K[:, :a.nk], b.K[:, :b.nk])
        assert torch.equal(Oa, Ob)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rebase_parity(dtype):
    rng = np.random.default_rng(5)
    hkv, cap, d, sections, base = 3, 700, 128, (32, 48, 48), 10000.0
    K = rng.standard_normal((hkv, cap, d)).astype(np.float32)
    if dtype == "bf16":
        K = synth.to_bf16(K)
    pos = rng.integers(0, 400, size=(hkv, cap, 3)).astype(np.int32)
    Kd, pd = dev(K, dtype), dev(pos, None)
    row0, n_rows, delta = 37, 601, 12
    pk.pc_rebase(Kd, pd, row0, n_rows, delta, sections, base)
    want_K, want_pos = orc.rebase(K[:, row0:row0 + n_rows], pos[:, row0:row0 + n_rows], delta, sections, base)
    got = host(Kd).astype(np.float64)
    tol = 2.0 ** -8 * np.abs(want_K) + 1e-6 if dtype == "bf16" else 1e-6
    assert np.all(np.abs(got[:, row0:row0 + n_rows] - want_K) <= tol)
    # rows outside the range, and the h / w sections inside it, keep their bits
    assert np.array_equal(got[:, :row0], K[:, :row0]) and np.array_equal(got[:, row0 + n_rows:], K[:, row0 + n_rows:])
    assert np.array_equal(got[:, :, 32:], K[:, :, 32:].astype(np.float64))
    hp = host(pd)
    assert np.array_equal(hp[:, row0:row0 + n_rows], want_pos)
    assert np.array_equal(hp[:, :row0], pos[:, :row0]) and np.array_equal(hp[:, row0 + n_rows:], pos[:, row0 + n_rows:])


@pytest.mark.parametrize("mode,b_min", [("half", 60), ("slide", 0), ("norm", 80)])
def test_sliding_window_with_rebase_matches_oracle_fp32(mode, b_min):
    # fp32 tier: the device's fp32 rotations and the oracle's fp64 ones differ by ~1e-7, far
    # inside the selection band, so kept sets and coordinates must agree exactly step after
    # step while rows are compared to 1e-5.
    case = synth.rolling_case(seed=21, n_steps=7, hq=4, hkv=2, d=128, dtype="f32")
    n, t_scale, gamma = case.n_frame, 4, 0.7
    rot = (case.sections, case.base)
    f32 = lambda a: np.asarray(a, dtype=np.float32).astype(np.float64)
    want = orc.rolling_rollout(case.anchor_K, case.anchor_V, case.anchor_pos, case.anchor_segments, case.frames,
                               case.queries, case.scale, _budget_fn(mode, case, gamma, b_min),
                               score_rows=case.score_rows, rotate=rot, query_pos=case.query_pos,
                               rebase_t_scale=t_scale, storage=f32)
    assert want[-1]["shift"] > 0, "the case must slide"
    layer = RollingLayer(case.Hq, case.Hkv, case.D, case.anchor_K.shape[1] + 3 * n, n, case.scale, mode=mode,
                         gamma=gamma, b_min=b_min, n_score=case.score_rows.size, sections=case.sections,
                         base=case.base, dtype=torch.float32, device=DEV, slide_t_scale=t_scale)
    k, v, p = layer.reserve(case.anchor_K.shape[1])
    k.copy_(dev(case.anchor_K, "f32")); v.copy_(dev(case.anchor_V, "f32"))
    apos = dev(case.anchor_pos, None)
    p.copy_(apos[None].expand_as(p))
    for (start, length, kind, frame) in case.anchor_segments:
        layer.commit(length, kind, frame, rotate_with=apos[start:start + length])
    for i, Q in enumerate(case.queries):
        shift = layer.advance_window()
        assert shift == want[i]["shift"]
        if i >= 1:
            Kf, Vf, pf = case.frames[i - 1]
            pf = pf.copy(); pf[:, 0] -= shift
            k, v, p = layer.reserve(n)
            k.copy_(dev(Kf, "f32")); v.copy_(dev(Vf, "f32"))
            pfd = dev(pf, None)
            p.copy_(pfd[None].expand_as(p))
            layer.commit(n, pk.PC_SEG_FRAME, i, rotate_with=pfd)
        qp = case.query_pos[i].copy(); qp[:, 0] -= shift
        O = layer.step(dev(Q, "f32"), q_pos=dev(qp, None))
        w = want[i]
        assert layer.segments == w["segments"], (mode, i, layer.segments, w["segments"])
        nk = layer.nk
        assert np.array_equal(host(layer.pos[:, :nk]), w["pos"]), f"step {i + 1}: kept set or coordinates differ"
        assert np.abs(host(layer.K[:, :nk]) - w["K"]).max() <= 1e-5
        assert np.array_equal(host(layer.V[:, :nk]).astype(np.float64), w["V"])
        assert np.abs(host(O) - w["O"]).max() <= 2e-5
