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

from test_gpu_parity import DEV, dev, host

pytestmark = pytest.mark.gpu


def _rotated(case):
    rnd = orc.round_to_bf16
    aK = rnd(orc.rope3d(case.anchor_K, case.anchor_pos, case.sections, case.base))
    frames = [(rnd(orc.rope3d(K, p, case.sections, case.base)), V, p) for K, V, p in case.frames]
    queries = [rnd(orc.rope3d(Q, p, case.sections, case.base)) for Q, p in zip(case.queries, case.query_pos)]
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
    pp.copy_(dev(np.broadcast_to(p[None], (layer.Hkv, n, 3)).copy(), None))
    layer.commit(n, kind, frame)


@pytest.mark.parametrize("mode,gamma,b_min", [("pow", 0.85, 32), ("pow", 0.6, 16), ("norm", 0.7, 20),
                                              ("half", 1.0, 30), ("half", 1.0, 60), ("slide", 1.0, 0),
                                              ("dense", 1.0, 0)])
def test_rolling_layer_matches_oracle(mode, gamma, b_min):
    case = synth.rolling_case(seed=11, n_steps=6)
    aK, frames, queries = _rotated(case)
    want = orc.rolling_rollout(aK, case.anchor_V, case.anchor_pos, case.anchor_segments, frames, queries,
                               case.scale, _budget_fn(mode, case, gamma, b_min), score_rows=case.score_rows)
    n = case.n_frame
    layer = RollingLayer(case.Hq, case.Hkv, case.D, case.anchor_K.shape[1] + len(frames) * n, n, case.scale,
                         mode=mode, gamma=gamma, b_min=b_min, n_score=case.score_rows.size,
                         sections=case.sections, base=case.base, device=DEV)
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
