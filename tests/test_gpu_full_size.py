"""GPU parity at the full sizes and in the launch configuration that bench.py times:
16 query heads, 4 KV heads, D = 128, 48x84 tokens per frame, 256 text tokens, at frames
2, 12, 24 and 48 (up to 193,792 dense keys), gamma = 0.85 with a 512-token minimum quota.

Each step is compared with the fp64 oracle on identical input bits:
  * pc_rope3d on the whole new frame (all elements);
  * pc_score over all keys with the 512 strided scoring rows (all elements);
  * the selected index sets (bit-exact outside the 1e-6 score band), the gathered rows
    and carried positions (bit-exact), out of place as in the frame-24 step and in place
    as in the frame-48 compaction runs, for gamma in {0.7, 0.85, 0.95};
  * pc_frame_attn, packed and dense, on 64 sampled query rows per head over all keys
    (max |err| <= 2e-2, mean |err| <= 2e-3), and its log-sum-exp output.
The stack call (pc_compact_batch, 8 layers at frame 48, in place) is compared with the per-layer
call bit for bit and with the oracle's top-k.
The rolling step (cache packed in place over several frame steps) is checked at the 28-layer
rollout's shape, 24 query / 8 KV heads, each step starting from the oracle's previous state.
The steps after the rotation read the ORACLE's rotated bits, so that every step is judged on
inputs identical to the oracle's; the chained device path is covered at reduced size in
test_gpu_parity.py.
"""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_2601_04359_amd as pk
from paper_2601_04359_amd import synth

from test_gpu_parity import BAND, DEV, LN2, check_selection, dev, host, q_fold

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

N_SAMPLE_ROWS = 64


def _budgets(w, gamma):
    b = pk.pc_budget(pk.PC_BUDGET_POW, w.n_frame, w.n_past, gamma, w.b_min)
    assert b == orc.budget_pow(w.n_frame, w.n_past, gamma, w.b_min)
    return pk.segment_budgets(w.segments, b)


# fold = True is the form bench.py times: the query rotation multiplies scale * log2(e) into Q
# and the scoring and attention calls get scale = ln 2
@pytest.mark.parametrize("fold", [False, True])
@pytest.mark.parametrize("frame", [2, 12, 24, 48])
def test_full_size_frame(frame, fold):
    w = synth.config2(seed=1000, n_past=frame - 1)
    q_scale = q_fold(w.scale) if fold else 1.0
    scale = LN2 if fold else w.scale
    Hq, Hkv, Nk, Nq = w.Hq, w.Hkv, w.Nk, w.Nq
    newest = w.segments[-1]
    a, n_new = newest[0], newest[1]
    print(f"frame {frame}: Nk={Nk}", flush=True)

    # ---- a1: rotation of the new frame's queries and of the newest cached frame's keys
    Qd, Kd = dev(w.Q, "bf16"), dev(w.K, "bf16")
    pk.pc_rope3d(Qd, dev(w.pos_q, None), w.sections, w.base, out_scale=q_scale)
    kn = Kd[:, a:a + n_new]
    pk.pc_rope3d(kn, dev(w.pos_k[a:a + n_new], None), w.sections, w.base)
    q_rot = orc.rope3d(w.Q, w.pos_q, w.sections, w.base) * q_scale
    k_rot = orc.rope3d(w.K[:, a:a + n_new], w.pos_k[a:a + n_new], w.sections, w.base)
    for got, want, floor in ((host(Qd), q_rot, 1e-6 * min(q_scale, 1.0)), (host(kn), k_rot, 1e-6)):
        assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + floor)
    assert torch.equal(Kd[:, :a], dev(w.K[:, :a], "bf16")), "rows outside the new frame must not change"
    del Qd, Kd, kn

    # the oracle's rotated bits feed every later step on both sides
    Qo = orc.round_to_bf16(q_rot)
    Ko = w.K.astype(np.float64)
    Ko[:, a:a + n_new] = orc.round_to_bf16(k_rot)
    Vo = w.V.astype(np.float64)
    Q, K, V = dev(Qo.astype(np.float32), "bf16"), dev(Ko.astype(np.float32), "bf16"), dev(w.V, "bf16")
    assert np.array_equal(host(Q), Qo) and np.array_equal(host(K[:, a:]), Ko[:, a:])
    pos_host = np.broadcast_to(w.pos_k[None], (Hkv, Nk, 3)).copy()
    pos = dev(pos_host, None)

    # ---- a2: importance of every key
    rows = dev(w.score_rows.astype(np.int32), None)
    sc = pk.pc_score(Q, K, Nk, scale, q_rows=rows)
    sco = orc.score(Qo[:, w.score_rows], Ko, scale)
    got = host(sc).astype(np.float64)
    err = np.abs(got - sco)
    assert np.all(err <= 2e-7 + 2e-5 * sco), (err.max(), (err / (sco + 1e-30)).max())
    np.testing.assert_allclose(got.sum(1), w.score_rows.size * (Hq // Hkv), rtol=1e-5)
    print("score ok", flush=True)

    # ---- a3..a5: budgets, selection, gather; out of place and in place
    kept = {}
    for gamma in (0.85, 0.7, 0.95):
        budgets = _budgets(w, gamma)
        segs_want = orc.packed_segments(w.segments, budgets)
        nk_want = segs_want[-1][0] + segs_want[-1][1]
        Kp, Vp = torch.empty((Hkv, nk_want, w.D), dtype=K.dtype, device=DEV), torch.empty(
            (Hkv, nk_want, w.D), dtype=K.dtype, device=DEV)
        pp = torch.empty((Hkv, nk_want, 3), dtype=torch.int32, device=DEV)
        idx = torch.empty((Hkv, nk_want), dtype=torch.int32, device=DEV)
        segs, nk = pk.pc_compact(K, V, pos, sc, w.segments, budgets, out=(Kp, Vp, pp), idx=idx)
        assert nk == nk_want and segs == segs_want
        ig = host(idx)
        check_selection(ig, sco, w.segments, budgets, band=BAND)
        for h in range(Hkv):
            sel = idx[h].long()
            assert torch.equal(Kp[h], K[h].index_select(0, sel))
            assert torch.equal(Vp[h], V[h].index_select(0, sel))
            assert np.array_equal(host(pp[h]), w.pos_k[ig[h]])
        # in place on a copy of the cache: the same rows must end up in the packed prefix
        K2, V2, p2 = K.clone(), V.clone(), pos.clone()
        idx2 = torch.empty_like(idx)
        segs2, nk2 = pk.pc_compact(K2, V2, p2, sc, w.segments, budgets, idx=idx2)
        assert nk2 == nk and segs2 == segs and torch.equal(idx2, idx)
        assert torch.equal(K2[:, :nk], Kp) and torch.equal(V2[:, :nk], Vp) and torch.equal(p2[:, :nk], pp)
        del K2, V2, p2
        if gamma == w.gamma:
            kept = {"K": Kp, "V": Vp, "idx": ig, "nk": nk}
        print(f"compact gamma={gamma} ok, Nk_packed={nk}", flush=True)

    # ---- a6: attention over the kept keys, and over the dense cache, on sampled query rows
    rs = synth.strided_rows(Nq, N_SAMPLE_ROWS)
    ig, nk = kept["idx"], kept["nk"]
    lse = torch.empty((Hq, Nq), dtype=torch.float32, device=DEV)
    O = pk.pc_frame_attn(Q, kept["K"], kept["V"], nk, scale, lse=lse)
    Kk = np.stack([Ko[g][ig[g]] for g in range(Hkv)])
    Vk = np.stack([Vo[g][ig[g]] for g in range(Hkv)])
    Ow, Lw = orc.frame_attn(Qo[:, rs], Kk, Vk, scale)
    err = np.abs(host(O)[:, rs].astype(np.float64) - Ow)
    assert err.max() <= 2e-2 and err.mean() <= 2e-3, (err.max(), err.mean())
    assert np.abs(host(lse)[:, rs] - Lw).max() <= 1e-3
    O = pk.pc_frame_attn(Q, K, V, Nk, scale, lse=lse)
    Ow, Lw = orc.frame_attn(Qo[:, rs], Ko, Vo, scale)
    err = np.abs(host(O)[:, rs].astype(np.float64) - Ow)
    assert err.max() <= 2e-2 and err.mean() <= 2e-3, (err.max(), err.mean())
    assert np.abs(host(lse)[:, rs] - Lw).max() <= 1e-3


@pytest.mark.parametrize("gamma", [0.7, 0.95])
def test_full_size_stack_compaction_equals_layer_by_layer_and_the_oracle(gamma):
    """pc_compact_batch at frame 48 as bench.py's batched leg runs it (4 KV heads, 193,792 rows,
    in place), on 8 layers drawn on the device from their own seeds: 1,568 selections in one
    call, which takes the one-wave-per-segment select.  Every layer must come out bit for bit as
    one pc_compact call per layer leaves it (the form the test above checks against the oracle),
    and the index sets of the first and last layer are compared with the oracle's top-k on the
    same fp32 scores (exact: no band)."""
    L, Hq, Hkv, D, n_past, n_text, gh, gw = 8, 16, 4, 128, 47, 256, 48, 84
    n = gh * gw
    Nk = n_text + n * (1 + n_past)
    segments = synth.segment_table(n_text, n, n_past)
    rows = dev(synth.strided_rows(n, 512).astype(np.int32), None)
    pos_k = synth.cache_positions(n_text, gh, gw, n_past)
    KL = torch.empty((L, Hkv, Nk, D), dtype=torch.bfloat16, device=DEV)
    VL = torch.empty_like(KL)
    PL = dev(np.broadcast_to(pos_k[None, None], (L, Hkv, Nk, 3)).copy(), None)
    SL = torch.empty((L, Hkv, Nk), dtype=torch.float32, device=DEV)
    Q = torch.empty((Hq, n, D), dtype=torch.bfloat16, device=DEV)
    for l in range(L):
        synth.device_frame_layer(4000 + l, n_past, KL[l], VL[l], Q)
        pk.pc_score(Q, KL[l], Nk, D ** -0.5, score=SL[l], q_rows=rows)
    b = pk.pc_budget(pk.PC_BUDGET_POW, n, n_past, gamma, 512)
    assert b == orc.budget_pow(n, n_past, gamma, 512)
    budgets = pk.segment_budgets(segments, b)
    plan, nk_out = pk.pc_compact_plan(segments, budgets)
    ref = []
    for l in range(L):                                   # one call per layer, out of place
        Ko = torch.empty((Hkv, nk_out, D), dtype=KL.dtype, device=DEV)
        Vo, po = torch.empty_like(Ko), torch.empty((Hkv, nk_out, 3), dtype=torch.int32, device=DEV)
        io = torch.empty((Hkv, nk_out), dtype=torch.int32, device=DEV)
        pk.pc_compact(KL[l], VL[l], PL[l], SL[l], segments, budgets, out=(Ko, Vo, po), idx=io)
        ref.append((Ko, Vo, po, io))
    idx = torch.full((L, Hkv, nk_out), -1, dtype=torch.int32, device=DEV)
    segs, nk = pk.pc_compact_batch(KL, VL, PL, SL, segments, budgets, idx=idx)       # in place
    assert segs == plan and nk == nk_out
    for l in range(L):
        Ko, Vo, po, io = ref[l]
        assert torch.equal(idx[l], io), l
        assert torch.equal(KL[l, :, :nk], Ko) and torch.equal(VL[l, :, :nk], Vo) and torch.equal(PL[l, :, :nk], po), l
    for l in (0, L - 1):
        n_ex = check_selection(host(idx[l]), host(SL[l]).astype(np.float64), segments, budgets, band=0.0)
        assert n_ex == 0
    print(f"stack compaction gamma={gamma} ok, Nk_packed={nk}", flush=True)


def test_rolling_steps_at_full_frame_size():
    """The rolling step at the shape of the 28-layer rollout: 24 query / 8 KV heads, 48x84-token
    frames, 256 text tokens, 512 scoring rows, gamma 0.85 with a 512-token minimum, cache packed
    in place, attention cut into key shares, softmax scale folded into the queries.  Every step starts from the ORACLE's cache after the
    previous step (so a selection that falls inside the score band cannot carry over), and is
    compared with the oracle's next state: segment table, kept rows (bit-exact outside the band),
    moved K / V / positions, and the attention of 64 sampled query rows per head."""
    from paper_2601_04359_amd.rollout import RollingLayer
    gamma, b_min, n_steps = 0.85, 512, 4
    case = synth.rolling_case(seed=7, n_steps=n_steps, hq=24, hkv=8, d=128, n_text=256, gh=48, gw=84, n_score=512)
    rnd = orc.round_to_bf16
    aK = rnd(orc.rope3d(case.anchor_K, case.anchor_pos, case.sections, case.base))
    frames = [(rnd(orc.rope3d(K, p, case.sections, case.base)), V, p) for K, V, p in case.frames]
    q_scale, scale = q_fold(case.scale), LN2   # the form bench.py's rollout runs
    queries = [rnd(orc.rope3d(Q, p, case.sections, case.base) * q_scale)
               for Q, p in zip(case.queries, case.query_pos)]
    n, Hkv = case.n_frame, case.Hkv
    rows = np.union1d(case.score_rows, synth.strided_rows(n, N_SAMPLE_ROWS))   # the rows the oracle is given
    score_sub = np.searchsorted(rows, case.score_rows)
    sample_sub = np.searchsorted(rows, synth.strided_rows(n, N_SAMPLE_ROWS))
    budget_fn = lambda w: orc.budget_pow(n, w, gamma, b_min)
    want = orc.rolling_rollout(aK, case.anchor_V, case.anchor_pos, case.anchor_segments, frames,
                               [Q[:, rows] for Q in queries], scale, budget_fn, score_rows=score_sub)
    capacity = case.anchor_K.shape[1] + n_steps * n

    def insert(layer, K, V, pos_h, kind, frame):
        m = K.shape[1]
        k, v, pp = layer.reserve(m)
        k.copy_(dev(np.asarray(K, dtype=np.float32), "bf16"))
        v.copy_(dev(np.asarray(V, dtype=np.float32), "bf16"))
        pp.copy_(dev(np.ascontiguousarray(pos_h, dtype=np.int32), None))
        layer.commit(m, kind, frame)

    exempted = 0
    for i, Q in enumerate(queries):
        layer = RollingLayer(case.Hq, Hkv, case.D, capacity, n, case.scale, mode="pow", gamma=gamma, b_min=b_min,
                             n_score=case.score_rows.size, sections=case.sections, base=case.base, device=DEV,
                             fold_scale=True)
        assert np.array_equal(host(layer.q_rows), case.score_rows)
        if i == 0:
            pre = {"K": aK, "V": case.anchor_V, "segments": list(case.anchor_segments),
                   "pos": np.broadcast_to(case.anchor_pos[None], (Hkv,) + case.anchor_pos.shape)}
        else:
            pre = want[i - 1]
        for (start, length, kind, frame) in pre["segments"]:
            insert(layer, pre["K"][:, start:start + length], pre["V"][:, start:start + length],
                   pre["pos"][:, start:start + length], kind, frame)
        if i >= 1:
            Kf, Vf, pf = frames[i - 1]
            insert(layer, Kf, Vf, np.broadcast_to(pf[None], (Hkv,) + pf.shape), pk.PC_SEG_FRAME, i)
        segs_pre, nk_pre = list(layer.segments), layer.nk
        K_pre, V_pre, pos_pre = (np.asarray(pre[k], dtype=t) for k, t in (("K", np.float64), ("V", np.float64),
                                                                          ("pos", np.int32)))
        if i >= 1:
            K_pre, V_pre = np.concatenate([K_pre, Kf], 1), np.concatenate([V_pre, Vf.astype(np.float64)], 1)
            pos_pre = np.concatenate([pos_pre, np.broadcast_to(pf[None], (Hkv,) + pf.shape)], 1)
        assert np.array_equal(host(layer.K[:, :nk_pre]), K_pre) and np.array_equal(host(layer.V[:, :nk_pre]), V_pre)
        assert np.array_equal(host(layer.pos[:, :nk_pre]), pos_pre)    # the device starts from the oracle's bits
        O = layer.step(dev(Q.astype(np.float32), "bf16"))
        w = want[i]
        nk = layer.nk
        assert layer.segments == w["segments"] and nk == w["K"].shape[1], i
        pos_got = host(layer.pos[:, :nk])
        # source row of every kept row: (t, h, w) is unique inside the cache
        code = lambda p: (p[..., 0].astype(np.int64) * 4096 + p[..., 1]) * 4096 + p[..., 2]
        idx = np.empty((Hkv, nk), dtype=np.int64)
        for h in range(Hkv):
            order = np.argsort(code(pos_pre[h]), kind="stable")
            at = np.searchsorted(code(pos_pre[h])[order], code(pos_got[h]))
            idx[h] = order[at]
            assert np.array_equal(pos_pre[h][idx[h]], pos_got[h])
        if not np.array_equal(pos_got, w["pos"]):   # allowed only inside the score band
            n_past = sum(1 for s in segs_pre if s[2] == pk.PC_SEG_FRAME)
            per_d = budget_fn(n_past)
            budgets, d = [], n_past
            for s in segs_pre:
                budgets.append(per_d[d - 1] if s[2] == pk.PC_SEG_FRAME else s[1])
                d -= s[2] == pk.PC_SEG_FRAME
            sco = orc.score(Q[:, case.score_rows], K_pre, scale)
            exempted += check_selection(idx, sco, segs_pre, budgets, band=BAND)
        Kg, Vg = host(layer.K[:, :nk]).astype(np.float64), host(layer.V[:, :nk]).astype(np.float64)
        for h in range(Hkv):
            assert np.array_equal(Kg[h], K_pre[h][idx[h]]) and np.array_equal(Vg[h], V_pre[h][idx[h]])
        Ow, _ = orc.frame_attn(Q[:, rows[sample_sub]], Kg, Vg, scale)
        err = np.abs(host(O)[:, rows[sample_sub]].astype(np.float64) - Ow)
        assert err.max() <= 2e-2 and err.mean() <= 2e-3, (i, err.max(), err.mean())
        if np.array_equal(pos_got, w["pos"]):
            err = np.abs(host(O)[:, rows].astype(np.float64) - w["O"])
            assert err.max() <= 2e-2 and err.mean() <= 2e-3, (i, err.max(), err.mean())
        print(f"step {i + 1}: Nk {nk_pre} -> {nk}, band-exempt keys so far {exempted}", flush=True)
        del layer
