"""pc_compact_static (the entry point for callers that cannot allocate: its scratch is an array
inside the library) against pc_compact with a caller's workspace, through the C ABI: same packed
rows, positions, indices and tables, bit for bit, on two calls in a row, the second on a smaller
input (the array keeps the first call's contents; every call must clear what it uses)."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle as orc
import paper_2601_04359_amd as pk
from paper_2601_04359_amd import synth
from paper_2601_04359_amd.binding import pc_segment

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _raw_call(name, K, V, pos, score, segments, budgets, idx, ws=None):
    """The C entry point itself (ctypes), in place."""
    L = pk.lib()
    n = len(segments)
    seg = (pc_segment * n)(*[pc_segment(*map(int, s)) for s in segments])
    seg_out = (pc_segment * n)()
    b = (C.c_int32 * n)(*[int(v) for v in budgets])
    nk = C.c_int32(0)
    Hkv, _, D = K.shape
    args = [K.data_ptr(), V.data_ptr(), pos.data_ptr(), pk.PC_BF16, Hkv, D, K.stride(0), pos.stride(0),
            score.data_ptr(), score.stride(0), seg, n, b, 0, K.data_ptr(), V.data_ptr(), pos.data_ptr(),
            K.stride(0), pos.stride(0), idx.data_ptr(), idx.stride(0), seg_out, C.byref(nk)]
    stream = torch.cuda.current_stream().cuda_stream
    if name == "pc_compact":
        rc = L.pc_compact(*args, ws.data_ptr(), ws.numel(), stream)
    else:
        rc = L.pc_compact_static(*args, stream)
    assert rc == 0, L.pc_last_error_detail().decode()
    return [(s.start, s.len, s.kind, s.frame) for s in seg_out], nk.value


def _case(seed, n_past):
    w = synth.midsize(seed=seed, n_past=n_past)
    sc = orc.score(w.Q[:, w.score_rows], w.K, w.scale).astype(np.float32)
    budgets = pk.segment_budgets(w.segments, pk.pc_budget(pk.PC_BUDGET_POW, w.n_frame, w.n_past, w.gamma, w.b_min))
    bf = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).to(DEV)
    mk = lambda: (bf(w.K), bf(w.V),
                  torch.from_numpy(np.broadcast_to(w.pos_k[None], (w.Hkv, w.Nk, 3)).copy()).to(DEV),
                  torch.from_numpy(sc).to(DEV))
    return w, budgets, mk


def test_static_scratch_entry_matches_the_workspace_entry_twice_in_a_row():
    assert pk.pc_compact_static_capacity() == 4 << 20
    for seed, n_past in ((41, 9), (42, 4)):          # the second call is the smaller one
        w, budgets, mk = _case(seed, n_past)
        nk_out = pk.pc_compact_plan(w.segments, budgets)[1]
        Ka, Va, pa, sa = mk()
        Kb, Vb, pb, sb = mk()
        ia = torch.full((w.Hkv, nk_out), -1, dtype=torch.int32, device=DEV)
        ib = torch.full_like(ia, -2)
        ws = torch.empty(pk.pc_compact_workspace_bytes(w.Hkv, w.Nk), dtype=torch.uint8, device=DEV)
        seg_a, nk_a = _raw_call("pc_compact", Ka, Va, pa, sa, w.segments, budgets, ia, ws=ws)
        seg_b, nk_b = _raw_call("pc_compact_static", Kb, Vb, pb, sb, w.segments, budgets, ib)
        torch.cuda.synchronize()
        assert seg_a == seg_b and nk_a == nk_b == nk_out and nk_out < w.Nk
        assert torch.equal(ia, ib)
        assert torch.equal(Ka[:, :nk_out], Kb[:, :nk_out]) and torch.equal(Va[:, :nk_out], Vb[:, :nk_out])
        assert torch.equal(pa[:, :nk_out], pb[:, :nk_out])
        # and against the oracle's selection on the same scores (fp32 image; exact up to fp32 ties)
        want = orc.compact(w.K, w.V, np.broadcast_to(w.pos_k[None], (w.Hkv, w.Nk, 3)),
                           sb.cpu().numpy().astype(np.float64), w.segments, budgets)
        assert np.array_equal(ib.cpu().numpy(), want[3]) and seg_b == want[4]


def test_static_scratch_entry_rejects_what_does_not_fit():
    n = 300_000                                   # 8 heads x 300k rows of indices: beyond the array
    segs = [(0, n, pk.PC_SEG_COND, 0)]
    t = torch.empty((8, 16, 128), dtype=torch.bfloat16, device=DEV)    # never touched: rejected first
    p = torch.empty((8, 16, 3), dtype=torch.int32, device=DEV)
    s = torch.empty((8, 16), dtype=torch.float32, device=DEV)
    with pytest.raises(pk.PackCacheError) as e:
        pk.pc_compact_static(t, t, p, s, segs, [n])
    assert e.value.status == -6 and "scratch" in str(e.value)


def test_static_scratch_entry_replays_from_a_hip_graph():
    """What the entry point is for: a caller under graph capture.  After one eager call (which
    looks the array's address up) the call is recorded and re-played; every replay must give the
    eager result (the bookkeeping in the array is cleared by a kernel of the call itself)."""
    w, budgets, mk = _case(43, 7)
    nk_out = pk.pc_compact_plan(w.segments, budgets)[1]
    K0, V0, p0, sc = mk()
    K, V, p = K0.clone(), V0.clone(), p0.clone()
    idx = torch.empty((w.Hkv, nk_out), dtype=torch.int32, device=DEV)

    def step():
        K.copy_(K0), V.copy_(V0), p.copy_(p0)
        pk.pc_compact_static(K, V, p, sc, w.segments, budgets, idx=idx)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (K[:, :nk_out], V[:, :nk_out], p[:, :nk_out], idx)]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for replay in range(3):
        K.zero_(), idx.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (g, x) in enumerate(zip((K[:, :nk_out], V[:, :nk_out], p[:, :nk_out], idx), want)):
            assert torch.equal(g, x), f"replay {replay}: output {i} differs from the eager run"
