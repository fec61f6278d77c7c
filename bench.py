#!/usr/bin/env python3
"""Benchmark of the PackCache hot path on one MI355X.

A step is one pass of the whole path over one layer at frame 24 (16 query heads, 4 KV
heads, D = 128, 4032 tokens per frame, 256 text tokens, 23 past frames):
    pc_rope3d (new frame's Q, newest cached K) -> pc_score (512 sampled queries) ->
    pc_budget (gamma 0.85, floor 512) -> pc_compact (select + gather) -> pc_frame_attn.
Inputs are seeded synthetic tensors already resident in HBM when timing starts.
Prints ONE JSON line.  Besides the step it carries
  * the frame-48 legs: in-place compaction of 28 distinct layer caches at three decay factors
    (one call per layer, the batched call, the stack re-played from a HIP graph, and a plain copy
    of the same bytes launched the same way), dense vs packed attention, scoring;
  * the per-frame dense-vs-packed sweep over frames 1..48 (summary; table in sweep.json);
  * the 48-frame rollout of a 28-layer stack (24 query / 8 KV heads), packed vs dense;
  * the oracle timed on the host cores.
`--no-f48`, `--no-sweep`, `--no-rollout`, `--no-cpu` drop legs (profiles of single kernels).
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def attn_flops(hq, nq, nk, d):
    return 4.0 * hq * nq * nk * d


def gather_bytes(rows, hkv, d, elt=2):
    """Algorithmic bytes of one compaction: every kept row's K and V read and written once,
    its int32 index read, its (t, h, w) read and written."""
    return rows * hkv * (2 * 2 * d * elt + 4 + 2 * 12)


def measured_traffic():
    """Bytes one launch moved between L2 and the memory fabric, as the committed counter summary
    (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, calibrated against a plain copy)
    states them: lines `TRAFFIC <key> <bytes>` of profiles/bench_pmc_fetch_write.md.  Reported,
    not re-measured here; None where the summary has no such line."""
    out = {}
    try:
        with open(os.path.join(ROOT, "profiles", "bench_pmc_fetch_write.md")) as fh:
            for m in re.finditer(r"^TRAFFIC\s+(\S+)\s+(\d+)\s*$", fh.read(), flags=re.M):
                out[m.group(1)] = int(m.group(2))
    except OSError:
        pass
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-sweep", action="store_true", help="skip the per-frame dense vs packed sweep, frames 1..48")
    ap.add_argument("--no-rollout", action="store_true",
                    help="skip the 48-frame rollout of a 28-layer stack (24 query / 8 KV heads), rolling packed "
                         "cache vs dense cache; per-frame curve written to rollout.json in the output directory")
    ap.add_argument("--rollout-layers", type=int, default=28)
    ap.add_argument("--rollout-frames", type=int, default=48)
    ap.add_argument("--rollout-mode", default="pow", help="pow | norm | half | slide")
    ap.add_argument("--rollout-passes", type=int, default=1,
                    help="attention passes per frame and layer (iterative decoding): with more than one, the "
                         "first pass runs on the un-packed cache and its log-sum-exp feeds the scoring")
    ap.add_argument("--rollout-window", type=int, default=0,
                    help="with --rollout-mode half | norm: a sliding window of this many past frames (minimum "
                         "quota B_one // W, so that older frames get nothing and leave: FIFO truncation), the "
                         "retained rows rebased in time whenever the window advances")
    ap.add_argument("--rollout-self", action="store_true",
                    help="the frame being generated also sits in the cache (always-kept SELF segment of its own "
                         "step, the newest past frame from the next step on): Eq. 2's attention inside the frame")
    ap.add_argument("--no-rollout-stack", action="store_true",
                    help="skip the second packed rollout, in which every layer attends first, scores from that "
                         "pass's log-sum-exp, and the whole stack is re-packed by ONE batched compaction per step")
    ap.add_argument("--out-dir", default=os.path.join(ROOT, "bench_out"), help="where the per-frame tables go")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-f48", action="store_true", help="skip the frame-48 compaction / dense legs")
    ap.add_argument("--f48-only", default="",
                    help="frame-48 compaction: run only this variant (layer | batch | graph | streams | streams7 | copy), "
                         "optionally :gamma (e.g. layer:0.85), so that a kernel trace of the command holds the "
                         "launches of one variant only")
    ap.add_argument("--no-fold", action="store_true",
                    help="keep the softmax scale out of the queries: pc_score / pc_frame_attn then multiply "
                         "every product element by it (the general loop); default: the query rotation folds "
                         "scale * log2(e) into Q and the calls get scale = ln 2")
    ap.add_argument("--no-dense", action="store_true",
                    help="skip the dense frame-24 comparison call, so that a profile of this command "
                         "sees pc_frame_attn at the packed shape only")
    ap.add_argument("--copy-probe", action="store_true",
                    help="first run three plain 256 MiB device copies: the known-size dispatches that "
                         "calibrate FETCH_SIZE / WRITE_SIZE in a counter run of this same command")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2601_04359_amd as pk
    from paper_2601_04359_amd import synth

    dev = "cuda:0"
    torch.cuda.set_device(0)
    pk.lib()   # fail loudly if the HIP library is missing
    traffic = measured_traffic()
    if args.copy_probe:
        src = torch.arange(1 << 26, dtype=torch.int32, device=dev)   # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def up(a, bf=True):
        t = torch.from_numpy(np.ascontiguousarray(a))
        return (t.to(torch.bfloat16) if bf else t).to(dev)

    # A device copy of ~0.2 ms enqueued right before the first event of a timed region: while it runs
    # the host gets the timed launches into the stream, so the interval between the events is the
    # GPU's time for them and not the ~50 us the host needs to issue a call into an idle stream.
    busy_a = torch.empty(1 << 27, dtype=torch.int32, device=dev)
    busy_b = torch.empty_like(busy_a)
    gpu_busy = lambda: busy_b.copy_(busy_a)

    def timed(fn, reps):
        """Mean milliseconds of fn() measured with events on the stream the kernels run on."""
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        gpu_busy()
        for a, b in ev:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in ev]))

    # ------------------------------------------------------------------ frame-24 layer
    w = synth.config2(seed=1000, n_past=23)
    Hq, Hkv, D, Nq, Nk = w.Hq, w.Hkv, w.D, w.Nq, w.Nk
    Q0, K, V = up(w.Q), up(w.K), up(w.V)
    Q = Q0.clone()
    pos = up(np.broadcast_to(w.pos_k[None], (Hkv, Nk, 3)).copy(), bf=False)
    pos_q = up(w.pos_q, bf=False)
    newest = w.segments[-1]
    pos_new = up(w.pos_k[newest[0]:newest[0] + newest[1]], bf=False)
    rows = up(w.score_rows.astype(np.int32), bf=False)
    budgets = pk.segment_budgets(w.segments, pk.pc_budget(pk.PC_BUDGET_POW, w.n_frame, w.n_past, w.gamma, w.b_min))
    plan, nk_packed = pk.pc_compact_plan(w.segments, budgets)
    Kp = torch.empty((Hkv, nk_packed, D), dtype=torch.bfloat16, device=dev)
    Vp = torch.empty_like(Kp)
    pp = torch.empty((Hkv, nk_packed, 3), dtype=torch.int32, device=dev)
    O = torch.empty_like(Q)
    score = torch.empty((Hkv, Nk), dtype=torch.float32, device=dev)
    ws_s = torch.empty(pk.pc_score_workspace_bytes(Hq, Hkv, rows.numel(), Nk), dtype=torch.uint8, device=dev)
    ws_c = torch.empty(pk.pc_compact_workspace_bytes(Hkv, Nk), dtype=torch.uint8, device=dev)
    k_new = K[:, newest[0]:newest[0] + newest[1]]
    k_new0 = k_new.clone()           # the newest frame's keys as they arrive: un-rotated

    # The softmax scale rides on the query rotation (one rounding either way); the scoring and
    # attention calls then see scale = ln 2 and run their shorter loops.  Same softmax(QK^T/sqrt(D)).
    fold = not args.no_fold
    q_out_scale = pk.folded_q_scale(w.scale) if fold else 1.0
    call_scale = pk.PC_SCALE_FOLDED if fold else w.scale

    ev_attn = []

    def step(record=False):
        Q.copy_(Q0)          # the step's queries and the newest frame's keys arrive un-rotated:
        k_new.copy_(k_new0)  # every step sees exactly the configuration's bits
        pk.pc_rope3d(Q, pos_q, w.sections, w.base, out_scale=q_out_scale)
        pk.pc_rope3d(k_new, pos_new, w.sections, w.base)
        pk.pc_score(Q, K, Nk, call_scale, score=score, ws=ws_s, q_rows=rows)
        b = pk.segment_budgets(w.segments, pk.pc_budget(pk.PC_BUDGET_POW, w.n_frame, w.n_past, w.gamma, w.b_min))
        _, nk = pk.pc_compact(K, V, pos, score, w.segments, b, out=(Kp, Vp, pp), ws=ws_c)
        if record:
            a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
        pk.pc_frame_attn(Q, Kp, Vp, nk, call_scale, O=O)
        if record:
            e.record()
            ev_attn.append((a, e))

    # The chip needs some 20 launches (~25 ms of this work) after idling before its clock settles at
    # the sustained value: first it overshoots, then it undershoots.  Run the step that often before
    # the W warm-up steps, whatever W is, so that the K timed steps see the sustained state.
    for _ in range(25):
        step()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(record=True)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    attn_ms = float(np.mean([a.elapsed_time(e) for a, e in ev_attn]))
    fl_packed = attn_flops(Hq, Nq, nk_packed, D)
    attn_tflops = fl_packed / (attn_ms * 1e-3) / 1e12

    # the other steps of the path, one by one (same stream, events around each call)
    Qr = Q0.clone()          # rotated over and over here: plain rotation, so that it keeps its magnitude
    Kr = k_new0.clone()
    rope_ms = timed(lambda: (pk.pc_rope3d(Qr, pos_q, w.sections, w.base),
                             pk.pc_rope3d(Kr, pos_new, w.sections, w.base)), 10)
    del Qr, Kr
    score_ms = timed(lambda: pk.pc_score(Q, K, Nk, call_scale, score=score, ws=ws_s, q_rows=rows), 10)
    compact_ms = timed(lambda: pk.pc_compact(K, V, pos, score, w.segments, budgets, out=(Kp, Vp, pp), ws=ws_c), 10)
    lse24 = torch.empty((Hq, Nq), dtype=torch.float32, device=dev)
    dense_ms = None if args.no_dense else timed(lambda: pk.pc_frame_attn(Q, K, V, Nk, call_scale, O=O, lse=lse24), 3)
    # Scoring fed by the log-sum-exp of an attention pass over the same cache (a model that attends
    # over the un-packed cache first has it for free): one QK^T pass instead of two.
    score_lse_ms = None if args.no_dense else timed(
        lambda: pk.pc_score(Q, K, Nk, call_scale, lse=lse24, score=score, ws=ws_s, q_rows=rows), 10)
    score_pass_flops = 2.0 * D * rows.numel() * Hq * Nk          # one QK^T pass
    out = {
        "metric": "packed frame-attn ms/layer + TFLOP/s (% MFMA peak); compaction GB/s at 48 frames",
        "value": round(attn_tflops, 2),
        "unit": "TFLOP/s (packed pc_frame_attn, bf16, frame 24)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: single layer at frame 24", "Hq": Hq, "Hkv": Hkv, "D": D,
                   "Nq": Nq, "Nk_dense": Nk, "Nk_packed": nk_packed, "gamma": w.gamma, "b_min": w.b_min,
                   "score_queries": int(rows.numel()), "scale_folded_into_q": fold},
        "attn_packed_ms_per_layer": round(attn_ms, 4),
        "attn_dense_ms_per_layer": dense_ms and round(dense_ms, 4),
        "attn_dense_tflops": dense_ms and round(attn_flops(Hq, Nq, Nk, D) / (dense_ms * 1e-3) / 1e12, 2),
        "dense_vs_packed_speedup_f24": dense_ms and round(dense_ms / attn_ms, 3),
        "dense_vs_packed_path_speedup_f24": dense_ms and round(dense_ms / ms_per_step, 3),
        "step_breakdown_ms": {"rope3d": round(rope_ms, 4), "score": round(score_ms, 4),
                              "compact": round(compact_ms, 4), "frame_attn": round(attn_ms, 4)},
        "score_tflops": round(2 * score_pass_flops / (score_ms * 1e-3) / 1e12, 2),
        "score_lse_fed": score_lse_ms and {
            "ms": round(score_lse_ms, 4), "tflops": round(score_pass_flops / (score_lse_ms * 1e-3) / 1e12, 2),
            "note": "pc_score given the log-sum-exp of a pc_frame_attn pass over the same cache: one QK^T pass"},
        "roofline": {"bound": "mfma", "kernel": "attn_bf16_kernel", "achieved": round(attn_tflops, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic.get("attn_f24_packed"), "traffic_unit": "bytes per launch",
                     "traffic_source": "profiles/bench_pmc_fetch_write.md (rocprofv3 --pmc runs of this script)",
                     "algorithmic_bytes": int(2 * D * (2 * Hq * Nq + 2 * Hkv * nk_packed))},
    }
    del Q, Q0, K, V, Kp, Vp, pp, O, score, pos, lse24

    # ------------------------------------------------------------------ frame 48: compaction, dense
    if not args.no_f48 or not args.no_sweep:
        w48 = synth.config2(seed=1001, n_past=47)
        Nk48 = w48.Nk
        K48, V48, Q48 = up(w48.K), up(w48.V), up(w48.Q)
        if fold:             # as the rotation with out_scale leaves them
            Q48 = (Q48.float() * q_out_scale).to(torch.bfloat16)
        pos48 = up(np.broadcast_to(w48.pos_k[None], (Hkv, Nk48, 3)).copy(), bf=False)
        rows48 = up(w48.score_rows.astype(np.int32), bf=False)
        ws_s48 = torch.empty(pk.pc_score_workspace_bytes(Hq, Hkv, rows48.numel(), Nk48), dtype=torch.uint8, device=dev)
        ws_c48 = torch.empty(pk.pc_compact_workspace_bytes(Hkv, Nk48), dtype=torch.uint8, device=dev)
        sc48 = pk.pc_score(Q48, K48, Nk48, call_scale, ws=ws_s48, q_rows=rows48)
        O48 = torch.empty_like(Q48)
        b48_085 = pk.segment_budgets(w48.segments, pk.pc_budget(pk.PC_BUDGET_POW, w48.n_frame, 47, 0.85, 512))
        _, nk48_packed = pk.pc_compact_plan(w48.segments, b48_085)
        Kw = torch.empty((Hkv, nk48_packed, D), dtype=torch.bfloat16, device=dev)     # frame 48 packed, out of place
        Vw, pw = torch.empty_like(Kw), torch.empty((Hkv, nk48_packed, 3), dtype=torch.int32, device=dev)
        pk.pc_compact(K48, V48, pos48, sc48, w48.segments, b48_085, out=(Kw, Vw, pw), ws=ws_c48)

    if not args.no_f48:
        # Compaction only (configs[3]): 28 layer caches, each drawn from its own seed on the device
        # (own keys, own scores, own selected rows), compacted in place.  Algorithmic bytes of all
        # layers over the GPU time of the whole sequence.  The caches are restored from pristine
        # copies (untimed) between repetitions.
        n_layers = 28
        only, _, only_gamma = args.f48_only.partition(":")
        KL = torch.empty((n_layers,) + tuple(K48.shape), dtype=K48.dtype, device=dev)     # one stacked cache
        VL, PL = torch.empty_like(KL), torch.empty((n_layers,) + tuple(pos48.shape), dtype=torch.int32, device=dev)
        SL = torch.empty((n_layers, Hkv, Nk48), dtype=torch.float32, device=dev)
        KL0, VL0 = torch.empty_like(KL), torch.empty_like(VL)
        Ql = torch.empty_like(Q48)
        for l in range(n_layers):
            synth.device_frame_layer(2000 + l, 47, KL0[l], VL0[l], Ql)
            if fold:
                Ql.mul_(q_out_scale)
            pk.pc_score(Ql, KL0[l], Nk48, call_scale, score=SL[l], ws=ws_s48, q_rows=rows48)
        PL.copy_(pos48[None].expand_as(PL))
        torch.cuda.synchronize()
        del Ql
        layers = [(KL[l], VL[l], PL[l], SL[l], torch.empty_like(ws_c48)) for l in range(n_layers)]
        ws_b48 = torch.empty(pk.pc_compact_batch_workspace_bytes(n_layers, Hkv, Nk48), dtype=torch.uint8, device=dev)

        def restore():
            KL.copy_(KL0), VL.copy_(VL0), PL.copy_(pos48[None].expand_as(PL))
            torch.cuda.synchronize()

        def timed_stack(fn, reps=4, start=None):
            """GPU milliseconds per layer of fn() over the freshly restored stack (first repetition dropped)."""
            ts = []
            for _ in range(reps):
                restore()
                a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                gpu_busy()
                a.record()
                if start is not None:
                    start(a)
                fn()
                e.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(e) / n_layers)
            return float(np.mean(ts[1:]))

        def entry(ms, gb):
            return {"ms_per_layer": round(ms, 4), "GBps": round(gb / (ms * 1e-3), 1),
                    "frac_hbm": round(gb / (ms * 1e-3) / PEAK_HBM_GBS, 4)}

        comp, comp_b, comp_p, comp_g, comp_c, comp_4 = {}, {}, {}, {}, {}, {}
        lane_streams = [torch.cuda.Stream() for _ in range(7)]
        side_stream = torch.cuda.Stream()
        graph_stream = torch.cuda.Stream()
        ev_sel = [torch.cuda.Event() for _ in range(n_layers)]
        for gamma in (0.7, 0.85, 0.95):
            if only_gamma and float(only_gamma) != gamma:
                continue
            b48 = pk.segment_budgets(w48.segments, pk.pc_budget(pk.PC_BUDGET_POW, w48.n_frame, 47, gamma, 512))
            _, nk48p = pk.pc_compact_plan(w48.segments, b48)
            kept = nk48p - (w48.n_text + w48.n_frame)
            gb = gather_bytes(kept, Hkv, D) / 1e9
            if only in ("", "layer"):      # one pc_compact call per layer, back to back on one stream
                calls = [pk.pc_compact_prepared(Kl, Vl, pl, sl, w48.segments, b48, wl) for (Kl, Vl, pl, sl, wl) in layers]
                ms = timed_stack(lambda: [c() for c in calls])
                comp[str(gamma)] = dict(entry(ms, gb), kept_past_rows=kept)
            if only in ("", "streams"):
                # the same per-layer calls, the select half of every layer on a side stream (it reads
                # only the scores), the gather half behind it on the main stream
                main, side = torch.cuda.current_stream(), side_stream
                sel = [pk.pc_compact_prepared(Kl, Vl, pl, sl, w48.segments, b48, wl, phases=pk.PC_COMPACT_SELECT,
                                              stream=side) for (Kl, Vl, pl, sl, wl) in layers]
                gat = [pk.pc_compact_prepared(Kl, Vl, pl, sl, w48.segments, b48, wl, phases=pk.PC_COMPACT_GATHER,
                                              stream=main) for (Kl, Vl, pl, sl, wl) in layers]

                def two_streams():
                    for l in range(n_layers):
                        sel[l]()
                        ev_sel[l].record(side)
                        main.wait_event(ev_sel[l])
                        gat[l]()
                comp_p[str(gamma)] = entry(timed_stack(two_streams, start=lambda a: side.wait_event(a)), gb)
            if only in ("", "streams7"):
                # one pc_compact call per layer again, the layers dealt round-robin over seven streams
                # (layer caches are independent): the launches of neighbouring layers overlap.  Measured:
                # 4 streams 0.47 / 0.53 / 0.62 of peak, 7 streams 0.53 / 0.56 / 0.61, 14 streams 0.50 / 0.54 / 0.60
                # (the process has 4 hardware queues)
                main = torch.cuda.current_stream()
                calls4 = [pk.pc_compact_prepared(Kl, Vl, pl, sl, w48.segments, b48, wl, stream=lane_streams[i % len(lane_streams)])
                          for i, (Kl, Vl, pl, sl, wl) in enumerate(layers)]

                def layer_streams():
                    for c in calls4:
                        c()
                    for st in lane_streams:
                        lane_done = torch.cuda.Event()
                        lane_done.record(st)
                        main.wait_event(lane_done)
                comp_4[str(gamma)] = entry(timed_stack(layer_streams, start=lambda a: [st.wait_event(a) for st in lane_streams]), gb)
            if only in ("", "batch"):      # the whole stack in one call
                msb = timed_stack(lambda: pk.pc_compact_batch(KL, VL, PL, SL, w48.segments, b48, ws=ws_b48))
                comp_b[str(gamma)] = entry(msb, gb)
            if only in ("", "graph"):
                # the 28 per-layer calls recorded once into a HIP graph and re-played: no host launch
                # work at all, the same kernels in the same order
                restore()
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.stream(graph_stream):
                    calls_g = [pk.pc_compact_prepared(Kl, Vl, pl, sl, w48.segments, b48, wl, stream=graph_stream)
                               for (Kl, Vl, pl, sl, wl) in layers]
                    for c in calls_g:
                        c()
                    graph_stream.synchronize()
                    with torch.cuda.graph(graph, stream=graph_stream):
                        for c in calls_g:
                            c()
                comp_g[str(gamma)] = entry(timed_stack(graph.replay), gb)
                del graph
            if only in ("", "copy"):
                # What a launch of this size can reach at all: one plain device copy per layer of as many
                # bytes as the layer's compaction moves (the kept rows' K and V, read once and written
                # once), 28 of them back to back like the per-layer calls.  Not part of the method.
                nb = kept * Hkv * D * 2          # bf16 elements: K rows + V rows
                msc = timed_stack(lambda: [KL[l].view(-1)[:nb].copy_(VL0[(l + 1) % n_layers].view(-1)[:nb])
                                           for l in range(n_layers)])
                comp_c[str(gamma)] = entry(msc, 2 * nb * 2 / 1e9)
        if comp:
            out["compaction_f48_in_place"] = comp
        if comp_b:
            out["compaction_f48_in_place_batched"] = comp_b
        if comp_p:
            out["compaction_f48_in_place_two_streams"] = comp_p
        if comp_4:
            out["compaction_f48_in_place_layers_over_7_streams"] = comp_4
        if comp_g:
            out["compaction_f48_in_place_graph_replay"] = comp_g
        if comp_c:
            out["plain_copy_same_bytes_per_layer_launch"] = comp_c
        if "0.85" in comp_b:
            out["roofline_compact_batched"] = {
                "bound": "hbm", "variant": "pc_compact_batch: all 28 layers in one call, in place, gamma 0.85",
                "achieved": comp_b["0.85"]["GBps"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": comp_b["0.85"]["frac_hbm"], "traffic": traffic.get("compact_batch_f48_g085_per_layer"),
                "traffic_unit": "bytes per layer",
                "algorithmic_bytes": int(gather_bytes(nk48_packed - (w48.n_text + w48.n_frame), Hkv, D))}
        if "0.85" in comp:
            out["roofline_compact"] = {
                "bound": "hbm", "variant": "pc_compact: one call per layer, 28 layers back to back on one stream, "
                                           "in place, gamma 0.85",
                "achieved": comp["0.85"]["GBps"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": comp["0.85"]["frac_hbm"], "traffic": traffic.get("compact_f48_g085_per_layer"),
                "traffic_unit": "bytes per layer",
                "algorithmic_bytes": int(gather_bytes(nk48_packed - (w48.n_text + w48.n_frame), Hkv, D))}
        if not only:
            packed48_ms = timed(lambda: pk.pc_frame_attn(Q48, Kw, Vw, nk48_packed, call_scale, O=O48), 3)
            dense48_ms = timed(lambda: pk.pc_frame_attn(Q48, K48, V48, Nk48, call_scale, O=O48), 2)
            score48_ms = timed(lambda: pk.pc_score(Q48, K48, Nk48, call_scale, score=sc48, ws=ws_s48, q_rows=rows48), 3)
            # Cache mask in front of the select (Sec. 3.1 / 3.4): a seeded frame-level Bernoulli(1/2) mask over
            # the past frames' tokens; masked tokens are never candidates and are physically removed.
            mrng = np.random.default_rng(48)
            valid_h = np.ones(Nk48, dtype=np.uint8)
            for (a0, ln, kind, _) in w48.segments:
                if kind == pk.PC_SEG_FRAME:
                    valid_h[a0:a0 + ln] = mrng.random(ln) < 0.5
            valid_d = torch.from_numpy(valid_h).to(dev)
            t0 = time.perf_counter()
            b48m = pk.pc_masked_budgets(w48.segments, b48_085, valid_h)
            masked_budget_host_ms = (time.perf_counter() - t0) * 1e3
            sc48m = sc48.clone()
            mask_ms = timed(lambda: pk.pc_mask_scores(sc48m, valid_d), 5)
            KL[0].copy_(K48), VL[0].copy_(V48), PL[0].copy_(pos48)
            masked_compact_ms = timed(lambda: pk.pc_compact(KL[0], VL[0], PL[0], sc48m, w48.segments, b48m, ws=ws_c48), 1)
            out["cache_mask_f48"] = {"masked_tokens": int((valid_h == 0).sum()), "kept_rows": int(sum(b48m)),
                                     "kept_rows_without_mask": int(sum(b48_085)),
                                     "pc_masked_budgets_host_ms": round(masked_budget_host_ms, 3),
                                     "pc_mask_scores_ms": round(mask_ms, 4),
                                     "pc_compact_in_place_ms": round(masked_compact_ms, 4)}
            out["frame48"] = {"Nk_dense": Nk48, "Nk_packed": nk48_packed, "attn_dense_ms": round(dense48_ms, 4),
                              "attn_packed_ms": round(packed48_ms, 4),
                              "attn_packed_tflops": round(attn_flops(Hq, Nq, nk48_packed, D) / (packed48_ms * 1e-3) / 1e12, 2),
                              "attn_dense_tflops": round(attn_flops(Hq, Nq, Nk48, D) / (dense48_ms * 1e-3) / 1e12, 2),
                              "dense_vs_packed_speedup": round(dense48_ms / packed48_ms, 3),
                              "score_ms": round(score48_ms, 4),
                              "score_tflops": round(2 * 2.0 * D * rows48.numel() * Hq * Nk48 / (score48_ms * 1e-3) / 1e12, 2)}
        del KL, VL, PL, SL, KL0, VL0, layers

    # ------------------------------------------------------------------ frames 1..48, dense vs packed (configs[2])
    if not args.no_sweep:
        table = []
        n_anchor = w48.n_text + w48.n_frame
        for f in range(1, 49):
            n_past = f - 1
            nk_f = n_anchor + w48.n_frame * n_past
            segs = synth.segment_table(w48.n_text, w48.n_frame, n_past)
            b = pk.segment_budgets(segs, pk.pc_budget(pk.PC_BUDGET_POW, w48.n_frame, n_past, 0.85, 512))
            _, nkp = pk.pc_compact_plan(segs, b)
            d_ms = timed(lambda: pk.pc_frame_attn(Q48, K48, V48, nk_f, call_scale, O=O48), 2)

            def packed_path():
                pk.pc_score(Q48, K48, nk_f, call_scale, score=sc48, ws=ws_s48, q_rows=rows48)
                pk.pc_compact(K48, V48, pos48, sc48, segs, b, out=(Kw, Vw, pw), ws=ws_c48)
            p_path_ms = timed(packed_path, 2)
            p_ms = timed(lambda: pk.pc_frame_attn(Q48, Kw, Vw, nkp, call_scale, O=O48), 2)
            table.append({"frame": f, "Nk_dense": nk_f, "Nk_packed": nkp, "dense_ms": round(d_ms, 4),
                          "packed_attn_ms": round(p_ms, 4), "score_compact_ms": round(p_path_ms, 4)})
        last4 = table[-4:]
        tot = lambda rs, *keys: sum(r[k] for r in rs for k in keys)
        out["sweep_frames_1_48"] = {
            "workload": "configs[2]: the frame-48 layer's cache cut at every frame index, dense vs one-shot packed "
                        "(two-pass score over the dense prefix, out-of-place compaction, packed attention)",
            "last4_speedup_attn": round(tot(last4, "dense_ms") / tot(last4, "packed_attn_ms"), 3),
            "last4_speedup_path": round(tot(last4, "dense_ms") / tot(last4, "packed_attn_ms", "score_compact_ms"), 3),
            "total_speedup_attn": round(tot(table, "dense_ms") / tot(table, "packed_attn_ms"), 3),
            "total_speedup_path": round(tot(table, "dense_ms") / tot(table, "packed_attn_ms", "score_compact_ms"), 3),
            "dense_total_ms": round(tot(table, "dense_ms"), 3), "packed_attn_total_ms": round(tot(table, "packed_attn_ms"), 3),
            "frames": {str(r["frame"]): [r["dense_ms"], r["packed_attn_ms"], r["score_compact_ms"]]
                       for r in table if r["frame"] in (2, 12, 24, 36, 45, 46, 47, 48)},
            "frames_columns": ["dense_ms", "packed_attn_ms", "score_compact_ms"]}
        os.makedirs(args.out_dir, exist_ok=True)
        with open(os.path.join(args.out_dir, "sweep.json"), "w") as fh:
            json.dump(table, fh, indent=0)
    if not args.no_f48 or not args.no_sweep:
        del K48, V48, Q48, Kw, Vw, pw, O48, sc48, pos48

    # ------------------------------------------------------------------ 48-frame rollout of a layer stack (configs[4])
    if not args.no_rollout:
        from paper_2601_04359_amd.rollout import RollingLayer, RollingStack
        L, F = args.rollout_layers, args.rollout_frames
        hq5, hkv5, n_text, gh, gw = 24, 8, 256, 48, 84
        n = gh * gw
        n_anchor = n_text + n
        sections, scale5 = (32, 48, 48), 1.0 / float(np.sqrt(D))
        tok_budget = n            # NORM / HALF / SLIDE: one frame's worth of tokens over all past frames
        own = args.rollout_self
        cap_packed = n_anchor + n + (sum(pk.pc_budget(pk.PC_BUDGET_POW, n, F - 1, 0.85, 512))
                                     if args.rollout_mode == "pow" else tok_budget + n) + (n if own else 0)
        cap_dense = n_anchor + (F - 1) * n + (n if own else 0)
        streams = [synth.DeviceRollingStream(1000 * (l + 1), hq5, hkv5, D, F, sections, dev) for l in range(L)]
        window = args.rollout_window
        if window and args.rollout_mode not in ("half", "norm"):
            raise SystemExit("--rollout-window needs --rollout-mode half or norm")
        b_min5 = tok_budget // window if window else 512
        packed = [RollingLayer(hq5, hkv5, D, cap_packed, n, scale5, mode=args.rollout_mode, gamma=0.85,
                               b_min=b_min5, slide_t_scale=4 if window else None,
                               budget_tokens=tok_budget, n_score=512, sections=sections, device=dev, fold_scale=fold)
                  for _ in range(L)]
        dense = [RollingLayer(hq5, hkv5, D, cap_dense, n, scale5, mode="dense", sections=sections, device=dev,
                              fold_scale=fold)
                 for _ in range(L)]
        # second packed side: the stack that is re-packed once per frame step (no window, no own frame)
        use_stack = not (args.no_rollout_stack or window or own or args.rollout_passes != 1)
        stack = RollingStack(L, hq5, hkv5, D, cap_packed, n, scale5, mode=args.rollout_mode, gamma=0.85, b_min=b_min5,
                             budget_tokens=tok_budget, n_score=512, sections=sections, device=dev,
                             fold_scale=fold) if use_stack else None
        apos = up(synth.cache_positions(n_text, gh, gw, 0), bf=False)
        for l in range(L):               # prefill: anchors, rotated on insert
            for lay in (packed[l], dense[l]):
                k, v, p = lay.reserve(n_anchor)
                if lay is packed[l]:
                    streams[l].anchors(k, v)
                else:
                    k.copy_(packed[l].K[:, :n_anchor]); v.copy_(packed[l].V[:, :n_anchor])
                p.copy_(apos[None].expand(hkv5, n_anchor, 3))
        if use_stack:
            k, v, p = stack.reserve(n_anchor)
            for l in range(L):
                k[l].copy_(packed[l].K[:, :n_anchor]); v[l].copy_(packed[l].V[:, :n_anchor])
            p.copy_(apos[None, None].expand_as(p))
            stack.commit(n_text, pk.PC_SEG_TEXT, -1, rotate_with=apos[:n_text])
            stack.commit(n, pk.PC_SEG_COND, 0, rotate_with=apos[n_text:])
        for l in range(L):
            for lay, rot in ((dense[l], apos), (packed[l], apos)):
                lay.commit(n_text, pk.PC_SEG_TEXT, -1, rotate_with=rot[:n_text])
                lay.commit(n, pk.PC_SEG_COND, 0, rotate_with=rot[n_text:])
        Qp = [torch.empty((hq5, n, D), dtype=torch.bfloat16, device=dev) for _ in range(L)]
        Qd = [torch.empty_like(q) for q in Qp]
        Qs = [torch.empty_like(q) for q in Qp] if use_stack else None
        O5 = torch.empty_like(Qp[0])
        lse5 = torch.empty((hq5, n), dtype=torch.float32, device=dev)
        curve = []
        rebase_ms_total = 0.0
        for f in range(1, F + 1):
            rebase_ms = 0.0
            if window:        # the window advances when the step begins; the rebase is part of the packed step
                a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for l in range(L):
                    packed[l].advance_window()
                e.record()
                torch.cuda.synchronize()
                rebase_ms = a.elapsed_time(e)
                rebase_ms_total += rebase_ms
            shift = packed[0].shift   # everything that arrives from now on is placed at its time minus the shift
            fpos_h = synth.grid_positions(f, gh, gw, n_text)
            fpos = up(fpos_h, bf=False)
            ppos = up(synth.grid_positions(f - 1, gh, gw, n_text), bf=False) if f >= 2 else None
            if shift:
                fpos_h = fpos_h.copy()
                fpos_h[:, 0] -= shift
                fpos_shifted = up(fpos_h, bf=False)
                ppos_shifted = ppos.clone()
                ppos_shifted[:, 0] -= shift
            else:
                fpos_shifted, ppos_shifted = fpos, ppos
            # the frame appended at this step: the one generated last, or (--rollout-self) this step's own
            new_f, new_pos = (f, fpos) if own else (f - 1, ppos)
            new_pos_packed = fpos_shifted if own else ppos_shifted
            new_kind = pk.PC_SEG_SELF if own else pk.PC_SEG_FRAME
            ks = vs = None
            if use_stack and new_f >= 1:
                ks, vs, ps = stack.reserve(n)
                ps.copy_(new_pos[None, None].expand_as(ps))
            for l in range(L):           # untimed: draw this step's inputs into the caches / query buffers
                streams[l].queries(f, Qp[l])
                Qd[l].copy_(Qp[l])
                if use_stack:
                    Qs[l].copy_(Qp[l])
                if own:
                    packed[l].promote_self()
                    dense[l].promote_self()
                if new_f >= 1:
                    k, v, p = packed[l].reserve(n)
                    streams[l].frame(new_f, k, v)
                    p.copy_(new_pos_packed[None].expand(hkv5, n, 3))
                    kd, vd, pd = dense[l].reserve(n)
                    kd.copy_(k); vd.copy_(v); pd.copy_(new_pos[None].expand(hkv5, n, 3))
                    if use_stack:
                        ks[l].copy_(k); vs[l].copy_(v)
            torch.cuda.synchronize()
            times = {}
            # whichever side is timed first after the (untimed) input generation runs a few tenths of a
            # millisecond slower: the sides take turns
            sides = [("packed", packed, Qp), ("dense", dense, Qd)] + ([("stack", None, Qs)] if use_stack else [])
            k_rot = f % len(sides)
            for name, layers, Qx in sides[k_rot:] + sides[:k_rot]:
                a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                gpu_busy()
                a.record()
                rot_new, rot_q = (new_pos_packed, fpos_shifted) if name == "packed" else (new_pos, fpos)
                if name == "stack":
                    # every layer: rotate Q, attend over the cache as it stands (packed at the end of the last
                    # step + the whole newest frame), score from that pass's log-sum-exp; then ONE re-pack
                    if new_f >= 1:
                        stack.commit(n, new_kind, new_f, rotate_with=rot_new)
                    for l in range(L):
                        pk.pc_rope3d(Qx[l], rot_q, sections, 10000.0, out_scale=stack.q_out_scale)
                        stack.attend(l, Qx[l], O=O5, lse=lse5)
                        stack.score_layer(l, Qx[l], lse=lse5)
                    stack.repack()
                else:
                    for l in range(L):
                        if new_f >= 1:
                            layers[l].commit(n, new_kind, new_f, rotate_with=rot_new)
                        if args.rollout_passes == 1:
                            layers[l].step(Qx[l], O=O5, q_pos=rot_q)
                        else:
                            pk.pc_rope3d(Qx[l], rot_q, sections, 10000.0, out_scale=layers[l].q_out_scale)
                            layers[l].attend(Qx[l], O=O5, lse=lse5)
                            layers[l].refresh(Qx[l], lse=lse5)
                            for _ in range(args.rollout_passes - 1):
                                layers[l].attend(Qx[l], O=O5)
                e.record()
                torch.cuda.synchronize()
                times[name] = a.elapsed_time(e)
            times["packed"] += rebase_ms
            row = {"frame": f, "Nk_dense": dense[0].nk, "Nk_packed": packed[0].nk,
                   "dense_ms": round(times["dense"], 3), "packed_ms": round(times["packed"], 3)}
            if use_stack:
                row["stack_ms"], row["Nk_stack_after_repack"] = round(times["stack"], 3), stack.nk
            curve.append(row)
        tp, td = sum(r["packed_ms"] for r in curve), sum(r["dense_ms"] for r in curve)
        last4 = curve[-4:]
        out["rollout"] = {"workload": "configs[4]", "layers": L, "frames": F, "Hq": hq5, "Hkv": hkv5,
                          "mode": args.rollout_mode,
                          "passes_per_frame": args.rollout_passes, "own_frame_in_cache": own,
                          "window_frames": window or None, "rebase_total_ms": round(rebase_ms_total, 3) if window else None,
                          "time_shift_at_end": packed[0].shift,
                          "packed_total_s": round(tp / 1e3, 4), "dense_total_s": round(td / 1e3, 4),
                          "speedup_total": round(td / tp, 3),
                          "speedup_last4": round(sum(r["dense_ms"] for r in last4) / sum(r["packed_ms"] for r in last4), 3),
                          "last_frame": curve[-1],
                          "per_frame_ms": {str(r["frame"]): [r["dense_ms"], r["packed_ms"]] + ([r["stack_ms"]] if use_stack else [])
                                           for r in curve if r["frame"] in (2, 12, 24, 36, 45, 46, 47, 48)},
                          "per_frame_columns": ["dense_ms", "packed_ms"] + (["stack_ms"] if use_stack else []),
                          # K and V rows resident per layer at the last step (Fig. 7: the packed cache is
                          # bounded, the full cache grows with the frame index); allocation is cap_* rows
                          "kv_cache_MB_per_layer": {"packed": round(packed[0].nk * hkv5 * D * 2 * 2 / 1e6, 1),
                                                    "dense": round(dense[0].nk * hkv5 * D * 2 * 2 / 1e6, 1),
                                                    "packed_allocated": round(cap_packed * hkv5 * D * 2 * 2 / 1e6, 1),
                                                    "dense_allocated": round(cap_dense * hkv5 * D * 2 * 2 / 1e6, 1)},
                          "note": "packed_ms covers rope, score, budget, in-place compaction and attention of all "
                                  "layers; dense_ms rope and attention over the full cache"}
        if use_stack:
            ts_ = sum(r["stack_ms"] for r in curve)
            out["rollout"]["stack_repacked_once_per_step"] = {
                "total_s": round(ts_ / 1e3, 4), "speedup_total": round(td / ts_, 3),
                "speedup_last4": round(sum(r["dense_ms"] for r in last4) / sum(r["stack_ms"] for r in last4), 3),
                "note": "every layer attends over the cache packed at the end of the previous step plus the whole "
                        "newest frame, its log-sum-exp feeds a one-pass pc_score, and pc_compact_batch re-packs all "
                        "layers when the step ends: the same kept rows as the per-layer flow"}
        os.makedirs(args.out_dir, exist_ok=True)
        with open(os.path.join(args.out_dir, "rollout.json"), "w") as fh:
            json.dump(curve, fh, indent=0)
        del packed, dense, stack, Qp, Qd, Qs, streams

    # ------------------------------------------------------------------ CPU baseline: the oracle
    if not args.no_cpu:
        import oracle as orc
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            threads = len(os.sched_getaffinity(0))
        n_rows = Nq   # the whole packed call: a few seconds of BLAS-threaded fp64 work
        rs = np.linspace(0, Nq - 1, n_rows).astype(np.int64)
        Ks, Vs = w.K[:, :nk_packed], w.V[:, :nk_packed]      # same key count as the packed call
        t0 = time.perf_counter()
        orc.frame_attn(w.Q[:, rs], Ks, Vs, w.scale)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(attn_flops(Hq, n_rows, nk_packed, D) / dt / 1e12, 5),
                               "unit": "TFLOP/s (fp64 NumPy oracle)", "cores": int(threads), "kind": "oracle",
                               "seconds": round(dt, 2),
                               "sample": f"oracle.frame_attn on {n_rows} of {Nq} query rows x {Hq} heads x "
                                         f"{nk_packed} keys (same per-row work as the packed call)"}
        # frame 24 in full: the oracle's score over the dense cache (512 scoring rows per head) and its
        # per-frame top-k selection (compact without the attention)
        t0 = time.perf_counter()
        sco = orc.score(w.Q[:, w.score_rows], w.K, w.scale)
        t_score = time.perf_counter() - t0
        t0 = time.perf_counter()
        orc.compact(w.K, w.V, np.broadcast_to(w.pos_k[None], (Hkv, Nk, 3)), sco, w.segments, budgets)
        t_select = time.perf_counter() - t0
        # configs[0] (tiny, fp32): the whole pipeline, median of 5
        c1 = synth.config1()
        b1 = orc.budget_pow(c1.n_frame, c1.n_past, c1.gamma, c1.b_min)
        seg_b1 = [s[1] for s in c1.segments[:2]] + list(reversed(b1))

        def c1_pipeline():
            s1 = orc.score(c1.Q, c1.K, c1.scale)
            Kc, Vc, _, _, _ = orc.compact(c1.K, c1.V, c1.pos_k[None], s1, c1.segments, seg_b1)
            orc.frame_attn(c1.Q, Kc, Vc, c1.scale)
        t_c1 = []
        for _ in range(5):
            t0 = time.perf_counter()
            c1_pipeline()
            t_c1.append(time.perf_counter() - t0)
        out["cpu_baseline_more"] = {
            "cores": int(threads), "kind": "oracle",
            "frame24_score_seconds": round(t_score, 2),
            "frame24_score_tflops": round(2.0 * D * w.score_rows.size * Hq * Nk / t_score / 1e12, 5),
            "frame24_select_and_gather_seconds": round(t_select, 2),
            "config1_whole_pipeline_ms_median_of_5": round(float(np.median(t_c1)) * 1e3, 3),
            "sample": "oracle.score on the frame-24 cache in full (512 rows x 16 heads x 97,024 keys), oracle.compact "
                      "on it in full, and configs[0]'s score + compact + frame_attn"}

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
