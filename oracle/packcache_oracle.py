"""fp64 CPU oracle of the PackCache hot path (arXiv 2601.04359).

TEST INFRASTRUCTURE ONLY -- never imported by the product path.  Plain NumPy in
double precision, one step per function, in the order the method takes them:

  rope3d      3D rotary embedding on (t, h, w) coordinates        Sec. 3.1, Eq. 2
  score       importance = column mass of the softmax probabilities
              (the paper only says "attention-relevant"; the column-mass
              reading is this build's, see `score`)                Sec. 3.4
  budget_*    per-frame token budgets from the decay kernel        Eq. 4-8
  select_topk per-frame top-k, ties toward the lower index         Sec. 3.4
  compact     physical removal of the dropped rows; anchors kept   Fig. 5(b), Sec. 3.4
  frame_attn  exact softmax attention over the keys presented      Eq. 2

Pins (tests/test_oracle_*.py): the half-life series printed under Eq. 7, the
geometric closed form of Eq. 6, the 8,417-token budget of Sec. 4.1, complex-number
1D RoPE, scipy's softmax/logsumexp, triple-loop brute force, closed-form attention
cases and the packed/dense/masked invariants.  The *selected sets* themselves are
"parity unpinned" against the paper: it prints no selected set and no attention
value, so beyond brute force on tiny inputs they are pinned only by this oracle.

No blocking, fusion or reordering: every function is the definition written out.
"""
from __future__ import annotations

from fractions import Fraction
from math import floor

import numpy as np

__all__ = [
    "SEG_TEXT", "SEG_COND", "SEG_FRAME", "SEG_SELF",
    "bf16_bits_to_f64", "round_to_bf16", "f64",
    "budget_pow", "budget_norm", "budget_half", "budget_slide",
    "rope_angles", "rope3d", "rebase",
    "logits", "softmax_rows", "score", "select_topk", "compact", "packed_segments", "masked_budgets",
    "frame_attn", "frame_attn_bruteforce", "score_bruteforce", "rolling_rollout",
]

SEG_TEXT, SEG_COND, SEG_FRAME, SEG_SELF = 0, 1, 2, 3


# --------------------------------------------------------------------------------------
# storage formats
# --------------------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) exactly to float64."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even); returned as float64 values.

    Models a bf16 store of a value held in fp32 registers: fp64 -> fp32 -> bf16.
    """
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(x))


def f64(x) -> np.ndarray:
    """Inputs arrive as float32/float64 arrays holding exactly representable values."""
    return np.asarray(x, dtype=np.float64)


# --------------------------------------------------------------------------------------
# budgets (Sec. 3.4, Eq. 4-8)
# --------------------------------------------------------------------------------------
def budget_pow(n_frame_tokens: int, n_past: int, gamma: float, b_min: int) -> list[int]:
    """Un-normalised decay budget b(d) = max(b_min, floor(N * gamma^d)), d = 1..n_past.

    The decay kernel g(d) = rho^d of Eq. 5 applied to a full frame of N tokens, with
    the minimum quota of Sec. 3.4 as a floor.  gamma is taken as the exact value of
    the double handed in, and the product is floored exactly (rational arithmetic).
    A frame never keeps more than it has: the result is clamped to N.
    """
    g = Fraction(gamma)
    out = []
    for d in range(1, n_past + 1):
        b = floor(n_frame_tokens * g ** d)
        out.append(min(n_frame_tokens, max(b_min, b)))
    return out


def _waterfill(b_one: int, shares: list[Fraction], q_min: int, n_total: int) -> list[int]:
    """t_d = q_min + floor((B_one - W q_min) * share_d); what flooring leaves over
    goes to the most recent frame, so that sum_d t_d = B_one (Eq. 8)."""
    w = len(shares)
    free = b_one - w * q_min
    t = [q_min + floor(free * s) for s in shares]
    if w:
        t[0] += b_one - sum(t)
    return t + [0] * (n_total - w)


def _active_window(b_one: int, w: int, q_min: int) -> int:
    """Minimum quota with FIFO truncation (Sec. 3.4): if W * b_min exceeds the whole
    budget the oldest frames are dropped until it does not."""
    if q_min <= 0:
        return w
    return min(w, b_one // q_min)


def budget_norm(b_one: int, w: int, rho: float, q_min: int = 0) -> list[int]:
    """Normalised allocation of Eq. 6: b_d = rho^d / sum_{j<=W} rho^j, t_d = B_one b_d."""
    we = _active_window(b_one, w, q_min)
    r = Fraction(rho)
    den = sum(r ** j for j in range(1, we + 1))
    shares = [r ** d / den for d in range(1, we + 1)]
    return _waterfill(b_one, shares, q_min, w)


def budget_half(b_one: int, w: int, q_min: int = 0) -> list[int]:
    """Closed-form half-life allocation of Eq. 7: b_d = 2^{-min(d, W-1)}."""
    we = _active_window(b_one, w, q_min)
    shares = [Fraction(1, 2 ** min(d, we - 1)) for d in range(1, we + 1)]
    return _waterfill(b_one, shares, q_min, w)


def budget_slide(b_one: int, w: int) -> list[int]:
    """Sliding-window baseline of Sec. 3.3: only the most recent frame is kept."""
    return [b_one] + [0] * (w - 1) if w > 0 else []


# --------------------------------------------------------------------------------------
# 3D rotary embedding (Sec. 3.1; spatially preserving positions, Sec. 3.4 / Eq. 9)
# --------------------------------------------------------------------------------------
def rope_angles(pos: np.ndarray, sections: tuple[int, int, int], base: float) -> np.ndarray:
    """Angle of every rotary pair: [n][D/2].

    The head dimension is cut into three contiguous sections (t, h, w).  Inside a
    section of width s, pair i is dims (2i, 2i+1) and turns by pos_axis * base^(-2i/s).
    """
    pos = np.asarray(pos, dtype=np.float64)
    cols = []
    for axis, s in enumerate(sections):
        i = np.arange(s // 2, dtype=np.float64)
        inv_freq = np.power(np.float64(base), -2.0 * i / np.float64(s))
        cols.append(pos[:, axis:axis + 1] * inv_freq[None, :])
    return np.concatenate(cols, axis=1)


def rope3d(x: np.ndarray, pos: np.ndarray, sections: tuple[int, int, int], base: float) -> np.ndarray:
    """Rotate x [H][n][D] by the 3D rotary operator R of Eq. 2; pos is int [n][3]."""
    x = f64(x)
    assert x.shape[-1] == sum(sections) and all(s % 2 == 0 for s in sections)
    phi = rope_angles(pos, sections, base)          # [n][D/2]
    c, s = np.cos(phi)[None], np.sin(phi)[None]
    x0, x1 = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = x0 * c - x1 * s
    out[..., 1::2] = x0 * s + x1 * c
    return out


def rebase(K: np.ndarray, pos: np.ndarray, delta_t: int, sections: tuple[int, int, int], base: float):
    """Temporal rebase of cached, already rotated keys (Sec. 3.4, the rebase equation):
    pos_t <- pos_t - delta_t with pos_h, pos_w fixed.  Rotations about one axis compose, so a
    key rotated at pos_t becomes the key rotated at pos_t - delta_t by one more rotation of
    -delta_t on the temporal section only.  K [H][n][D], pos [..][n][3] -> (K', pos')."""
    pos = np.asarray(pos)
    shift = np.zeros((K.shape[1], 3), dtype=np.int64)
    shift[:, 0] = -int(delta_t)
    out_pos = pos.copy()
    out_pos[..., 0] -= int(delta_t)
    return rope3d(K, shift, sections, base), out_pos


# --------------------------------------------------------------------------------------
# attention pieces (Eq. 2).  For one frame's queries against earlier frames and the
# anchors the causal mask is all-visible, so no mask appears.
# --------------------------------------------------------------------------------------
def logits(q_h: np.ndarray, k_g: np.ndarray, scale: float) -> np.ndarray:
    return (f64(q_h) @ f64(k_g).T) * np.float64(scale)


def softmax_rows(s: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    """Row softmax and log-sum-exp of a logit matrix."""
    m = np.max(s, axis=1, keepdims=True)
    e = np.exp(s - m)
    l = np.sum(e, axis=1, keepdims=True)
    return e / l, (m + np.log(l))[:, 0]


def frame_attn(Q, K, V, scale: float, keep: np.ndarray | None = None):
    """O = softmax(Q K^T * scale) V per query head; query head h reads KV head
    h // (Hq / Hkv).  `keep` ([Hkv][Nk] bool) masks dropped keys to -inf instead of
    removing them.  Returns (O [Hq][Nq][D], LSE [Hq][Nq])."""
    Q, K, V = f64(Q), f64(K), f64(V)
    hq, nq, d = Q.shape
    hkv = K.shape[0]
    rep = hq // hkv
    O = np.empty((hq, nq, d))
    L = np.empty((hq, nq))
    for h in range(hq):
        g = h // rep
        s = logits(Q[h], K[g], scale)
        if keep is not None:
            s = np.where(np.asarray(keep[g], dtype=bool)[None, :], s, -np.inf)
        p, lse = softmax_rows(s)
        O[h] = p @ V[g]
        L[h] = lse
    return O, L


def score(Qs, K, scale: float, share_heads: bool = False, valid=None) -> np.ndarray:
    """Importance of every cached key: the softmax probability it receives, summed
    over the scoring queries and over the query heads of its KV group.
    The softmax runs over ALL keys presented (anchors included).
    valid ([Nk] bool, the cache mask of Sec. 3.1 / Eq. 1, one flag per token for all heads):
    a masked key is ignored in attention, i.e. its logit is -inf: it receives no probability
    and does not count in any query's normaliser.  The same result as deleting the masked
    keys first (which is what the cache does with them, Sec. 3.4) and scoring the rest.
    Returns [Hkv][Nk], or [1][Nk] (summed over KV heads too) when share_heads."""
    Qs, K = f64(Qs), f64(K)
    hq, hkv = Qs.shape[0], K.shape[0]
    rep = hq // hkv
    out = np.zeros((hkv, K.shape[1]))
    for h in range(hq):
        s = logits(Qs[h], K[h // rep], scale)
        if valid is not None:
            s = np.where(np.asarray(valid, dtype=bool)[None, :], s, -np.inf)
        p, _ = softmax_rows(s)
        out[h // rep] += p.sum(axis=0)
    return out.sum(axis=0, keepdims=True) if share_heads else out


# --------------------------------------------------------------------------------------
# selection and compaction (Sec. 3.4, Fig. 5(b))
# --------------------------------------------------------------------------------------
def select_topk(s: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries, equal scores going to the lower index,
    returned in ascending index order."""
    s = np.asarray(s)
    order = np.lexsort((np.arange(s.size), -s))      # by -score, then by index
    return np.sort(order[:k]).astype(np.int64)


def packed_segments(segments, budgets):
    """Segment table after compaction: same order, anchors and the current frame at
    full length, a past frame at min(len, budget)."""
    out, at = [], 0
    for (start, length, kind, frame), b in zip(segments, budgets):
        n = min(length, b) if kind == SEG_FRAME else length
        out.append((at, n, kind, frame))
        at += n
    return out


def masked_budgets(segments, budgets, valid):
    """Budgets under a cache mask (Sec. 3.1, the binary cache mask; Sec. 3.4: masked
    positions are removed, not stored): a past frame can keep at most its unmasked tokens."""
    valid = np.asarray(valid, dtype=bool)
    return [min(b, int(valid[start:start + length].sum())) if kind == SEG_FRAME else b
            for (start, length, kind, _), b in zip(segments, budgets)]


def compact(K, V, pos, sc, segments, budgets, share_heads: bool = False, valid=None):
    """Keep, per selection head and per past-frame segment, the top-budget keys by
    score; remove everything else; keep chronological order and carry each kept row's
    (t, h, w) unchanged.  K, V: [Hkv][Nk][D]; pos: [Hsel][Nk][3]; sc: [Hsel][Nk].
    Hsel = 1 when share_heads (every KV head keeps the same rows) else Hkv.
    valid ([Nk] bool, the cache mask, one flag per token for all heads): masked tokens of
    a past frame are never candidates, whatever their score and the budget.
    Returns K', V' [Hkv][Nk'][D], pos' [Hsel][Nk'][3], idx [Hsel][Nk'], segments'."""
    K, V = np.asarray(K), np.asarray(V)
    pos, sc = np.asarray(pos), np.asarray(sc)
    hkv = K.shape[0]
    hsel = 1 if share_heads else hkv
    assert pos.shape[0] == hsel and sc.shape[0] == hsel
    if valid is not None:
        valid = np.asarray(valid, dtype=bool)
        budgets = masked_budgets(segments, budgets, valid)
    idx = []
    for h in range(hsel):
        rows = []
        for (start, length, kind, _), b in zip(segments, budgets):
            if kind == SEG_FRAME and valid is not None:
                cand = np.flatnonzero(valid[start:start + length])          # unmasked tokens only
                rows.append(start + cand[select_topk(sc[h, start + cand], min(cand.size, b))])
            elif kind == SEG_FRAME:
                rows.append(start + select_topk(sc[h, start:start + length], min(length, b)))
            else:
                rows.append(np.arange(start, start + length, dtype=np.int64))
        idx.append(np.concatenate(rows) if rows else np.zeros(0, np.int64))
    idx = np.stack(idx)
    Kp = np.stack([K[g][idx[0 if share_heads else g]] for g in range(hkv)])
    Vp = np.stack([V[g][idx[0 if share_heads else g]] for g in range(hkv)])
    pp = np.stack([pos[h][idx[h]] for h in range(hsel)])
    return Kp, Vp, pp, idx, packed_segments(segments, budgets)


# --------------------------------------------------------------------------------------
# rolling rollout (Sec. 3.4: every retained frame is re-packed at every step under the same
# allocation rule, so eviction is irreversible: the candidates of a frame at step f are
# its survivors of step f - 1)
# --------------------------------------------------------------------------------------
def rolling_rollout(anchor_K, anchor_V, anchor_pos, anchor_segments, frames, queries, scale: float,
                    budget_fn, score_rows=None, share_heads: bool = False, rotate=None, query_pos=None,
                    rebase_t_scale=None, storage=None, include_self: bool = False):
    """Generate-time cache management over several frame steps.

    anchor_K, anchor_V [Hkv][A][D], anchor_pos [A][3], anchor_segments: the always-kept
    text / conditioning-image rows.
    frames[j] = (K_j, V_j, pos_j): keys, values and (t, h, w) of generated frame j + 1,
    appended whole to the cache before the step that generates frame j + 2.
    queries[i]: queries [Hq][Nq][D] of step i + 1, which sees frames 1..i.
    budget_fn(n_past) -> per-distance budgets, entry d - 1 for distance d.
    rotate = None: keys and queries come already rotated.  rotate = (sections, base): they
    come un-rotated and are rotated here, keys once on insertion, queries (at
    query_pos[i]) at their step.
    rebase_t_scale (needs rotate): sliding window.  The window advances when a step begins:
    oldest frames that the previous step evicted completely leave the segment table and
    every retained frame row is rebased by delta_t = rebase_t_scale * (frames dropped);
    the frame appended now, the step's queries and everything that arrives later are
    placed at their position minus the total shift so far, so scoring and attention of a
    step see one consistent set of coordinates.  The anchors keep theirs.
    storage: rounding applied to keys whenever they are written to the cache (the cache's
    storage format), and to rotated queries; None keeps fp64.
    include_self: the frame being generated attends to its own keys too (attention inside a
    frame is bidirectional, Eq. 2 / Sec. 3.1).  frames[i] is then appended when step i + 1
    begins, as an always-kept SELF segment that takes part in the softmax of scoring and
    attention but is never pruned; when the next step begins it turns into the newest past
    frame (distance 1) and is pruned from then on.
    Each step: slide the window, append the newest frame, score all cached keys with the
    scoring rows of the step's queries, keep the per-frame top-budget keys (anchors whole),
    attend over what is left.  Returns one dict per step: K, V, pos, segments (the cache
    the step attended over), O, lse and the total temporal shift so far."""
    store = (lambda a: a) if storage is None else storage
    hkv = np.asarray(anchor_K).shape[0]
    hsel = 1 if share_heads else hkv
    anchor_pos = np.asarray(anchor_pos)
    K = f64(anchor_K) if rotate is None else store(rope3d(anchor_K, anchor_pos, *rotate))
    V = f64(anchor_V)
    pos = np.broadcast_to(anchor_pos[None], (hsel,) + anchor_pos.shape).copy()
    segments = list(anchor_segments)
    shift = 0
    steps = []
    for i, Q in enumerate(queries):
        if rebase_t_scale is not None:
            first = next((j for j, s in enumerate(segments) if s[2] == SEG_FRAME), len(segments))
            n_drop = 0
            while first + n_drop < len(segments) and segments[first + n_drop][1] == 0:
                n_drop += 1
            if n_drop and first + n_drop < len(segments):
                delta = int(rebase_t_scale) * n_drop
                segments = segments[:first] + segments[first + n_drop:]
                a = segments[first][0]
                Kr, pr = rebase(K[:, a:], pos[:, a:], delta, *rotate)
                K = np.concatenate([K[:, :a], store(Kr)], axis=1)
                pos = np.concatenate([pos[:, :a], pr], axis=1)
                shift += delta
        if include_self:   # last step's own frame is a past frame from now on
            segments = [(a, n, SEG_FRAME if kind == SEG_SELF else kind, f) for (a, n, kind, f) in segments]
        if i >= 1 or include_self:
            Kf, Vf, pf = frames[i if include_self else i - 1]
            pf = np.asarray(pf).copy()
            pf[:, 0] -= shift
            Kf = f64(Kf) if rotate is None else store(rope3d(Kf, pf, *rotate))
            at = K.shape[1]
            K = np.concatenate([K, Kf], axis=1)
            V = np.concatenate([V, f64(Vf)], axis=1)
            pos = np.concatenate([pos, np.broadcast_to(pf[None], (hsel,) + pf.shape)], axis=1)
            segments.append((at, Kf.shape[1], SEG_SELF if include_self else SEG_FRAME, i + 1 if include_self else i))
        if rotate is None:
            Q = f64(Q)
        else:
            qp = np.asarray(query_pos[i]).copy()
            qp[:, 0] -= shift
            Q = store(rope3d(Q, qp, *rotate))
        n_past = sum(1 for s in segments if s[2] == SEG_FRAME)
        per_distance = budget_fn(n_past)
        # the newest past frame is the LAST frame segment: distance 1
        budgets, d = [], n_past
        for (_, length, kind, _) in segments:
            if kind == SEG_FRAME:
                budgets.append(per_distance[d - 1])
                d -= 1
            else:
                budgets.append(length)
        sc = score(Q if score_rows is None else Q[:, score_rows], K, scale, share_heads=share_heads)
        K, V, pos, _, segments = compact(K, V, pos, sc, segments, budgets, share_heads=share_heads)
        O, lse = frame_attn(Q, K, V, scale)
        steps.append({"K": K, "V": V, "pos": pos, "segments": list(segments), "O": O, "lse": lse, "shift": shift})
    return steps


# --------------------------------------------------------------------------------------
# brute force (pure Python loops; tiny inputs only)
# --------------------------------------------------------------------------------------
def frame_attn_bruteforce(Q, K, V, scale: float):
    from math import exp
    Q, K, V = f64(Q), f64(K), f64(V)
    hq, nq, d = Q.shape
    rep = hq // K.shape[0]
    nk = K.shape[1]
    O = np.zeros((hq, nq, d))
    for h in range(hq):
        g = h // rep
        for i in range(nq):
            s = [sum(Q[h, i, c] * K[g, j, c] for c in range(d)) * scale for j in range(nk)]
            m = max(s)
            e = [exp(v - m) for v in s]
            z = sum(e)
            for c in range(d):
                O[h, i, c] = sum(e[j] * V[g, j, c] for j in range(nk)) / z
    return O


def score_bruteforce(Qs, K, scale: float) -> np.ndarray:
    from math import exp
    Qs, K = f64(Qs), f64(K)
    hq, nq, d = Qs.shape
    hkv, nk, _ = K.shape
    rep = hq // hkv
    out = np.zeros((hkv, nk))
    for h in range(hq):
        g = h // rep
        for i in range(nq):
            s = [sum(Qs[h, i, c] * K[g, j, c] for c in range(d)) * scale for j in range(nk)]
            m = max(s)
            e = [exp(v - m) for v in s]
            z = sum(e)
            for j in range(nk):
                out[g, j] += e[j] / z
    return out
