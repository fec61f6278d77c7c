"""Seeded synthetic inputs shaped like the paper's workloads.

Serves both the HIP path and the CPU oracle and therefore holds none of the method's
arithmetic: only random draws, the storage rounding of the inputs, segment tables and
token coordinates.  Shapes follow Sec. 4.1 of the paper (a 48x84 latent token grid per
frame at 384x672, a few hundred prompt tokens, a conditioning image of one frame) and
the attention structure follows Sec. 3.2 (anchors attract attention, attention to past
frames decays with temporal distance).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

SEG_TEXT, SEG_COND, SEG_FRAME, SEG_SELF = 0, 1, 2, 3


def to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), kept as float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are exactly representable in bfloat16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value is not a bfloat16"
    return (u >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def segment_table(n_text: int, n_frame: int, n_past: int) -> list[tuple[int, int, int, int]]:
    """[text | conditioning image | oldest past frame ... newest past frame]."""
    segs = [(0, n_text, SEG_TEXT, -1), (n_text, n_frame, SEG_COND, 0)]
    at = n_text + n_frame
    for f in range(1, n_past + 1):
        segs.append((at, n_frame, SEG_FRAME, f))
        at += n_frame
    return segs


def grid_positions(frame: int, gh: int, gw: int, t0: int) -> np.ndarray:
    """(t, h, w) of a frame's tokens in raster order, latent coordinates scaled by
    (4, 8, 8) as in Sec. 3.1."""
    r, c = np.meshgrid(np.arange(gh), np.arange(gw), indexing="ij")
    t = np.full(gh * gw, t0 + 4 * frame)
    return np.stack([t, 8 * r.ravel(), 8 * c.ravel()], axis=1).astype(np.int32)


def cache_positions(n_text: int, gh: int, gw: int, n_past: int) -> np.ndarray:
    """Text token i sits at (i, i, i); visual frames follow, conditioning image = frame 0."""
    i = np.arange(n_text, dtype=np.int32)
    rows = [np.stack([i, i, i], axis=1)]
    for f in range(0, n_past + 1):
        rows.append(grid_positions(f, gh, gw, n_text))
    return np.concatenate(rows).astype(np.int32)


def low_frequency_dims(sections: tuple[int, int, int], pairs: int = 4) -> np.ndarray:
    """The last `pairs` rotary pairs of every section: the slowest-turning dims, on which
    a direction shared by queries and keys survives the rotation."""
    dims, off = [], 0
    for s in sections:
        for i in range(s // 2 - pairs, s // 2):
            dims += [off + 2 * i, off + 2 * i + 1]
        off += s
    return np.asarray(dims)


@dataclass
class Workload:
    name: str
    dtype: str                      # "f32" | "bf16"
    Hq: int
    Hkv: int
    D: int
    n_text: int
    gh: int
    gw: int
    n_past: int
    gamma: float
    b_min: int
    Q: np.ndarray                   # [Hq][Nq][D] float32 (bf16-representable when dtype == bf16)
    K: np.ndarray                   # [Hkv][Nk][D]
    V: np.ndarray                   # [Hkv][Nk][D]
    pos_k: np.ndarray               # [Nk][3] int32
    pos_q: np.ndarray               # [Nq][3] int32
    segments: list = field(default_factory=list)
    sections: tuple | None = None   # rotary split of D over (t, h, w); None: no RoPE
    base: float = 10000.0
    score_rows: np.ndarray | None = None   # query rows that score (same for every head)

    @property
    def n_frame(self) -> int:
        return self.gh * self.gw

    @property
    def Nk(self) -> int:
        return self.K.shape[1]

    @property
    def Nq(self) -> int:
        return self.Q.shape[1]

    @property
    def scale(self) -> float:
        return float(self.D) ** -0.5


def strided_rows(nq: int, n_sample: int) -> np.ndarray:
    """Scoring subset: n_sample query rows spread evenly over the frame."""
    n = min(nq, n_sample)
    return (np.arange(n, dtype=np.int64) * nq) // n


def config1(seed: int = 0) -> Workload:
    """Tiny fp32 case: 2 query heads, 1 KV head, D = 64; 16 text + 8x8 conditioning
    image + 4 past frames of 8x8; anchor keys pulled toward the query mean."""
    rng = np.random.default_rng(seed)
    hq, hkv, d, n_text, gh, gw, n_past = 2, 1, 64, 16, 8, 8, 4
    n = gh * gw
    nk = n_text + n * (1 + n_past)
    Q = rng.standard_normal((hq, n, d)).astype(np.float32)
    K = rng.standard_normal((hkv, nk, d)).astype(np.float32)
    V = rng.standard_normal((hkv, nk, d)).astype(np.float32)
    qmean = Q.reshape(-1, d).mean(axis=0)
    K[:, : n_text + n, :] += np.float32(0.5) * qmean[None, None, :]
    return Workload("c1", "f32", hq, hkv, d, n_text, gh, gw, n_past, 0.7, 8, Q, K, V,
                    cache_positions(n_text, gh, gw, n_past), grid_positions(n_past + 1, gh, gw, n_text),
                    segment_table(n_text, n, n_past), None, 10000.0, np.arange(n))


def frame_layer(name: str, seed: int, hq: int, hkv: int, d: int, n_text: int, gh: int, gw: int,
                n_past: int, gamma: float, b_min: int, sections: tuple[int, int, int],
                n_score: int = 512, dtype: str = "bf16") -> Workload:
    """One attention layer at frame n_past + 1 in the style of the frame-24 / frame-48
    configurations: V ~ N(0,1); K ~ N(0,1) plus, for the past frame at distance dist,
    0.3 * 0.9^dist along a unit direction u of its KV group (0.5 for the anchors);
    Q ~ N(0,1) plus sqrt(D) * u, so that u is the query mean direction and the mean logit
    of a segment is shifted by exactly its bias magnitude.  u lives on the slowest rotary
    pairs, so the structure survives 3D RoPE whichever side of it the data is read."""
    rng = np.random.default_rng(seed)
    n = gh * gw
    nk = n_text + n * (1 + n_past)
    rep = hq // hkv
    lf = low_frequency_dims(sections)
    u = np.zeros((hkv, d), np.float32)
    u[:, lf] = rng.standard_normal((hkv, lf.size)).astype(np.float32)
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    K = rng.standard_normal((hkv, nk, d), dtype=np.float32)
    V = rng.standard_normal((hkv, nk, d), dtype=np.float32)
    Q = rng.standard_normal((hq, n, d), dtype=np.float32)
    K[:, : n_text + n, :] += np.float32(0.5) * u[:, None, :]
    for f in range(1, n_past + 1):
        dist = n_past + 1 - f
        a = n_text + n * f
        K[:, a:a + n, :] += np.float32(0.3 * 0.9 ** dist) * u[:, None, :]
    for h in range(hq):
        Q[h] += np.float32(np.sqrt(d)) * u[h // rep][None, :]
    if dtype == "bf16":
        Q, K, V = to_bf16(Q), to_bf16(K), to_bf16(V)
    return Workload(name, dtype, hq, hkv, d, n_text, gh, gw, n_past, gamma, b_min, Q, K, V,
                    cache_positions(n_text, gh, gw, n_past), grid_positions(n_past + 1, gh, gw, n_text),
                    segment_table(n_text, n, n_past), sections, 10000.0, strided_rows(n, n_score))


def config2(seed: int = 1000, n_past: int = 23, hq: int = 16, hkv: int = 4) -> Workload:
    """Single layer at frame 24 (n_past = 23) or frame 48 (n_past = 47): 48x84 tokens per
    frame, 256 text tokens, D = 128 split 32/48/48, gamma 0.85, minimum quota 512."""
    return frame_layer(f"frame{n_past + 1}", seed, hq, hkv, 128, 256, 48, 84, n_past, 0.85, 512,
                       (32, 48, 48))


def midsize(seed: int = 7, dtype: str = "bf16", n_past: int = 6, hq: int = 8, hkv: int = 2,
            gh: int = 12, gw: int = 21, n_text: int = 40, b_min: int = 32,
            gamma: float = 0.85) -> Workload:
    """A scaled-down frame layer the oracle finishes in seconds; sizes are deliberately
    ragged (252 tokens per frame, 40 text tokens) so tiles have tails."""
    return frame_layer("mid", seed, hq, hkv, 128, n_text, gh, gw, n_past, gamma, b_min, (32, 48, 48),
                       n_score=100, dtype=dtype)


# --------------------------------------------------------------------------------------
# rolling rollout: one layer's stream of frames
# --------------------------------------------------------------------------------------
@dataclass
class RollingCase:
    """Inputs of a multi-step rollout of one layer.  Keys and queries are UN-rotated;
    frames[j] belongs to generated frame j + 1, queries[i] to the step that generates
    frame i + 1 and sees frames 1..i."""
    dtype: str
    Hq: int
    Hkv: int
    D: int
    n_text: int
    gh: int
    gw: int
    sections: tuple
    base: float
    anchor_K: np.ndarray
    anchor_V: np.ndarray
    anchor_pos: np.ndarray
    anchor_segments: list
    frames: list            # (K [Hkv][n][D], V, pos [n][3])
    queries: list           # Q [Hq][n][D]
    query_pos: list         # [n][3] per step
    score_rows: np.ndarray

    @property
    def n_frame(self) -> int:
        return self.gh * self.gw

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.D))


def rolling_directions(rng, hkv: int, d: int, n_dir: int, sections) -> np.ndarray:
    """[Hkv][n_dir][D] unit vectors on the slowest rotary pairs (direction 0: anchors,
    direction j: generated frame j)."""
    lf = low_frequency_dims(sections)
    u = np.zeros((hkv, n_dir, d), np.float32)
    u[:, :, lf] = rng.standard_normal((hkv, n_dir, lf.size)).astype(np.float32)
    u /= np.linalg.norm(u, axis=2, keepdims=True)
    return u


def query_direction(u: np.ndarray, step: int) -> np.ndarray:
    """Mean direction of the queries of `step` (1-based): anchors at full weight, frame j
    at 0.9^(step - j), so that the mean logit of a cached frame decays with its age."""
    w = u[:, 0].copy()
    for j in range(1, step):
        w += np.float32(0.9 ** (step - j)) * u[:, j]
    return w


def rolling_case(seed: int = 11, n_steps: int = 6, hq: int = 8, hkv: int = 2, d: int = 128, n_text: int = 40,
                 gh: int = 12, gw: int = 21, sections=(32, 48, 48), n_score: int = 100,
                 dtype: str = "bf16") -> RollingCase:
    """A rollout of n_steps frame steps: V ~ N(0,1); K ~ N(0,1) + 0.5 u_0 for the anchors
    and + 0.3 u_j for generated frame j; Q of step f ~ N(0,1) + sqrt(D) * (u_0 + sum_j
    0.9^(f-j) u_j).  The directions u live on the slowest rotary pairs, so the structure
    survives the rotation; they are random, not orthogonal, so frames leak a little into
    each other's mean logit."""
    rng = np.random.default_rng(seed)
    n = gh * gw
    rep = hq // hkv
    u = rolling_directions(rng, hkv, d, n_steps + 1, sections)
    rnd = to_bf16 if dtype == "bf16" else (lambda a: a)
    n_anchor = n_text + n
    aK = rng.standard_normal((hkv, n_anchor, d), dtype=np.float32) + np.float32(0.5) * u[:, 0][:, None, :]
    aV = rng.standard_normal((hkv, n_anchor, d), dtype=np.float32)
    frames, queries, qpos = [], [], []
    for step in range(1, n_steps + 1):
        Q = rng.standard_normal((hq, n, d), dtype=np.float32)
        w = query_direction(u, step)
        for h in range(hq):
            Q[h] += np.float32(np.sqrt(d)) * w[h // rep][None, :]
        queries.append(rnd(Q))
        qpos.append(grid_positions(step, gh, gw, n_text))
        Kf = rng.standard_normal((hkv, n, d), dtype=np.float32) + np.float32(0.3) * u[:, step][:, None, :]
        Vf = rng.standard_normal((hkv, n, d), dtype=np.float32)
        frames.append((rnd(Kf), rnd(Vf), grid_positions(step, gh, gw, n_text)))
    return RollingCase(dtype, hq, hkv, d, n_text, gh, gw, tuple(sections), 10000.0, rnd(aK), rnd(aV),
                       cache_positions(n_text, gh, gw, 0), segment_table(n_text, n, 0), frames, queries, qpos,
                       strided_rows(n, n_score))


class DeviceRollingStream:
    """The rolling_case recipe drawn on the GPU (torch generator, seeded per layer) for
    rollouts too large to draw on the host: fills caller-provided bf16 buffers in place."""

    def __init__(self, seed: int, hq: int, hkv: int, d: int, n_frames: int, sections=(32, 48, 48),
                 device: str = "cuda:0"):
        import torch
        self.torch = torch
        self.hq, self.hkv, self.d = hq, hkv, d
        u = rolling_directions(np.random.default_rng(seed), hkv, d, n_frames + 1, sections)
        self.u = torch.from_numpy(u).to(device)                                  # [Hkv][n_frames+1][D]
        self.w = [torch.from_numpy(query_direction(u, step)).to(device) for step in range(1, n_frames + 1)]
        self.gen = torch.Generator(device=device)
        self.gen.manual_seed(seed)

    def _fill(self, out, shift):
        out.normal_(generator=self.gen)
        if shift is not None:
            out.add_(shift[:, None, :].to(out.dtype))

    def anchors(self, out_k, out_v):
        self._fill(out_k, 0.5 * self.u[:, 0])
        self._fill(out_v, None)

    def frame(self, j: int, out_k, out_v):
        """Keys / values of generated frame j (1-based)."""
        self._fill(out_k, 0.3 * self.u[:, j])
        self._fill(out_v, None)

    def queries(self, step: int, out_q):
        """Queries of the step that generates frame `step` (1-based)."""
        rep = self.hq // self.hkv
        self._fill(out_q, float(np.sqrt(self.d)) * self.w[step - 1].repeat_interleave(rep, dim=0))


def device_frame_layer(seed: int, n_past: int, K_out, V_out, Q_out, n_text: int = 256, gh: int = 48, gw: int = 84,
                       sections=(32, 48, 48)) -> None:
    """The frame_layer recipe drawn on the GPU (seeded torch generator) into caller-provided
    bf16 buffers: K_out, V_out [Hkv][Nk][D], Q_out [Hq][n][D] or None.  For stacks of layers too
    large to draw on the host: every layer gets its own seed, hence its own keys, scores and
    selected rows."""
    import torch
    hkv, nk, d = K_out.shape
    n = gh * gw
    assert nk == n_text + n * (1 + n_past)
    dev = K_out.device
    lf = low_frequency_dims(tuple(sections))
    rng = np.random.default_rng(seed)
    u = np.zeros((hkv, d), np.float32)
    u[:, lf] = rng.standard_normal((hkv, lf.size)).astype(np.float32)
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    ud = torch.from_numpy(u).to(dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    K_out.normal_(generator=gen)
    V_out.normal_(generator=gen)
    bias = torch.empty((hkv, nk, 1), dtype=torch.float32, device=dev)
    bias[:, : n_text + n] = 0.5
    for f in range(1, n_past + 1):
        a = n_text + n * f
        bias[:, a:a + n] = 0.3 * 0.9 ** (n_past + 1 - f)
    K_out.add_((bias * ud[:, None, :]).to(K_out.dtype))
    if Q_out is not None:
        rep = Q_out.shape[0] // hkv
        Q_out.normal_(generator=gen)
        Q_out.add_((float(np.sqrt(d)) * ud.repeat_interleave(rep, dim=0))[:, None, :].to(Q_out.dtype))
