"""Rolling PackCache for one attention layer: the cache stays packed across frame steps.

Host-side bookkeeping only (buffers, the segment table, which C-ABI call comes next); every
step of the path runs in libpackcache kernels.  Per frame step (Sec. 3.4, Fig. 5(b)):

    reserve()/commit()  the frame generated last is appended whole (keys rotated on insert)
    pc_score            importance of every cached key under the step's queries
    pc_budget           per-distance token budgets (config rule or the paper's Eq. 6 / Eq. 7)
    pc_compact          in place: anchors stay, each past frame keeps its top-budget keys
    pc_frame_attn       the step's queries over the packed cache

The frame being generated may sit in the cache too (attention inside a frame is
bidirectional, Eq. 2): commit it with kind PC_SEG_SELF before step(); it takes part in the
softmax of scoring and attention, is never pruned at its own step, and promote_self() turns
it into the newest past frame when the next step begins, without moving a row.

A model that makes several attention passes per frame (iterative decoding) calls attend()
on the un-packed cache first, hands its log-sum-exp to refresh() and makes the remaining
passes on the packed cache: the compaction is paid once per frame.

With slide_t_scale set the window slides (Sec. 3.4, Slide-Cache): when a step begins, the
oldest frames that the step before evicted completely leave the segment table and
pc_rebase lowers the temporal coordinate of every retained frame row by slide_t_scale per
dropped frame; `shift` is the total so far, and the caller places the frame it appends and
its queries at their coordinates minus `shift`.

Eviction is irreversible: a frame's candidates at one step are its survivors of the step
before.  With mode "dense" nothing is evicted (the full-cache baseline); with mode "slide"
only the newest frame survives (the sliding-window baseline of Sec. 3.3).
"""
from __future__ import annotations

from . import binding as pk

MODES = {"pow": pk.PC_BUDGET_POW, "norm": pk.PC_BUDGET_NORM, "half": pk.PC_BUDGET_HALF,
         "slide": pk.PC_BUDGET_SLIDE, "dense": None}


class RollingLayer:
    """The packed K/V cache of one layer in HBM and its host-side segment table."""

    def __init__(self, Hq: int, Hkv: int, D: int, capacity: int, n_frame: int, scale: float,
                 mode: str = "pow", gamma: float = 0.85, b_min: int = 512, budget_tokens: int | None = None,
                 n_score: int = 512, sections=(32, 48, 48), base: float = 10000.0, dtype=None, device="cuda:0",
                 slide_t_scale: int | None = None, share_heads: bool = False, fold_scale: bool = False):
        import torch
        if mode not in MODES:
            raise ValueError(f"mode {mode!r} not in {sorted(MODES)}")
        self.Hq, self.Hkv, self.D, self.capacity, self.n_frame = Hq, Hkv, D, capacity, n_frame
        self.scale, self.mode, self.gamma, self.b_min = scale, mode, gamma, b_min
        # fold_scale: the queries carry scale * log2(e) (step() multiplies it in while rotating; a
        # caller that rotates them itself passes them that way) and the scoring and attention calls
        # get ln 2 as their scale: the same softmax on the kernels' shorter loops
        self.fold_scale = fold_scale
        self.q_out_scale = pk.folded_q_scale(scale) if fold_scale else 1.0
        self.call_scale = pk.PC_SCALE_FOLDED if fold_scale else scale
        # POW floors gamma^d of a whole frame; NORM / HALF / SLIDE split a fixed token budget
        self.budget_tokens = n_frame if budget_tokens is None else budget_tokens
        self.sections, self.base = tuple(sections), base
        dtype = torch.bfloat16 if dtype is None else dtype
        # share_heads: one selection for all KV heads (the paper's per-token cache mask) instead
        # of one per KV head; positions and scores then have a single head
        self.share_heads = share_heads
        hsel = 1 if share_heads else Hkv
        self.K = torch.empty((Hkv, capacity, D), dtype=dtype, device=device)
        self.V = torch.empty_like(self.K)
        self.pos = torch.empty((hsel, capacity, 3), dtype=torch.int32, device=device)
        self.segments: list[tuple[int, int, int, int]] = []
        self.nk = 0
        self.slide_t_scale, self.shift = slide_t_scale, 0
        n_rows = min(n_score, n_frame)
        self.q_rows = ((torch.arange(n_rows, dtype=torch.int64) * n_frame) // n_rows).to(torch.int32).to(device)
        # room for the partial results of up to four key shares (the split depends on the key
        # count of the call; a workspace that is too small only means no split)
        self._ws_attn = torch.empty(4 * Hq * n_frame * (D * 4 + 8) + 1024, dtype=torch.uint8, device=device)
        if mode != "dense":   # the full-cache baseline neither scores nor compacts
            self.score = torch.empty((hsel, capacity), dtype=torch.float32, device=device)
            self._ws_score = torch.empty(pk.pc_score_workspace_bytes(Hq, Hkv, n_rows, capacity, share_heads),
                                         dtype=torch.uint8, device=device)
            self._ws_compact = torch.empty(pk.pc_compact_workspace_bytes(Hkv, capacity, share_heads),
                                           dtype=torch.uint8, device=device)

    # ---- insertion: the producer writes straight into the cache, no copy ----------------------
    def reserve(self, n: int):
        """Views of the next n free rows: (K rows, V rows, pos rows [Hsel][n][3])."""
        if self.nk + n > self.capacity:
            raise ValueError(f"cache capacity {self.capacity} < {self.nk} + {n}")
        a = self.nk
        return self.K[:, a:a + n], self.V[:, a:a + n], self.pos[:, a:a + n]

    def commit(self, n: int, kind: int, frame: int, rotate_with=None, valid=None) -> None:
        """Make the n reserved rows part of the cache.  rotate_with: int32 [n][3] device
        positions; when given the new keys are rotated in place (a1) on insertion.
        valid (host array of n flags, the cache mask of Sec. 3.1 for this frame): only the
        unmasked tokens enter the cache.  The masked rows are removed on insertion by the
        compaction call itself (mask as the score, budget = unmasked count; the rest of the
        cache keeps every row), so no later scoring or attention ever sees them: masked
        entries are ignored in attention (Sec. 3.1), and removed rather than stored (Sec. 3.4)."""
        a = self.nk
        if rotate_with is not None:
            pk.pc_rope3d(self.K[:, a:a + n], rotate_with, self.sections, self.base)
        if valid is not None:
            import numpy as np
            import torch
            if kind != pk.PC_SEG_FRAME:
                raise ValueError("a cache mask applies to a generated frame entering the cache (PC_SEG_FRAME)")
            v = np.ascontiguousarray(np.asarray(valid) != 0, dtype=np.uint8)
            if v.shape != (n,):
                raise ValueError(f"valid must hold {n} flags, got shape {v.shape}")
            n_valid = int(v.sum())
            if n_valid < n:
                if not hasattr(self, "score"):      # the full-cache baseline scores nothing else
                    self.score = torch.empty((self.pos.shape[0], self.capacity), dtype=torch.float32,
                                             device=self.K.device)
                    self._ws_compact = torch.empty(pk.pc_compact_workspace_bytes(self.Hkv, self.capacity,
                                                                                 self.share_heads),
                                                   dtype=torch.uint8, device=self.K.device)
                sc_new = self.score[:, a:a + n]
                sc_new.zero_()
                pk.pc_mask_scores(sc_new, torch.from_numpy(v).to(self.K.device))    # masked -> -1 < 0
                table = self.segments + [(a, n, kind, frame)]
                keep = [s[1] for s in self.segments] + [n_valid]
                self.segments, self.nk = pk.pc_compact(self.K, self.V, self.pos, self.score, table, keep,
                                                       share_heads=self.share_heads, ws=self._ws_compact)
                return
        self.segments.append((a, n, kind, frame))
        self.nk = a + n

    def promote_self(self) -> None:
        """Call when a step begins: the frame that was generated last and sat in the cache as the
        always-kept SELF segment of its own step (commit(..., kind=PC_SEG_SELF)) becomes the newest
        past frame.  A table edit only: its rows are already in place."""
        self.segments = [(a, n, pk.PC_SEG_FRAME if kind == pk.PC_SEG_SELF else kind, f)
                         for (a, n, kind, f) in self.segments]

    def advance_window(self) -> int:
        """Call when a step begins, before reserve(): drops the oldest frame segments that
        are empty and rebases the retained frame rows.  Returns the total shift so far."""
        if self.slide_t_scale is None:
            return self.shift
        first = next((j for j, s in enumerate(self.segments) if s[2] == pk.PC_SEG_FRAME), len(self.segments))
        n_drop = 0
        while first + n_drop < len(self.segments) and self.segments[first + n_drop][1] == 0:
            n_drop += 1
        if n_drop and first + n_drop < len(self.segments):
            delta = self.slide_t_scale * n_drop
            self.segments = self.segments[:first] + self.segments[first + n_drop:]
            a = self.segments[first][0]
            pk.pc_rebase(self.K, self.pos, a, self.nk - a, delta, self.sections, self.base)
            self.shift += delta
        return self.shift

    # ---- one frame step -----------------------------------------------------------------------
    def budgets(self) -> list[int]:
        """Budget of every segment for the cache as it stands (anchors: their length)."""
        n_past = sum(1 for s in self.segments if s[2] == pk.PC_SEG_FRAME)
        if self.mode == "dense":
            return [s[1] for s in self.segments]
        if self.mode == "pow":
            per_d = pk.pc_budget(pk.PC_BUDGET_POW, self.n_frame, n_past, self.gamma, self.b_min)
        else:
            per_d = pk.pc_budget(MODES[self.mode], self.budget_tokens, n_past, self.gamma, self.b_min)
        return pk.segment_budgets(self.segments, per_d)

    def refresh(self, Q, lse=None) -> None:
        """Score every cached key under the (rotated) queries Q and re-pack the cache in
        place.  lse (fp32 [Hq][n_frame]): log-sum-exp of Q's rows over the cache as it
        stands, e.g. from attend(): scoring then needs one QK^T pass instead of two."""
        if self.mode == "dense":
            return
        budgets = self.budgets()
        if all(b >= s[1] for s, b in zip(self.segments, budgets) if s[2] == pk.PC_SEG_FRAME):
            return   # every frame is within its budget: nothing to score, nothing to move
        # only segments that lose rows at this step need scores (anchors never do, a frame that sits at
        # its budget does not either): the scoring covers the span from the first to the last of them
        prunable = [s for s, b in zip(self.segments, budgets) if s[2] == pk.PC_SEG_FRAME and b < s[1]]
        span = (prunable[0][0], prunable[-1][0] + prunable[-1][1])
        pk.pc_score(Q, self.K, self.nk, self.call_scale, lse=lse, score=self.score, share_heads=self.share_heads,
                    ws=self._ws_score, q_rows=self.q_rows, key_range=span)
        self.segments, self.nk = pk.pc_compact(self.K, self.V, self.pos, self.score, self.segments,
                                               budgets, share_heads=self.share_heads, ws=self._ws_compact)

    def attend(self, Q, O=None, lse=None):
        """The (rotated) queries Q over the cache as it stands -> O (and the log-sum-exp)."""
        return pk.pc_frame_attn(Q, self.K, self.V, self.nk, self.call_scale, O=O, lse=lse, ws=self._ws_attn)

    def step(self, Q, O=None, q_pos=None, lse=None):
        """Queries Q [Hq][n_frame][D] of the frame being generated -> O.  q_pos (int32
        [n_frame][3], device): rotate Q in place first (with fold_scale, times scale * log2(e))."""
        if q_pos is not None:
            pk.pc_rope3d(Q, q_pos, self.sections, self.base, out_scale=self.q_out_scale)
        self.refresh(Q)
        return self.attend(Q, O=O, lse=lse)


class RollingStack:
    """The packed caches of a stack of layers in one allocation, re-packed TOGETHER when a frame
    step ends (Sec. 3.4 re-packs the cache at the frame step, not per attention call).

    Per frame step:
        reserve()/commit()   the frame generated last is appended whole to every layer's cache
        per layer:           attend() over the cache as it stands, with the log-sum-exp of the pass;
                             score_layer() turns that log-sum-exp into importances with ONE QK^T pass
        repack()             budgets, then one pc_compact_batch for the whole stack

    All layers share one segment table: budgets depend on the temporal distance only, so every
    layer keeps the same COUNT of rows per frame (each its own rows).  The cache a step attends
    over is the one the previous step packed plus the whole newest frame; the cache repack()
    leaves is the one RollingLayer.step() would have attended over at the same step (same keys
    scored by the same queries under the same budgets).
    """

    def __init__(self, n_layers: int, Hq: int, Hkv: int, D: int, capacity: int, n_frame: int, scale: float,
                 mode: str = "pow", gamma: float = 0.85, b_min: int = 512, budget_tokens: int | None = None,
                 n_score: int = 512, sections=(32, 48, 48), base: float = 10000.0, dtype=None, device="cuda:0",
                 share_heads: bool = False, fold_scale: bool = False):
        import torch
        if mode not in MODES or mode == "dense":
            raise ValueError(f"mode {mode!r} not in {sorted(m for m in MODES if m != 'dense')}")
        self.L, self.Hq, self.Hkv, self.D, self.capacity, self.n_frame = n_layers, Hq, Hkv, D, capacity, n_frame
        self.scale, self.mode, self.gamma, self.b_min = scale, mode, gamma, b_min
        self.fold_scale = fold_scale
        self.q_out_scale = pk.folded_q_scale(scale) if fold_scale else 1.0
        self.call_scale = pk.PC_SCALE_FOLDED if fold_scale else scale
        self.budget_tokens = n_frame if budget_tokens is None else budget_tokens
        self.sections, self.base, self.share_heads = tuple(sections), base, share_heads
        dtype = torch.bfloat16 if dtype is None else dtype
        hsel = 1 if share_heads else Hkv
        self.K = torch.empty((n_layers, Hkv, capacity, D), dtype=dtype, device=device)
        self.V = torch.empty_like(self.K)
        self.pos = torch.empty((n_layers, hsel, capacity, 3), dtype=torch.int32, device=device)
        self.score = torch.empty((n_layers, hsel, capacity), dtype=torch.float32, device=device)
        self.segments: list[tuple[int, int, int, int]] = []
        self.nk = 0
        n_rows = min(n_score, n_frame)
        self.q_rows = ((torch.arange(n_rows, dtype=torch.int64) * n_frame) // n_rows).to(torch.int32).to(device)
        self._ws_attn = torch.empty(4 * Hq * n_frame * (D * 4 + 8) + 1024, dtype=torch.uint8, device=device)
        self._ws_score = torch.empty(pk.pc_score_workspace_bytes(Hq, Hkv, n_rows, capacity, share_heads),
                                     dtype=torch.uint8, device=device)
        self._ws_compact = torch.empty(pk.pc_compact_batch_workspace_bytes(n_layers, Hkv, capacity, share_heads),
                                       dtype=torch.uint8, device=device)

    def reserve(self, n: int):
        """Views of the next n free rows of every layer: K, V [L][Hkv][n][D], pos [L][Hsel][n][3]."""
        if self.nk + n > self.capacity:
            raise ValueError(f"cache capacity {self.capacity} < {self.nk} + {n}")
        a = self.nk
        return self.K[:, :, a:a + n], self.V[:, :, a:a + n], self.pos[:, :, a:a + n]

    def commit(self, n: int, kind: int, frame: int, rotate_with=None) -> None:
        """Make the n reserved rows part of every layer's cache; rotate_with (int32 [n][3], device)
        rotates the new keys of all layers in place with one call (layers x KV heads as heads)."""
        a = self.nk
        if rotate_with is not None:
            pk.pc_rope3d(self.K.view(self.L * self.Hkv, self.capacity, self.D)[:, a:a + n], rotate_with,
                         self.sections, self.base)
        self.segments.append((a, n, kind, frame))
        self.nk = a + n

    def budgets(self) -> list[int]:
        n_past = sum(1 for s in self.segments if s[2] == pk.PC_SEG_FRAME)
        if self.mode == "pow":
            per_d = pk.pc_budget(pk.PC_BUDGET_POW, self.n_frame, n_past, self.gamma, self.b_min)
        else:
            per_d = pk.pc_budget(MODES[self.mode], self.budget_tokens, n_past, self.gamma, self.b_min)
        return pk.segment_budgets(self.segments, per_d)

    def _prunable_span(self, budgets):
        prunable = [s for s, b in zip(self.segments, budgets) if s[2] == pk.PC_SEG_FRAME and b < s[1]]
        return (prunable[0][0], prunable[-1][0] + prunable[-1][1]) if prunable else None

    def attend(self, layer: int, Q, O=None, lse=None):
        """Layer `layer`'s (rotated) queries over its cache as it stands -> O (and the log-sum-exp)."""
        return pk.pc_frame_attn(Q, self.K[layer], self.V[layer], self.nk, self.call_scale, O=O, lse=lse,
                                ws=self._ws_attn)

    def score_layer(self, layer: int, Q, lse=None) -> None:
        """Importance of layer `layer`'s cached keys under Q (lse: the log-sum-exp attend() gave for
        the same queries over the same cache; without it pc_score takes its extra pass)."""
        span = self._prunable_span(self.budgets())
        if span is None:
            return
        pk.pc_score(Q, self.K[layer], self.nk, self.call_scale, lse=lse, score=self.score[layer],
                    share_heads=self.share_heads, ws=self._ws_score, q_rows=self.q_rows, key_range=span)

    def repack(self) -> None:
        """End of the frame step: every layer keeps, per past frame, its top-budget keys; one
        select launch and one gather launch for the whole stack, in place."""
        budgets = self.budgets()
        if self._prunable_span(budgets) is None:
            return
        self.segments, self.nk = pk.pc_compact_batch(self.K, self.V, self.pos, self.score, self.segments, budgets,
                                                     share_heads=self.share_heads, ws=self._ws_compact)
