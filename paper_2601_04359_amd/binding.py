"""ctypes binding of libpackcache.so: same names as the C ABI, argument marshalling only.

PyTorch supplies device memory and the current stream; every step of the path runs in the
library's HIP kernels.  A missing library raises: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Sequence

__all__ = [
    "PC_F32", "PC_BF16", "PC_SEG_TEXT", "PC_SEG_COND", "PC_SEG_FRAME", "PC_SEG_SELF",
    "PC_BUDGET_POW", "PC_BUDGET_NORM", "PC_BUDGET_HALF", "PC_BUDGET_SLIDE", "PC_MAX_SEGMENTS",
    "PackCacheError", "lib", "lib_path", "pc_version", "pc_strerror", "pc_budget", "pc_rope3d", "pc_rebase",
    "pc_score", "pc_score_workspace_bytes", "pc_compact_plan", "pc_compact", "pc_compact_batch", "pc_compact_batch_workspace_bytes", "PC_COMPACT_SELECT", "PC_COMPACT_GATHER", "PC_SCALE_FOLDED", "folded_q_scale", "pc_masked_budgets", "pc_mask_scores", "pc_compact_status",
    "pc_compact_workspace_bytes", "pc_compact_prepared", "pc_compact_static", "pc_compact_static_capacity", "pc_frame_attn", "pc_frame_attn_workspace_bytes",
    "segment_budgets",
]

PC_F32, PC_BF16 = 0, 1
PC_SEG_TEXT, PC_SEG_COND, PC_SEG_FRAME, PC_SEG_SELF = 0, 1, 2, 3
PC_BUDGET_POW, PC_BUDGET_NORM, PC_BUDGET_HALF, PC_BUDGET_SLIDE = 0, 1, 2, 3
PC_COMPACT_SELECT, PC_COMPACT_GATHER = 1, 2
PC_SCALE_FOLDED = 0.6931471805599453      # ln 2: the scale to pass when Q carries folded_q_scale(scale)


def folded_q_scale(scale: float) -> float:
    """scale * log2(e): multiplied into the queries (pc_rope3d's out_scale), it leaves ln 2 as the
    scale of pc_score / pc_frame_attn, which then run their shorter loops."""
    return float(scale) * 1.4426950408889634

PC_MAX_SEGMENTS = 120

_LIB = None


class PackCacheError(RuntimeError):
    def __init__(self, status: int, detail: str):
        super().__init__(f"libpackcache status {status}: {detail}")
        self.status = status


class pc_segment(C.Structure):
    _fields_ = [("start", C.c_int32), ("len", C.c_int32), ("kind", C.c_int32), ("frame", C.c_int32)]


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libpackcache.so")


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built (run __graft_entry__.build())."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise FileNotFoundError(
                f"{path} is missing: build it with `python -m paper_2601_04359_amd.build`; "
                "the HIP library is the only implementation of this package")
        L = C.CDLL(path)
        i32p, f32p, vp, i64, sz = C.POINTER(C.c_int32), C.POINTER(C.c_float), C.c_void_p, C.c_int64, C.c_size_t
        segp = C.POINTER(pc_segment)
        L.pc_strerror.restype = C.c_char_p
        L.pc_strerror.argtypes = [C.c_int]
        L.pc_last_error_detail.restype = C.c_char_p
        L.pc_version.restype = C.c_int
        L.pc_budget.argtypes = [C.c_int, C.c_int, C.c_int, C.c_double, C.c_int, i32p]
        L.pc_rope3d.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int, i64, vp, C.c_int, C.c_int, C.c_int,
                                C.c_double, C.c_double, vp]
        L.pc_rebase.argtypes = [vp, C.c_int, C.c_int, C.c_int, i64, vp, C.c_int, i64, C.c_int, C.c_int, C.c_int,
                                C.c_int, C.c_int, C.c_int, C.c_double, vp]
        L.pc_score_workspace_bytes.restype = sz
        L.pc_score_workspace_bytes.argtypes = [C.c_int] * 5
        L.pc_score.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, i64, i64, vp,
                               C.c_float, vp, i64, vp, i64, C.c_int, C.c_int, C.c_int, vp, sz, vp]
        L.pc_compact_batch_workspace_bytes.restype = sz
        L.pc_compact_batch_workspace_bytes.argtypes = [C.c_int] * 4
        L.pc_compact_batch.argtypes = [C.c_int, vp, vp, vp, C.c_int, C.c_int, C.c_int, i64, i64, i64, i64, vp, i64,
                                       i64, segp, C.c_int, i32p, C.c_int, vp, vp, vp, i64, i64, i64, i64, vp, i64,
                                       i64, segp, i32p, vp, sz, vp]
        L.pc_compact_batch_phase.argtypes = [C.c_int] + list(L.pc_compact_batch.argtypes)
        L.pc_masked_budgets.argtypes = [segp, C.c_int, i32p, vp, i32p]
        L.pc_mask_scores.argtypes = [vp, C.c_int, C.c_int, i64, vp, vp]
        L.pc_compact_status.argtypes = [vp, vp]
        L.pc_compact_plan.argtypes = [segp, C.c_int, i32p, segp, i32p]
        L.pc_compact_workspace_bytes.restype = sz
        L.pc_compact_workspace_bytes.argtypes = [C.c_int] * 3
        L.pc_compact.argtypes = [vp, vp, vp, C.c_int, C.c_int, C.c_int, i64, i64, vp, i64, segp, C.c_int,
                                 i32p, C.c_int, vp, vp, vp, i64, i64, vp, i64, segp, i32p, vp, sz, vp]
        L.pc_compact_static_capacity.restype = sz
        L.pc_compact_static_capacity.argtypes = []
        L.pc_compact_static.argtypes = L.pc_compact.argtypes[:-3] + [vp]
        L.pc_frame_attn_workspace_bytes.restype = sz
        L.pc_frame_attn_workspace_bytes.argtypes = [C.c_int] * 4
        L.pc_frame_attn.argtypes = [vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, i64,
                                    i64, i64, C.c_float, vp, vp, vp, sz, vp]
        _LIB = L
    return _LIB


def _check(status: int) -> None:
    if status != 0:
        raise PackCacheError(status, lib().pc_last_error_detail().decode())


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return PC_F32
    if t.dtype == torch.bfloat16:
        return PC_BF16
    raise PackCacheError(-3, f"unsupported tensor dtype {t.dtype}")


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _rows_dense(t, name: str) -> None:
    if t.stride(-1) != 1 or t.stride(-2) != t.shape[-1]:
        raise PackCacheError(-2, f"{name}: rows must be dense with the last dimension contiguous")


def _check_kv_layout(K, V, pos, out, share_heads: bool, layer_axis: bool = False) -> None:
    """The compaction calls take ONE head (and layer) stride for K and V and one for pos: refuse
    tensors whose strides differ, whose rows are not dense, or whose pos is not [..][Hsel][cap][3]."""
    _rows_dense(K, "K")
    _rows_dense(V, "V")
    lead = 2 if layer_axis else 1
    if V.shape != K.shape or V.stride()[:lead] != K.stride()[:lead]:
        raise PackCacheError(-2, "K and V must have the same shape and the same head / layer strides")
    _rows_dense(pos, "pos")
    hsel = 1 if share_heads else K.shape[lead - 1]
    if pos.shape[-1] != 3 or pos.shape[lead - 1] != hsel:
        raise PackCacheError(-2, f"pos must be int32 [..][{hsel}][cap][3], got {tuple(pos.shape)}")
    if out is not None:
        Ko, Vo, po = out
        _rows_dense(Ko, "K_out")
        _rows_dense(Vo, "V_out")
        _rows_dense(po, "pos_out")
        if Vo.shape != Ko.shape or Vo.stride()[:lead] != Ko.stride()[:lead]:
            raise PackCacheError(-2, "K_out and V_out must have the same shape and the same head / layer strides")
        if po.shape[-1] != 3 or po.shape[lead - 1] != hsel:
            raise PackCacheError(-2, f"pos_out must be int32 [..][{hsel}][cap][3], got {tuple(po.shape)}")


def _workspace(nbytes: int, like):
    import torch
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=like.device)


def _seg_array(segments: Sequence[Sequence[int]]):
    arr = (pc_segment * max(len(segments), 1))()
    for i, s in enumerate(segments):
        arr[i] = pc_segment(*[int(v) for v in s])
    return arr


def pc_version() -> int:
    return lib().pc_version()


def pc_strerror(status: int) -> str:
    return lib().pc_strerror(status).decode()


def pc_budget(mode: int, n_frame_tokens: int, n_past: int, gamma: float = 0.0, b_min: int = 0) -> list[int]:
    out = (C.c_int32 * max(n_past, 1))()
    _check(lib().pc_budget(mode, n_frame_tokens, n_past, float(gamma), b_min, out))
    return [out[i] for i in range(n_past)]


def segment_budgets(segments: Sequence[Sequence[int]], by_distance: Sequence[int]) -> list[int]:
    """Budget per segment from budgets per temporal distance: the newest FRAME segment in
    the table is at distance 1.  Non-FRAME segments get their own length."""
    frames = [i for i, s in enumerate(segments) if s[2] == PC_SEG_FRAME]
    out = [int(s[1]) for s in segments]
    for d, i in enumerate(reversed(frames), start=1):
        out[i] = int(by_distance[d - 1])
    return out


def pc_rope3d(x, pos, sections: Sequence[int], base: float = 10000.0, out_scale: float = 1.0) -> None:
    """x [H][n][D] (bf16/fp32, device) rotated in place by pos int32 [n][3] and multiplied by
    out_scale before the one rounding (folded_q_scale(scale) for queries that go to pc_score /
    pc_frame_attn with scale = PC_SCALE_FOLDED)."""
    H, n, D = x.shape
    _rows_dense(x, "x")
    _check(lib().pc_rope3d(x.data_ptr(), _dtype_code(x), H, n, D, x.stride(0), pos.data_ptr(),
                           int(sections[0]), int(sections[1]), int(sections[2]), float(base), float(out_scale),
                           _stream()))


def pc_rebase(K, pos, row0: int, n_rows: int, delta_t: int, sections: Sequence[int], base: float = 10000.0) -> None:
    """Rows row0 .. row0+n_rows-1 of K [Hkv][cap][D] and pos int32 [Hsel][cap][3]: temporal
    coordinate lowered by delta_t, keys turned accordingly, in place."""
    Hkv, _, D = K.shape
    _rows_dense(K, "K")
    _check(lib().pc_rebase(K.data_ptr(), _dtype_code(K), Hkv, D, K.stride(0), pos.data_ptr(), pos.shape[0],
                           pos.stride(0), int(row0), int(n_rows), int(delta_t), int(sections[0]), int(sections[1]),
                           int(sections[2]), float(base), _stream()))


def pc_score_workspace_bytes(Hq: int, Hkv: int, n_qs: int, Nk: int, share_heads: bool = False) -> int:
    return lib().pc_score_workspace_bytes(Hq, Hkv, n_qs, Nk, int(share_heads))


def pc_score(Qs, K, Nk: int, scale: float, lse=None, score=None, share_heads: bool = False, ws=None,
             q_rows=None, key_range=None):
    """Qs [Hq][rows][D], K [Hkv][>=Nk][D] -> score fp32 [Hsel][Nk].  q_rows (int32, device)
    picks the rows of Qs that score; None: all of them.  lse (fp32 [Hq][rows], optional) is
    indexed like the rows of Qs.  key_range = (begin, end): only these keys get a score (all of
    them still count in the softmax); the rest of `score` is left as it is."""
    import torch
    Hq, n_qs, D = Qs.shape
    if q_rows is not None:
        n_qs = q_rows.numel()
    Hkv = K.shape[0]
    _rows_dense(Qs, "Qs")
    _rows_dense(K, "K")
    hsel = 1 if share_heads else Hkv
    if score is None:
        score = torch.empty((hsel, Nk), dtype=torch.float32, device=K.device)
    if ws is None:
        ws = _workspace(pc_score_workspace_bytes(Hq, Hkv, n_qs, Nk, share_heads), K)
    _check(lib().pc_score(Qs.data_ptr(), K.data_ptr(), _dtype_code(K), Hq, Hkv, n_qs, Nk, D, Qs.stride(0),
                          K.stride(0), _ptr(q_rows), float(scale), _ptr(lse), 0 if lse is None else lse.stride(0),
                          score.data_ptr(), score.stride(0),
                          int(share_heads), 0 if key_range is None else int(key_range[0]),
                          0 if key_range is None else int(key_range[1]), ws.data_ptr(), ws.numel(), _stream()))
    return score


def pc_masked_budgets(segments, budgets, valid_host) -> list[int]:
    """valid_host: host uint8 array (numpy) with one flag per cached row."""
    import numpy as np
    n = len(segments)
    v = np.ascontiguousarray(valid_host, dtype=np.uint8)
    b = (C.c_int32 * max(n, 1))(*[int(x) for x in budgets])
    out = (C.c_int32 * max(n, 1))()
    _check(lib().pc_masked_budgets(_seg_array(segments), n, b, v.ctypes.data, out))
    return list(out[:n])


def pc_mask_scores(score, valid) -> None:
    """score fp32 [Hsel][Nk] (device), valid uint8 [Nk] (device): masked tokens get -1."""
    _check(lib().pc_mask_scores(score.data_ptr(), score.shape[0], score.shape[1], score.stride(0),
                                valid.data_ptr(), _stream()))


def pc_compact_status(ws, stream=None) -> None:
    """Waits for the stream and raises (status PC_ERR_ABORTED) if the last in-place compaction that
    used the workspace tensor `ws` gave up a wait."""
    _check(lib().pc_compact_status(ws.data_ptr(), _stream() if stream is None else stream))


def pc_compact_plan(segments, budgets):
    n = len(segments)
    seg_in, seg_out = _seg_array(segments), _seg_array([])
    seg_out = (pc_segment * max(n, 1))()
    b = (C.c_int32 * max(n, 1))(*[int(v) for v in budgets])
    nk = C.c_int32(0)
    _check(lib().pc_compact_plan(seg_in, n, b, seg_out, C.byref(nk)))
    return [(s.start, s.len, s.kind, s.frame) for s in seg_out[:n]], nk.value


def pc_compact_workspace_bytes(Hkv: int, Nk_in: int, share_heads: bool = False) -> int:
    return lib().pc_compact_workspace_bytes(Hkv, Nk_in, int(share_heads))


def pc_compact(K, V, pos, score, segments, budgets, share_heads: bool = False, out=None, idx=None, ws=None):
    """Select and compact.  out = None compacts in place; out = (K_out, V_out, pos_out)
    writes there.  Returns (segments_out, Nk_out)."""
    Hkv, _, D = K.shape
    _check_kv_layout(K, V, pos, out, share_heads)
    n = len(segments)
    nk_in = segments[-1][0] + segments[-1][1] if n else 0
    seg_in = _seg_array(segments)
    seg_out = (pc_segment * max(n, 1))()
    b = (C.c_int32 * max(n, 1))(*[int(v) for v in budgets])
    nk = C.c_int32(0)
    Ko, Vo, po = (K, V, pos) if out is None else out
    if ws is None:
        ws = _workspace(pc_compact_workspace_bytes(Hkv, nk_in, share_heads), K)
    _check(lib().pc_compact(K.data_ptr(), V.data_ptr(), pos.data_ptr(), _dtype_code(K), Hkv, D, K.stride(0),
                            pos.stride(0), score.data_ptr(), score.stride(0), seg_in, n, b, int(share_heads),
                            Ko.data_ptr(), Vo.data_ptr(), po.data_ptr(), Ko.stride(0), po.stride(0),
                            _ptr(idx), 0 if idx is None else idx.stride(0), seg_out, C.byref(nk),
                            ws.data_ptr(), ws.numel(), _stream()))
    return [(s.start, s.len, s.kind, s.frame) for s in seg_out[:n]], nk.value


def pc_compact_static_capacity() -> int:
    return lib().pc_compact_static_capacity()


def pc_compact_static(K, V, pos, score, segments, budgets, share_heads: bool = False, out=None, idx=None):
    """pc_compact without a workspace argument: the scratch is an array inside the library (at
    most pc_compact_static_capacity() bytes; larger requests raise).  Nothing is allocated, here
    or in the library.  Calls that overlap on one GPU race on that array."""
    Hkv, _, D = K.shape
    _check_kv_layout(K, V, pos, out, share_heads)
    n = len(segments)
    seg_in = _seg_array(segments)
    seg_out = (pc_segment * max(n, 1))()
    b = (C.c_int32 * max(n, 1))(*[int(v) for v in budgets])
    nk = C.c_int32(0)
    Ko, Vo, po = (K, V, pos) if out is None else out
    _check(lib().pc_compact_static(K.data_ptr(), V.data_ptr(), pos.data_ptr(), _dtype_code(K), Hkv, D, K.stride(0),
                                   pos.stride(0), score.data_ptr(), score.stride(0), seg_in, n, b, int(share_heads),
                                   Ko.data_ptr(), Vo.data_ptr(), po.data_ptr(), Ko.stride(0), po.stride(0),
                                   _ptr(idx), 0 if idx is None else idx.stride(0), seg_out, C.byref(nk), _stream()))
    return [(s.start, s.len, s.kind, s.frame) for s in seg_out[:n]], nk.value


def pc_compact_batch_workspace_bytes(n_layers: int, Hkv: int, Nk_in: int, share_heads: bool = False) -> int:
    return lib().pc_compact_batch_workspace_bytes(n_layers, Hkv, Nk_in, int(share_heads))


def pc_compact_batch(K, V, pos, score, segments, budgets, share_heads: bool = False, out=None, idx=None, ws=None,
                     phases: int = 3, stream=None):
    """pc_compact over a stack of layers in one call: K, V [L][Hkv][cap][D], pos int32
    [L][Hsel][cap][3], score fp32 [L][Hsel][>=Nk]; out / idx as in pc_compact with a leading
    layer axis.  phases: PC_COMPACT_SELECT, PC_COMPACT_GATHER or both (the two halves of
    pc_compact_batch_phase, for callers that overlap them on two streams; pass the same ws to
    both); stream: a torch stream (default: the current one).  Returns (segments_out, Nk_out)."""
    L, Hkv, _, D = K.shape
    _check_kv_layout(K, V, pos, out, share_heads, layer_axis=True)
    if ws is None and (int(phases) != 3 or stream is not None):
        # a workspace made here would be a fresh, uninitialised one per call (the GATHER half needs
        # the one its SELECT half filled) and would go back to the allocator of the CURRENT stream
        # while another stream's kernels may still be using it
        raise PackCacheError(-6, "pc_compact_batch: pass ws when phases != 3 or a stream is given")
    n = len(segments)
    nk_in = segments[-1][0] + segments[-1][1] if n else 0
    seg_out = (pc_segment * max(n, 1))()
    b = (C.c_int32 * max(n, 1))(*[int(v) for v in budgets])
    nk = C.c_int32(0)
    Ko, Vo, po = (K, V, pos) if out is None else out
    if ws is None:
        ws = _workspace(pc_compact_batch_workspace_bytes(L, Hkv, nk_in, share_heads), K)
    _check(lib().pc_compact_batch_phase(int(phases), L, K.data_ptr(), V.data_ptr(), pos.data_ptr(), _dtype_code(K),
                                        Hkv, D, K.stride(1), K.stride(0), pos.stride(1), pos.stride(0),
                                        score.data_ptr(), score.stride(1), score.stride(0), _seg_array(segments), n, b,
                                        int(share_heads), Ko.data_ptr(), Vo.data_ptr(), po.data_ptr(), Ko.stride(1),
                                        Ko.stride(0), po.stride(1), po.stride(0), _ptr(idx),
                                        0 if idx is None else idx.stride(1), 0 if idx is None else idx.stride(0),
                                        seg_out, C.byref(nk), ws.data_ptr(), ws.numel(),
                                        _stream() if stream is None else stream.cuda_stream))
    return [(s.start, s.len, s.kind, s.frame) for s in seg_out[:n]], nk.value


def pc_compact_prepared(K, V, pos, score, segments, budgets, ws, share_heads: bool = False, out=None, idx=None,
                        phases: int = 3, stream=None):
    """Marshal the arguments of pc_compact once; returns a callable that only makes the C
    call (for launch loops where Python-side marshalling would dominate).  phases: 1 = the
    select half, 2 = the gather half, 3 = both; stream: a torch stream (default: the
    current one at preparation time)."""
    Hkv, _, D = K.shape
    _check_kv_layout(K, V, pos, out, share_heads)
    n = len(segments)
    seg_in = _seg_array(segments)
    b = (C.c_int32 * max(n, 1))(*[int(v) for v in budgets])
    Ko, Vo, po = (K, V, pos) if out is None else out
    fn = lib().pc_compact_batch_phase
    args = (int(phases), 1, K.data_ptr(), V.data_ptr(), pos.data_ptr(), _dtype_code(K), Hkv, D, K.stride(0), 0,
            pos.stride(0), 0, score.data_ptr(), score.stride(0), 0, seg_in, n, b, int(share_heads), Ko.data_ptr(),
            Vo.data_ptr(), po.data_ptr(), Ko.stride(0), 0, po.stride(0), 0, _ptr(idx),
            0 if idx is None else idx.stride(0), 0, None, None, ws.data_ptr(), ws.numel(),
            _stream() if stream is None else stream.cuda_stream)

    def call():
        _check(fn(*args))
    return call


def pc_frame_attn_workspace_bytes(Hq: int, Nq: int, Nk: int, D: int) -> int:
    return lib().pc_frame_attn_workspace_bytes(Hq, Nq, Nk, D)


def pc_frame_attn(Q, K, V, Nk: int, scale: float, O=None, lse=None, ws=None):
    """Q [Hq][Nq][D], K/V [Hkv][>=Nk][D] -> O [Hq][Nq][D] (same dtype)."""
    import torch
    Hq, Nq, D = Q.shape
    Hkv = K.shape[0]
    for t, nm in ((Q, "Q"), (K, "K"), (V, "V")):
        _rows_dense(t, nm)
    if O is None:
        O = torch.empty_like(Q)
    nws = pc_frame_attn_workspace_bytes(Hq, Nq, Nk, D)
    if ws is None and nws:
        ws = _workspace(nws, Q)
    if K.stride(0) != V.stride(0):
        raise PackCacheError(-2, "K and V must share their head stride")
    if lse is not None and (tuple(lse.shape) != (Hq, Nq) or not lse.is_contiguous()):
        raise PackCacheError(-2, f"lse must be a contiguous fp32 [{Hq}][{Nq}] tensor")
    _check(lib().pc_frame_attn(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _dtype_code(Q), Hq, Hkv, Nq, Nk, D,
                               Q.stride(0), K.stride(0), O.stride(0), float(scale), O.data_ptr(), _ptr(lse),
                               _ptr(ws), 0 if ws is None else ws.numel(), _stream()))
    return O
