/*
 * packcache.h -- C ABI of the PackCache hot path for AMD MI355X (gfx950).
 *
 * PackCache (arXiv 2601.04359) keeps the KV cache of an autoregressive video generator
 * small: text and conditioning-image keys are always kept ("condition anchoring",
 * Sec. 3.4), every past frame keeps a token budget that decays with its temporal
 * distance (Eq. 4-8), the tokens kept inside a frame are the attention-relevant ones,
 * dropped tokens are physically removed (Fig. 5(b)), and every kept token retains its
 * original (t, h, w) rotary position (Sec. 3.4).  The current frame's queries then
 * attend to the compacted cache (Eq. 2).
 *
 * Conventions shared by every call
 *   - Return value: PC_OK (0) or a negative pc_status.  pc_last_error_detail() gives a
 *     thread-local message for the last failing call.  Nothing aborts or throws.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host addresses.
 *     The caller owns every buffer.  The library allocates no device memory: scratch is
 *     a caller-provided device workspace whose size the *_workspace_bytes calls return.
 *   - Device work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream).  No call synchronises the stream (pc_compact_status, a check a
 *     caller may ask for, is the one exception); host outputs (segment tables, counts)
 *     never depend on device results.
 *   - Tensors are row-major with the head dimension D contiguous and rows dense
 *     (row stride = D elements); the stride between heads is passed in ELEMENTS.
 *   - dtype: PC_F32 is the correctness tier (D = 64 or 128), PC_BF16 the fast tier
 *     (D = 128; MFMA kernels, fp32 accumulation and softmax).
 *   - Query head h reads KV head h / (Hq / Hkv); Hq must be a multiple of Hkv.
 */
#ifndef PACKCACHE_H_
#define PACKCACHE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum pc_status {
  PC_OK = 0,
  PC_ERR_NULL = -1,        /* a required pointer is NULL */
  PC_ERR_SHAPE = -2,       /* a size, stride or segment table is inconsistent */
  PC_ERR_DTYPE = -3,       /* dtype is not PC_F32 / PC_BF16 */
  PC_ERR_UNSUPPORTED = -4, /* valid request the kernels do not cover (e.g. bf16 with D != 128) */
  PC_ERR_BUDGET = -5,      /* negative budget, bad decay factor or mode */
  PC_ERR_WORKSPACE = -6,   /* workspace NULL or smaller than *_workspace_bytes says */
  PC_ERR_HIP = -7,         /* a HIP runtime call or kernel launch failed */
  PC_ERR_ABORTED = -8      /* pc_compact_status: an in-place gather gave up its bounded wait */
} pc_status;

enum { PC_F32 = 0, PC_BF16 = 1 };

/* Kinds of cache segment.  TEXT and COND are the anchors, FRAME is a past frame (the
 * only kind that is pruned), SELF is an always-kept block of current-frame keys. */
enum { PC_SEG_TEXT = 0, PC_SEG_COND = 1, PC_SEG_FRAME = 2, PC_SEG_SELF = 3 };

/* One contiguous run of cache rows; the table is the same for every head. */
typedef struct pc_segment {
  int32_t start; /* first row */
  int32_t len;   /* number of rows */
  int32_t kind;  /* PC_SEG_* */
  int32_t frame; /* frame id (caller's bookkeeping; copied through) */
} pc_segment;

#define PC_MAX_SEGMENTS 120
#define PC_MAX_SELECT_LEN 4096 /* longest FRAME segment the register-resident select handles
                                  (one work-group per segment); longer segments take a slower
                                  generic path */

const char* pc_strerror(int status);
const char* pc_last_error_detail(void);
int pc_version(void);

/* ---------------------------------------------------------------------------------------
 * pc_budget -- per-frame token budgets from the temporal decay kernel (Sec. 3.4, Eq. 4-8).
 * Host only, synchronous.  budget_out is a host array [n_past]; entry d-1 belongs to the
 * frame at temporal distance d (d = 1 is the most recent past frame).
 *
 *   PC_BUDGET_POW    b(d) = min(N, max(b_min, floor(N * gamma^d)))   decay kernel g(d) =
 *                    gamma^d (Eq. 5) on a full frame of N = n_frame_tokens tokens with the
 *                    minimum quota as a floor.  gamma is the exact value of the double and
 *                    the product is floored exactly.
 *   PC_BUDGET_NORM   Eq. 6: share b_d = gamma^d / sum_{j<=W} gamma^j of a fixed budget of
 *                    N tokens (B_one), W = n_past.
 *   PC_BUDGET_HALF   Eq. 7: share b_d = 2^-min(d, W-1); gamma is ignored.
 *   PC_BUDGET_SLIDE  sliding-window baseline (Sec. 3.3): [N, 0, 0, ...].
 *
 * NORM and HALF with a minimum quota b_min > 0 (tokens): if W * b_min > N the oldest
 * frames get 0 until it fits (FIFO truncation, Sec. 3.4); every remaining frame gets
 * b_min plus its share of what is left.  Flooring leftovers go to d = 1 so that the
 * budgets add up to N exactly (Eq. 8).
 * Errors: PC_ERR_NULL, PC_ERR_BUDGET (mode, N < 0, n_past < 0, b_min < 0, gamma outside
 * (0, 1] for POW/NORM).
 */
enum { PC_BUDGET_POW = 0, PC_BUDGET_NORM = 1, PC_BUDGET_HALF = 2, PC_BUDGET_SLIDE = 3 };
int pc_budget(int mode, int n_frame_tokens, int n_past, double gamma, int b_min,
              int32_t* budget_out /* host [n_past] */);

/* ---------------------------------------------------------------------------------------
 * pc_rope3d -- 3D rotary embedding, in place (the operator R of Eq. 2; positions are the
 * token's own (t, h, w), which compaction never changes: Sec. 3.4, Eq. 9).
 *   x    dev, [H][n][D] of dtype, head stride stride_h elements; rotated in place.
 *   pos  dev, int32 [n][3] = (t, h, w) per row, already scaled by the caller.
 * D is cut into contiguous sections sec_t + sec_h + sec_w = D (all even).  Pair i of a
 * section of width s is dims (2i, 2i+1) and turns by pos_axis * base^(-2i/s).  Angles are
 * formed in fp64, the rotation in fp32.  A rebase by (-dt, 0, 0) is the same call with
 * pos = (-dt, 0, 0): rotations compose.
 *   out_scale > 0: the rotated row is multiplied by it before the one rounding to dtype
 *   (1.0: plain rotation).  Queries rotated with out_scale = PC_FOLDED_Q_SCALE(scale) carry
 *   the softmax scale of Eq. 2 and the base-2 conversion with them; pc_score and
 *   pc_frame_attn called with scale = PC_SCALE_FOLDED then compute the same softmax(scale *
 *   Q K^T) with one vector instruction per product element fewer.
 * Errors: PC_ERR_NULL, PC_ERR_DTYPE, PC_ERR_SHAPE (sections, D > 256, stride, out_scale),
 * PC_ERR_HIP.
 */
#define PC_SCALE_FOLDED 0.693147180559945309f                 /* ln 2: the scale left after folding */
#define PC_FOLDED_Q_SCALE(scale) ((scale) * 1.4426950408889634) /* scale * log2(e): goes into Q */
int pc_rope3d(void* x, int dtype, int H, int n, int D, int64_t stride_h,
              const int32_t* pos, int sec_t, int sec_h, int sec_w, double base, double out_scale,
              void* stream);

/* ---------------------------------------------------------------------------------------
 * pc_rebase -- temporal rebase of cached keys when the sliding window advances (Sec. 3.4,
 * the rebase equation): pos_t <- pos_t - delta_t, pos_h and pos_w unchanged.  The cache
 * holds keys that were rotated on insertion; rotations about one axis compose, so rows
 * row0 .. row0+n_rows-1 of every KV head are turned by -delta_t on the temporal section
 * (the first sec_t dims) only, in place, and delta_t is subtracted from the t coordinate of
 * the same rows of pos.
 *   K      dev, [Hkv][*][D], head stride k_stride_h (elements)
 *   pos    dev, int32 [Hsel][*][3], head stride pos_stride_h (int32 elements)
 *   delta_t  in position units (frames dropped x the temporal scale of Sec. 3.1)
 * The temporal section must be a whole number of 16-byte chunks (sec_t % 8 == 0 for bf16,
 * % 4 for fp32), else PC_ERR_UNSUPPORTED.  Enqueued on `stream`; no synchronisation.
 * Errors: PC_ERR_NULL, PC_ERR_DTYPE, PC_ERR_SHAPE, PC_ERR_UNSUPPORTED, PC_ERR_HIP.
 */
int pc_rebase(void* K, int dtype, int Hkv, int D, int64_t k_stride_h, int32_t* pos, int Hsel,
              int64_t pos_stride_h, int row0, int n_rows, int delta_t, int sec_t, int sec_h, int sec_w,
              double base, void* stream);

/* ---------------------------------------------------------------------------------------
 * pc_score -- importance of every cached key: the softmax probability it receives
 * (Eq. 2 probabilities, softmax over ALL Nk keys presented), summed over the n_qs scoring
 * queries and over the query heads of its KV group.  The paper only asks for
 * "attention-relevant" tokens (Sec. 3.4); this column mass is the reading built here.
 *   Qs     dev, [Hq][*][D]     queries (already rotated), head stride q_stride_h
 *   q_rows dev or NULL, int32 [n_qs]: rows of Qs that score (the same for every head),
 *          e.g. an evenly spread sample of the frame.  NULL: rows 0 .. n_qs-1.
 *   K      dev, [Hkv][Nk][D]   cached keys (already rotated), head stride k_stride_h
 *   lse    dev or NULL, fp32, head stride lse_stride_h, indexed like the rows of Qs (row
 *          q_rows[i] of head h is lse[h * lse_stride_h + q_rows[i]]; without q_rows, row i):
 *          natural-log sum-exp of that query's scaled logits over the same Nk keys, e.g.
 *          the lse output of a pc_frame_attn call over the same cache (Sec. 3.4: the mask
 *          is refreshed from attention the model computes anyway).  NULL: computed here
 *          (one extra QK^T pass).
 *   score  dev, fp32 [Hsel][Nk], head stride score_stride_h; Hsel = Hkv, or 1 when
 *          share_heads != 0 (mass summed over the KV heads as well).
 *   scale  > 0, the softmax scale of Eq. 2 (1/sqrt(D)).  scale = PC_SCALE_FOLDED (ln 2) with
 *          queries that carry scale * log2(e) (see pc_rope3d) is the same computation and takes
 *          the bf16 kernels' shorter loop; lse stays the natural-log sum-exp of the logits.
 *   key_begin, key_end   only keys [key_begin, key_end) get a score (key_end = 0: up to Nk);
 *          entries of `score` outside the range are not written.  Every key still counts in
 *          every query's softmax normaliser.  For callers that know which rows can be pruned at
 *          all (anchors never are; a frame that already sits at its budget is not either) and do
 *          not want to pay for scores nobody reads.
 * Summation order is fixed (no atomics): results are bit-reproducible.
 * Errors: PC_ERR_NULL, PC_ERR_DTYPE, PC_ERR_SHAPE, PC_ERR_UNSUPPORTED, PC_ERR_WORKSPACE,
 * PC_ERR_HIP.
 */
size_t pc_score_workspace_bytes(int Hq, int Hkv, int n_qs, int Nk, int share_heads);
int pc_score(const void* Qs, const void* K, int dtype, int Hq, int Hkv, int n_qs, int Nk,
             int D, int64_t q_stride_h, int64_t k_stride_h, const int32_t* q_rows, float scale,
             const float* lse, int64_t lse_stride_h, float* score, int64_t score_stride_h,
             int share_heads, int key_begin, int key_end, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * pc_compact_plan -- host half of compaction: the segment table and key count after
 * compaction (anchors and SELF at full length, a FRAME segment at min(len, budget)).
 * seg_in/budget/seg_out are host arrays [n_seg]; budget entries of non-FRAME segments
 * are ignored.  Segments must tile [0, Nk_in) in order.
 * Errors: PC_ERR_NULL, PC_ERR_SHAPE, PC_ERR_BUDGET.
 */
int pc_compact_plan(const pc_segment* seg_in, int n_seg, const int32_t* budget,
                    pc_segment* seg_out, int32_t* Nk_out);

/* ---------------------------------------------------------------------------------------
 * pc_compact -- per-frame top-k selection and physical compaction (Sec. 3.4, Fig. 5(b)).
 * For every selection head and every FRAME segment the budget[s] rows with the largest
 * score are kept (equal scores: lower row index first); all other rows of the segment
 * are removed.  Kept rows stay in their original order; K, V and pos rows are moved
 * bit-for-bit, so every token keeps its (t, h, w).
 *   K, V      dev, [Hkv][cap][D] of dtype, head stride kv_stride_h
 *   pos       dev, int32 [Hsel][cap][3], head stride pos_stride_h (elements)
 *   score     dev, fp32 [Hsel][Nk_in], head stride score_stride_h; finite, >= 0
 *   seg_in    host [n_seg], budget host [n_seg]   (see pc_compact_plan)
 *   K_out, V_out, pos_out   dev, same layout with strides kv_out_stride_h /
 *             pos_out_stride_h.  They may be the input buffers themselves (all three or
 *             none): the compaction is then done in place.  Partial overlap is an error
 *             the library cannot detect.
 *   idx_out   dev or NULL, int32 [Hsel][Nk_out], head stride idx_stride_h: source row of
 *             every packed row (ascending).
 *   seg_out   host [n_seg] or NULL, Nk_out host or NULL: as from pc_compact_plan.
 * Hsel = Hkv (every KV head keeps its own rows; counts are equal so tensors stay
 * rectangular) or 1 when share_heads != 0 (one selection for all heads).
 * In place, work-groups take their chunk of packed rows by ticket, load it, and wait (a
 * bounded spin) until every earlier chunk that still has to read the destination rows has
 * loaded them.  The tickets, flags and an abort word live in the workspace, so two calls that
 * run concurrently must not share a workspace, and a workspace must not be reused by another
 * stream before the call that uses it has finished.  The spin bound cannot be hit while the
 * workspace is used by one call at a time; if it is, the waiting work-groups give up, the
 * result of that call is undefined, nothing hangs, and pc_compact_status reports it.
 * Errors: PC_ERR_NULL, PC_ERR_DTYPE, PC_ERR_SHAPE (n_seg > PC_MAX_SEGMENTS, strides,
 * table), PC_ERR_BUDGET, PC_ERR_WORKSPACE, PC_ERR_HIP.
 */
size_t pc_compact_workspace_bytes(int Hkv, int Nk_in, int share_heads);
int pc_compact(void* K, void* V, int32_t* pos, int dtype, int Hkv, int D,
               int64_t kv_stride_h, int64_t pos_stride_h, const float* score,
               int64_t score_stride_h, const pc_segment* seg_in, int n_seg,
               const int32_t* budget, int share_heads, void* K_out, void* V_out,
               int32_t* pos_out, int64_t kv_out_stride_h, int64_t pos_out_stride_h,
               int32_t* idx_out, int64_t idx_stride_h, pc_segment* seg_out, int32_t* Nk_out,
               void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * pc_compact_static -- pc_compact for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and errors as pc_compact, minus ws / ws_bytes: the
 * scratch (kept-row indices, tickets and flags of the in-place gather) lives in an array of
 * PC_COMPACT_STATIC_BYTES that is part of the library's device image; every GPU the library
 * runs on holds it until the process ends.  The call allocates and frees nothing.
 *   - A request that needs more than the array holds (pc_compact_workspace_bytes(Hkv, Nk_in,
 *     share_heads) > pc_compact_static_capacity()) is rejected with PC_ERR_WORKSPACE before any
 *     device work; use pc_compact with a workspace of your own for it.  The array covers
 *     4 KV heads x 193,792 rows (the 48-frame cache) and 8 KV heads x 98,304 rows.
 *   - All calls on one GPU share that GPU's array, which keeps the last call's contents; every
 *     call clears what it needs with its own kernel first.  Calls that overlap on one GPU (two
 *     streams, two host threads) race on it: issue them one after another on one stream, or
 *     order them with events.
 */
#define PC_COMPACT_STATIC_BYTES (4u << 20)
size_t pc_compact_static_capacity(void);
int pc_compact_static(void* K, void* V, int32_t* pos, int dtype, int Hkv, int D,
                      int64_t kv_stride_h, int64_t pos_stride_h, const float* score,
                      int64_t score_stride_h, const pc_segment* seg_in, int n_seg,
                      const int32_t* budget, int share_heads, void* K_out, void* V_out,
                      int32_t* pos_out, int64_t kv_out_stride_h, int64_t pos_out_stride_h,
                      int32_t* idx_out, int64_t idx_stride_h, pc_segment* seg_out, int32_t* Nk_out,
                      void* stream);

/* ---------------------------------------------------------------------------------------
 * pc_compact_batch -- pc_compact for n_layers layers at once (the caches of a layer stack are
 * re-packed together at a frame-step boundary): one select launch and one gather launch
 * cover every layer, so the small per-layer launches neither queue behind each other nor
 * leave the chip part empty.  Layer l of every tensor starts *_stride_l elements after
 * layer l-1 (K, V: elements of dtype; pos, idx: int32; score: fp32); everything else is as
 * in pc_compact and is the same for all layers: one segment table, one budget per segment
 * (budgets depend on the temporal distance only), one dtype, Hkv and D.  n_layers = 1 with
 * zero layer strides is pc_compact.  In place, n_layers * Hkv must not exceed 256.
 * The workspace is sized by pc_compact_batch_workspace_bytes.
 */
size_t pc_compact_batch_workspace_bytes(int n_layers, int Hkv, int Nk_in, int share_heads);
int pc_compact_batch(int n_layers, void* K, void* V, int32_t* pos, int dtype, int Hkv, int D,
                     int64_t kv_stride_h, int64_t kv_stride_l, int64_t pos_stride_h,
                     int64_t pos_stride_l, const float* score, int64_t score_stride_h,
                     int64_t score_stride_l, const pc_segment* seg_in, int n_seg,
                     const int32_t* budget, int share_heads, void* K_out, void* V_out,
                     int32_t* pos_out, int64_t kv_out_stride_h, int64_t kv_out_stride_l,
                     int64_t pos_out_stride_h, int64_t pos_out_stride_l, int32_t* idx_out,
                     int64_t idx_stride_h, int64_t idx_stride_l, pc_segment* seg_out,
                     int32_t* Nk_out, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * pc_compact_batch_phase -- the two halves of pc_compact_batch as separate calls, so that a
 * caller can overlap them on two streams: the SELECT of the next layer (reads only scores;
 * writes the kept-row indices and resets the in-place bookkeeping in the workspace) runs
 * while the GATHER of the current layer moves rows.  phases = PC_COMPACT_SELECT, then
 * PC_COMPACT_GATHER with the SAME arguments and workspace (the caller orders the two with an
 * event when they are on different streams), or both bits at once (= pc_compact_batch).
 * Every argument is checked in both calls; SELECT does not touch K, V or pos.
 */
enum { PC_COMPACT_SELECT = 1, PC_COMPACT_GATHER = 2 };
int pc_compact_batch_phase(int phases, int n_layers, void* K, void* V, int32_t* pos, int dtype, int Hkv,
                           int D, int64_t kv_stride_h, int64_t kv_stride_l, int64_t pos_stride_h,
                           int64_t pos_stride_l, const float* score, int64_t score_stride_h,
                           int64_t score_stride_l, const pc_segment* seg_in, int n_seg,
                           const int32_t* budget, int share_heads, void* K_out, void* V_out,
                           int32_t* pos_out, int64_t kv_out_stride_h, int64_t kv_out_stride_l,
                           int64_t pos_out_stride_h, int64_t pos_out_stride_l, int32_t* idx_out,
                           int64_t idx_stride_h, int64_t idx_stride_l, pc_segment* seg_out,
                           int32_t* Nk_out, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * pc_compact_status -- did the last in-place compaction that used workspace `ws` run to the
 * end?  Waits for `stream` (the stream that compaction was enqueued on), reads one word of
 * the workspace back and returns PC_OK, or PC_ERR_ABORTED when a work-group hit the spin bound
 * of its wait (the packed rows of that call are then not to be trusted).  The word is reset by
 * the next compaction call on the workspace.  For callers that want the check; the path itself
 * never needs it.  Errors: PC_ERR_NULL, PC_ERR_HIP, PC_ERR_ABORTED.
 */
int pc_compact_status(const void* ws, void* stream);

/* ---------------------------------------------------------------------------------------
 * Cache mask (Sec. 3.1: a binary mask says which generated tokens are visible to later
 * frames; Sec. 3.4: PackCache removes the masked positions instead of storing them).
 * One flag per cached token, the same for every head: valid[j] != 0 keeps token j a
 * candidate.  Two calls put the mask in front of pc_compact:
 *   pc_masked_budgets  host only: budget_out[s] = min(budget[s], unmasked tokens of segment
 *                      s) for FRAME segments, budget[s] otherwise.  valid is a HOST array
 *                      covering every row the table names.
 *   pc_mask_scores     device: score[h][j] = -1 where valid[j] == 0 (valid is a DEVICE array
 *                      [Nk]), so that a masked token never outranks an unmasked one.
 * pc_compact with the masked scores and budgets then keeps, per past frame, the
 * top-budget unmasked tokens and physically removes the rest.  Anchors are not pruned and
 * ignore the mask.
 * Masked entries are ignored in attention (Sec. 3.1, after Eq. 1): a masked key must not count
 * in the softmax of pc_score or pc_frame_attn either, and neither call takes a mask.  Remove the
 * masked rows of a frame when it ENTERS the cache instead: give its rows the score 0, call
 * pc_mask_scores on them, and call pc_compact over the whole table with the new segment's budget
 * = its unmasked count and every other segment's budget = its length (rows that stay where they
 * are cost nothing in place).  Only unmasked rows are then ever scored or attended to.
 * Errors: PC_ERR_NULL, PC_ERR_SHAPE, PC_ERR_BUDGET, PC_ERR_HIP.
 */
int pc_masked_budgets(const pc_segment* seg, int n_seg, const int32_t* budget, const uint8_t* valid,
                      int32_t* budget_out);
int pc_mask_scores(float* score, int Hsel, int Nk, int64_t score_stride_h, const uint8_t* valid,
                   void* stream);

/* ---------------------------------------------------------------------------------------
 * pc_frame_attn -- attention of one frame's queries over the keys presented (Eq. 2):
 * O = softmax(Q K^T * scale) V.  K is already rotated; for the current frame's queries
 * against anchors and earlier frames the causal mask of Eq. 2 hides nothing, so no mask
 * is applied.  The same call serves the packed and the full ("dense") cache.
 *   Q  dev [Hq][Nq][D], K, V dev [Hkv][Nk][D], O dev [Hq][Nq][D] (dtype; bf16 is rounded
 *   to nearest even), lse dev or NULL fp32 [Hq][Nq] = ln sum_j exp(scale * q.k_j).
 *   scale > 0.  scale = PC_SCALE_FOLDED with queries that carry scale * log2(e) (see
 *   pc_rope3d) is the same computation on the bf16 kernel's shorter loop: the scores start
 *   from minus the running reference inside the matrix product and the probability is a bare
 *   exp2.
 *   ws  dev or NULL: optional.  With a workspace of pc_frame_attn_workspace_bytes (0 for most
 *   shapes) the bf16 kernel may cut the keys into shares when Hq * ceil(Nq / 256) work-groups
 *   would fill the chip badly, and merge the partial results; without it (or with one that is
 *   too small) the keys are not split.  Results agree to the rounding of the output.
 * Nk >= 1, Nq >= 1.  Errors: PC_ERR_NULL, PC_ERR_DTYPE, PC_ERR_SHAPE, PC_ERR_UNSUPPORTED,
 * PC_ERR_HIP.
 */
size_t pc_frame_attn_workspace_bytes(int Hq, int Nq, int Nk, int D);
int pc_frame_attn(const void* Q, const void* K, const void* V, int dtype, int Hq, int Hkv,
                  int Nq, int Nk, int D, int64_t q_stride_h, int64_t kv_stride_h,
                  int64_t o_stride_h, float scale, void* O, float* lse, void* ws,
                  size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PACKCACHE_H_ */
