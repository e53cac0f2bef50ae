/*
 * metok.h -- C ABI of the METok token-compression hot path for AMD MI355X (gfx950).
 *
 * METok (arXiv 2506.02850) removes visual tokens of a video LLM in three stages:
 *   stage 1 (Sec. 3.2.1, Algorithm 1): split the frames into events at the lowest adjacent-frame
 *           cosine similarities (Eq. 4), rank events and frames against a text embedding (Eq. 5)
 *           and pool every frame's patch grid with a stride that depends on that ranking;
 *   stage 2 (Sec. 3.2.2, Eq. 6-7): at chosen prefill layers keep only the visual tokens that
 *           receive the most attention from the text, with per-class retention quotas, and
 *           compact the hidden states;
 *   stage 3 (Sec. 3.3): compact the KV cache to the retained rows.
 *
 * Conventions shared by every call
 *   - Every pointer named "device" is GPU memory of the current HIP device; "host" is ordinary
 *     host memory.  The library never allocates, frees or keeps a pointer: the caller owns all
 *     buffers, including the scratch `workspace`, whose minimum size comes from the matching
 *     *_workspace_bytes() query (called with the same shape arguments).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls only enqueue
 *     work on that stream; they never synchronise.  Results are deterministic: the same inputs
 *     give bit-identical outputs (no floating-point atomics anywhere).
 *   - Calls may be captured into a HIP graph (they only launch kernels: no memsets, no copies).  Make one
 *     ordinary call of each entry point on a device before capturing it there: the first call loads the
 *     code objects and, for metok_segment_compress, sets a launch attribute of one kernel once per device.
 *   - Return value: METOK_OK or a negative METOK_ERR_* code.  On error nothing has been
 *     enqueued (argument errors) or the launch failed (METOK_ERR_DEVICE); metok_last_error()
 *     returns a thread-local description.
 *   - dtype is METOK_F32 or METOK_BF16; tensors are dense, row-major, innermost dimension last,
 *     16-byte aligned.  Indices and counts stored in memory are int32.
 *   - Inputs must be finite.  NaN/Inf never cause out-of-bounds accesses but make the
 *     selections unspecified.
 *   - Ratios are turned into counts with ceil(x - 1e-9) evaluated in double precision, the
 *     guarded form of the paper's ceil(alpha k) (Sec. 3.2.1); ties in every ranking go to the
 *     lower index.
 */
#ifndef METOK_H
#define METOK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define METOK_API __attribute__((visibility("default")))

enum {
    METOK_OK = 0,
    METOK_ERR_INVALID_ARG = -1,  /* a shape, ratio, pointer or alignment is not acceptable */
    METOK_ERR_UNSUPPORTED = -2,  /* valid request that this build has no kernel for */
    METOK_ERR_WORKSPACE = -3,    /* workspace missing or smaller than *_workspace_bytes() */
    METOK_ERR_CAPACITY = -4,     /* an output buffer is smaller than the worst case */
    METOK_ERR_DEVICE = -5        /* the HIP runtime reported an error */
};

enum { METOK_F32 = 0, METOK_BF16 = 1 };
enum { METOK_SIM_FLAT = 0, METOK_SIM_TOKEN_MEAN = 1, METOK_SIM_POOLED = 2 };  /* readings of Eq. 4, see below */
enum { METOK_SCORE_CAUSAL_ALL = 0, METOK_SCORE_VISUAL_ONLY = 1 };             /* softmax support of the stage-2 score */
enum { METOK_EVENT_MEAN = 0, METOK_EVENT_MAX = 1 };/* event score: Sec. 3.2.1 text / Algorithm 1 */
enum { METOK_POOL_FLOOR = 0, METOK_POOL_CEIL = 1 };/* output side floor(g/s) or ceil(g/s) */

#define METOK_MAX_FRAMES 8192     /* T limit of the stage-1 calls */
#define METOK_MAX_BATCH 64        /* videos per batched call */
#define METOK_MAX_SEGMENTS 256    /* n_seg limit of metok_prefill_prune */
#define METOK_MAX_LAYERS 128      /* L limit of metok_kv_compact */

/*
 * The method's hyperparameters for one base model (Appendix "Implementation Details"; frame counts from
 * Sec. 4 "Implementation Details").  A plain record: the calls below take the individual values.
 *   frames     frames sampled per video          n_layers   transformer layers of the LLM
 *   k          events (Sec. 3.2.1)               layers_h   L_H = [l_1, l_2, l_3], 0-based (Sec. 3.2.2)
 *   alpha      key-event ratio                   beta       key-frame ratio inside an event
 *   s1, s2     pooling strides of key / non-key frames in key events
 *   r          retention ratio of Eq. 6-7
 */
typedef struct metok_params {
    int32_t frames;
    int32_t n_layers;
    int32_t k;
    int32_t s1, s2;
    int32_t layers_h[3];
    double alpha, beta, r;
} metok_params;

/* Initialisers in field order: frames, n_layers, k, s1, s2, {l_1, l_2, l_3}, alpha, beta, r. */
#define METOK_PRESET_LLAVA_OV_0_5B { 32, 24, 5, 2, 3, {3, 10, 19}, 0.5, 0.4, 0.76 }
#define METOK_PRESET_LLAVA_OV_7B   { 32, 28, 5, 2, 3, {3, 10, 19}, 0.5, 0.4, 0.76 }
#define METOK_PRESET_LONGVA_7B     { 128, 28, 13, 2, 3, {3, 10, 19}, 0.5, 0.45, 0.55 }
#define METOK_PRESET_VILA_13B      { 16, 40, 3, 2, 3, {13, 24, 34}, 0.5, 0.4, 0.65 }

enum { METOK_MODEL_LLAVA_OV_0_5B = 0, METOK_MODEL_LLAVA_OV_7B = 1, METOK_MODEL_LONGVA_7B = 2, METOK_MODEL_VILA_13B = 3 };

/* Copies the preset of METOK_MODEL_* into *out (for callers that cannot use the initialiser macros). */
METOK_API int metok_preset(int model, metok_params* out);

/* Thread-local text of the last error returned on this thread ("" if none). */
METOK_API const char* metok_last_error(void);

/* Library version: major * 10000 + minor * 100 + patch. */
METOK_API int metok_version(void);

/* ---------------------------------------------------------------------------------------------
 * Stage 1a -- temporal event segmentation (Sec. 3.2.1 "Temporal Event Segmentation", Eq. 4;
 * the segmentation step of Algorithm 1), optionally fused with the frame-text relevance of Eq. 5 so
 * that the frame features are streamed from HBM once.
 *
 *   feats        device, [T, N, d] of `dtype`: N patch tokens of width d for each of T frames.
 *   text_emb     device, [d] of `dtype`, or NULL.  When given, frame_score is produced.
 *   k            number of events, 1 <= k <= T.
 *   sim_mode     METOK_SIM_FLAT (default): S_i = <v_i, v_{i+1}> / (|v_i| |v_{i+1}|) with the inner product
 *                and norms over all N*d entries (a denominator below 1e-12 gives S_i = 0).
 *                METOK_SIM_TOKEN_MEAN: mean over the N token positions of the cosine of the two
 *                frames' tokens at that position.  METOK_SIM_POOLED: cosine of the two frames'
 *                mean tokens (one more pass over feats; d <= 4096).  Eq. 4 writes a cosine of two
 *                N x d embeddings without saying which of these it means.
 *   sim          device out, [T-1] float: S_i for the pair (i, i+1), i = 0..T-2.
 *   event_start  device out, [k+1] int32: event e covers frames [event_start[e], event_start[e+1]);
 *                event_start[0] = 0, event_start[k] = T, strictly increasing.  The k-1 lowest
 *                S_i are the boundaries; a boundary at i makes frame i+1 open an event.
 *   frame_event  device out, [T] int32: event id of every frame.
 *   frame_score  device out, [T] float, or NULL: mean over the frame's N tokens of
 *                cos(token, text_emb) (Eq. 5 read per token).  Requires text_emb.
 *   Limits: 1 <= T <= METOK_MAX_FRAMES (T = 1: no similarities, one event); T * N < 2^31;
 *   d a multiple of 8 (bf16) or 4 (f32) and at most 8192 (bf16) / 4096 (f32).
 * ------------------------------------------------------------------------------------------- */
METOK_API size_t metok_segment_events_workspace_bytes(int T, int N, int d, int dtype);

METOK_API int metok_segment_events(const void* feats, int dtype, int T, int N, int d,
                         const void* text_emb, int k, int sim_mode,
                         float* sim, int32_t* event_start, int32_t* frame_event,
                         float* frame_score,
                         void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Stage 1b -- key event / key frame identification and adaptive pooling (Sec. 3.2.1 "Key
 * Visual-Text Semantic Identification" and "Adaptive Pooling Strategy"; Algorithm 1 after its
 * segmentation step).
 *
 *   feats           device, [T, grid_h*grid_w, d] of `dtype`; tokens of a frame are row-major
 *                   over the grid_h x grid_w patch grid.
 *   text_emb        device, [d] of `dtype`; used only when frame_score_in is NULL.
 *   frame_score_in  device, [T] float from metok_segment_events, or NULL to compute it here.
 *   event_start     device, [k+1] int32 as written by metok_segment_events.
 *   alpha, beta     key-event and key-frame ratios, 0 < ratio <= 1: ceil(alpha k) events with
 *                   the best event score are key; in every event ceil(beta len) frames with the
 *                   best frame score are key frames.
 *   s1, s2          pooling strides (>= 1) of key / non-key frames in key events; non-key
 *                   events use ceil(s1/alpha), ceil(s2/alpha).  Strides are clamped to
 *                   max(grid_h, grid_w).
 *   event_reduce    METOK_EVENT_MEAN (default of the paper's text) or METOK_EVENT_MAX.
 *   pool_edge       METOK_POOL_FLOOR: output side max(1, floor(g/s)), trailing cells that do
 *                   not fill a window are dropped; METOK_POOL_CEIL: side ceil(g/s), edge
 *                   windows average their valid cells.  Pooling is a non-overlapping s x s mean.
 *   out_tokens      device out, [out_capacity_rows, d] of `out_dtype`: pooled frames appended in
 *                   temporal order; row count M = frame_offsets[T] (data dependent).  Means are
 *                   accumulated in fp32 and rounded once (nearest even) to out_dtype.
 *   out_capacity_rows  must be >= T * side(grid_h, min(s1,s2)) * side(grid_w, min(s1,s2)), the
 *                   worst case, else METOK_ERR_CAPACITY.
 *   frame_offsets   device out, [T+1] int32: pooled rows of frame i are [offsets[i], offsets[i+1]).
 *   token_event     device out, [out_capacity_rows] int32: event id of every pooled row.
 *   event_is_key    device out, [k] uint8.        frame_is_key  device out, [T] uint8.
 *   frame_stride    device out, [T] int32.        event_score   device out, [k] float.
 *   frame_score_out device out, [T] float or NULL (copy of the scores used).
 * ------------------------------------------------------------------------------------------- */
METOK_API size_t metok_compress_encoder_tokens_workspace_bytes(int T, int grid_h, int grid_w, int d, int dtype);

/* Rows that out_tokens / token_event must hold for these settings (the worst case over all segmentations:
 * every frame pooled with the smaller of s1, s2), or -1 for arguments the call would reject. */
METOK_API int64_t metok_compress_encoder_tokens_capacity_rows(int T, int grid_h, int grid_w, int s1, int s2, int pool_edge);

METOK_API int metok_compress_encoder_tokens(const void* feats, int dtype, int T, int grid_h, int grid_w, int d,
                                  const void* text_emb, const float* frame_score_in,
                                  const int32_t* event_start, int k,
                                  double alpha, double beta, int s1, int s2,
                                  int event_reduce, int pool_edge,
                                  void* out_tokens, int64_t out_capacity_rows, int out_dtype,
                                  int32_t* frame_offsets, int32_t* token_event,
                                  uint8_t* event_is_key, uint8_t* frame_is_key,
                                  int32_t* frame_stride, float* event_score, float* frame_score_out,
                                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Stage 1 in one call (Sec. 3.2.1, Algorithm 1: Eq. 4 segmentation, Eq. 5 scores, key events / key
 * frames, adaptive pooling).  Arguments and outputs are those of metok_segment_events followed by
 * metok_compress_encoder_tokens (N = grid_h * grid_w; text_emb and frame_score are required), and so are
 * the results.  When every frame is pooled with stride 2 whatever the segmentation decides -- s1, s2,
 * ceil(s1 / alpha), ceil(s2 / alpha) all equal 2 after clamping, e.g. the uniform setting s1 = s2 = 2,
 * alpha = 1 -- and both grid sides are even, sim_mode is METOK_SIM_FLAT and d spans at most 256 16-byte
 * chunks, the frame statistics and the pooled tokens are produced in ONE pass over the frame features;
 * in every other case the two calls run back to back on the same stream (two passes).
 * Workspace: metok_segment_compress_workspace_bytes.  Errors as for the two calls.
 */
METOK_API size_t metok_segment_compress_workspace_bytes(int T, int grid_h, int grid_w, int d, int dtype);

METOK_API int metok_segment_compress(const void* feats, int dtype, int T, int grid_h, int grid_w, int d,
                           const void* text_emb, int k, int sim_mode,
                           double alpha, double beta, int s1, int s2, int event_reduce, int pool_edge,
                           float* sim, int32_t* event_start, int32_t* frame_event,
                           void* out_tokens, int64_t out_capacity_rows, int out_dtype,
                           int32_t* frame_offsets, int32_t* token_event,
                           uint8_t* event_is_key, uint8_t* frame_is_key,
                           int32_t* frame_stride, float* event_score, float* frame_score,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Stage 1 in one call for a batch of videos of one shape (Sec. 3.2.1, Algorithm 1): metok_segment_compress on each of
 * `batch` videos (1 <= batch <= METOK_MAX_BATCH) with the same settings.  Every kernel is launched once for the whole
 * batch (four launches in the one-pass case, four in the two-pass case: statistics, segmentation, plan, pooling; the
 * planning kernels, one workgroup per video, run side by side); only with METOK_SIM_POOLED the videos are processed
 * one after the other.  Per video the results are those of metok_segment_compress, bit for bit.
 *   Every array carries a leading batch dimension and is tightly packed: feats [batch, T, N, d], text_emb [batch, d],
 *   sim [batch, T-1], event_start [batch, k+1], frame_event / frame_is_key / frame_stride / frame_score [batch, T],
 *   out_tokens [batch, out_capacity_rows, d], token_event [batch, out_capacity_rows], frame_offsets [batch, T+1],
 *   event_is_key / event_score [batch, k].  workspace: metok_segment_compress_batched_workspace_bytes(batch, ...).
 */
METOK_API size_t metok_segment_compress_batched_workspace_bytes(int batch, int T, int grid_h, int grid_w, int d, int dtype);

METOK_API int metok_segment_compress_batched(int batch, const void* feats, int dtype, int T, int grid_h, int grid_w, int d,
                           const void* text_emb, int k, int sim_mode,
                           double alpha, double beta, int s1, int s2, int event_reduce, int pool_edge,
                           float* sim, int32_t* event_start, int32_t* frame_event,
                           void* out_tokens, int64_t out_capacity_rows, int out_dtype,
                           int32_t* frame_offsets, int32_t* token_event,
                           uint8_t* event_is_key, uint8_t* frame_is_key,
                           int32_t* frame_stride, float* event_score, float* frame_score,
                           void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Stage 2 -- one level of hierarchical token pruning (Sec. 3.2.2).
 *
 * Retention quotas of Eq. 6-7 (host arithmetic only): level 0 = before l_1, 1 = [l_1, l_2),
 * 2 = [l_2, l_3), 3 = from l_3 on.  Key-event tokens keep 1, r, r^2, 0 of the n_key_orig tokens
 * that entered the LLM, non-key tokens keep 1, alpha r, 0, 0 of n_non_orig.
 * quota_out[0] = key quota, quota_out[1] = non-key quota.
 * ------------------------------------------------------------------------------------------- */
METOK_API int metok_retention_quotas(int level, double r, double alpha, int64_t n_key_orig, int64_t n_non_orig,
                           int32_t quota_out[2]);

/*
 * Closed-form bookkeeping of the three stages (host arithmetic only, no tensors): how many tokens
 * each stage leaves and how many (token, layer) pairs the prefill computes and the cache holds.
 *
 *   event_len, event_is_key  host, [k]: frames per event and its key flag (Sec. 3.2.1).
 *   grid_h, grid_w, alpha, beta, s1, s2, pool_edge  as in metok_compress_encoder_tokens: an event of
 *                n frames has ceil(beta n) key frames; strides s1 / s2 (key / non-key frames), divided
 *                by alpha and rounded up in non-key events; a frame pooled with stride s leaves
 *                side(grid_h, s) * side(grid_w, s) tokens.
 *   r, layers_h  Eq. 6-7: from layer layers_h[i-1] on (0-based, ascending) the level-i quotas of
 *                metok_retention_quotas apply to the key / non-key counts that entered the LLM.
 *   n_layers, n_text  LLM depth (<= METOK_MAX_LAYERS) and text rows.
 * Multiply a (token, layer) count by 2 * Hkv * dh * sizeof(dtype) for cache bytes.
 */
typedef struct metok_account_t {
    int64_t tokens_encoder;           /* frames * grid_h * grid_w */
    int64_t tokens_llm;               /* visual tokens after stage 1 = tokens_key + tokens_non */
    int64_t tokens_key, tokens_non;   /* of key / non-key events */
    int64_t level_tokens[4];          /* visual tokens alive at pruning level 0..3 */
    int64_t prefill_token_layers;     /* sum over layers of (visual tokens alive + n_text) */
    int64_t kv_token_layers_full;     /* cache without stages 2 and 3 */
    int64_t kv_token_layers_stage2;   /* every layer caches what it processed */
    int64_t kv_token_layers_stage3;   /* Sec. 3.3: layers >= layers_h[0] keep the text rows only */
} metok_account_t;

METOK_API int metok_account(const int32_t* event_len, const uint8_t* event_is_key, int k, int grid_h, int grid_w,
                  double alpha, double beta, int s1, int s2, int pool_edge, double r,
                  const int32_t layers_h[3], int n_layers, int64_t n_text, metok_account_t* out);

/*
 * The sequence is X = [prefix; X_vis; X_text] (Eq. 3): vis_start prefix rows, n_vis visual rows,
 * then S - vis_start - n_vis text rows.
 *
 *   hidden       device, [S, D] of `dtype`.
 *   q_text       device, [Hq, Tq, dh] of `dtype`: queries of the LAST Tq positions of the sequence
 *                (Tq <= number of text rows), or NULL: then `scores` is an input and the
 *                attention step is skipped.
 *   k_all        device, [Hkv, S, dh] of `dtype`: keys of all S positions (ignored if q_text NULL).
 *                Query head h reads kv head h / (Hq / Hkv).
 *   score_mode   METOK_SCORE_CAUSAL_ALL: the softmax of a query at position p runs over keys 0..p
 *                (prefix, visual and earlier text keys all take probability mass).
 *                METOK_SCORE_VISUAL_ONLY: it runs over the n_vis visual keys alone.
 *                Ignored if q_text is NULL.
 *   token_seg    device, [n_vis] int32 in [0, n_seg): retention class of each visual token
 *                (e.g. 0 = key event, 1 = non-key event; or the event id; or all 0).
 *   token_event  device, [n_vis] int32 in [0, n_events): event of each visual token.
 *   event_weight device, [n_events] float or NULL (= 1): importance multiplier w_e.
 *   seg_quota    host, [n_seg] int32: tokens to keep per class, 0 <= quota <= class population.
 *                (The populations live on the device and cannot be checked here: a quota above
 *                its class population keeps the whole class and the tail of the outputs is
 *                padded with index 0; nothing is read or written out of bounds.)
 *   orig_idx_in  device, [n_vis] int32 or NULL (= 0..n_vis-1): index of each visual token in the
 *                sequence that first entered the LLM (carried through the levels).
 *   scores       device, [n_vis] float.  Out (in when q_text is NULL):
 *                score_j = w_{e(j)} * mean over the Hq*Tq (head, query) pairs of the causal
 *                softmax probability of visual key j, logits q.k / sqrt(dh), each query at
 *                position p attending keys 0..p.
 *   kept_idx     device out, [sum quota] int32: kept visual positions (0-based inside the visual
 *                span), ascending.  Per class the quota highest scores are kept.
 *   hidden_out   device out, [S - n_vis + sum quota, D]: prefix rows, kept visual rows in order,
 *                text rows.  Either disjoint from `hidden` (a parallel gather, the fast path) or the very
 *                same pointer: then the sequence is compacted in place (rows move towards the front in
 *                ordered tiles, no second [S, D] buffer; rows of at most 16384 bytes; the rows behind the
 *                compacted sequence are unspecified afterwards).  Any other overlap is refused.
 *   token_seg_out, token_event_out, orig_idx_out  device out, [sum quota] int32 (each may be NULL).
 *   Limits: dh in {32, 64, 128, 256} for bf16, {32, 64, 128} for f32; Hq a multiple of Hkv;
 *   D * sizeof(dtype) a multiple of 16; n_seg <= METOK_MAX_SEGMENTS.
 */
METOK_API size_t metok_prefill_prune_workspace_bytes(int64_t S, int Hq, int Hkv, int dh, int Tq, int n_vis, int dtype);

METOK_API int metok_prefill_prune(const void* hidden, int64_t S, int D, int dtype,
                        const void* q_text, const void* k_all, int Hq, int Hkv, int dh, int Tq,
                        int score_mode, int vis_start, int n_vis,
                        const int32_t* token_seg, const int32_t* token_event,
                        const float* event_weight, int n_events,
                        int n_seg, const int32_t* seg_quota,
                        const int32_t* orig_idx_in,
                        float* scores, int32_t* kept_idx, void* hidden_out,
                        int32_t* token_seg_out, int32_t* token_event_out, int32_t* orig_idx_out,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Sec. 3.2.2 for a batch of videos of one shape: the call of metok_prefill_prune on each of `batch` videos
 * (1 <= batch <= METOK_MAX_BATCH), run as ONE sequence of launches whose grids span the whole batch, so that the
 * per-kernel launch cost and the tail of every grid are paid once per level, not once per video.  Per video the
 * results are those of metok_prefill_prune on that video: the same selection rule and the same row copies; the scores
 * may differ in the last bits, because a video's keys are split over fewer workgroups and the partial sums are added
 * in another order.
 *   Inputs carry a leading batch dimension and are tightly packed: hidden [batch, S, D], q_text [batch, Hq, Tq, dh],
 *   k_all [batch, Hkv, S, dh], token_seg / token_event / scores [batch, n_vis], event_weight [batch, n_events];
 *   orig_idx_in is [batch, orig_idx_in_stride] (>= n_vis; its own stride, like orig_idx_out below);
 *   seg_quota is host [batch, n_seg] (the kept count may differ between videos).
 *   Outputs: kept_idx, token_seg_out, token_event_out are [batch, keep_stride] (keep_stride >= the largest video's sum
 *   of quotas; entries past a video's own count are not written); orig_idx_out is [batch, orig_idx_stride] with the
 *   same rule (its own stride, so that it can be the leading columns of stage 3's index lists [batch, kept + text]);
 *   hidden_out is [batch, out_row_stride, D] (out_row_stride >= S - n_vis + that largest count; rows past a video's own
 *   count are not written).
 *   hidden_out == hidden compacts every video in place (out_row_stride must be S).
 *   workspace: metok_prefill_prune_batched_workspace_bytes(batch, ...) bytes.
 */
METOK_API size_t metok_prefill_prune_batched_workspace_bytes(int batch, int64_t S, int Hq, int Hkv, int dh, int Tq, int n_vis, int dtype);

METOK_API int metok_prefill_prune_batched(int batch, const void* hidden, int64_t S, int D, int dtype,
                        const void* q_text, const void* k_all, int Hq, int Hkv, int dh, int Tq,
                        int score_mode, int vis_start, int n_vis,
                        const int32_t* token_seg, const int32_t* token_event,
                        const float* event_weight, int n_events,
                        int n_seg, const int32_t* seg_quota,
                        const int32_t* orig_idx_in, int64_t orig_idx_in_stride,
                        float* scores, int32_t* kept_idx, int64_t keep_stride,
                        void* hidden_out, int64_t out_row_stride,
                        int32_t* token_seg_out, int32_t* token_event_out,
                        int32_t* orig_idx_out, int64_t orig_idx_stride,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * metok_prefill_prune without a workspace argument, for callers that cannot allocate device memory
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the scratch
 * memory is a fixed METOK_STATIC_SCRATCH_BYTES array inside the library's device image (every GPU the
 * library runs on holds one copy until the process ends).  Arguments, results and errors are those of
 * metok_prefill_prune; the call allocates nothing and launches the same kernels.
 *   - Shapes whose metok_prefill_prune_workspace_bytes() exceeds METOK_STATIC_SCRATCH_BYTES are refused
 *     with METOK_ERR_WORKSPACE before anything is enqueued.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 *     streams or threads) race on it; serialise them or use metok_prefill_prune.  Nothing in the array
 *     has to survive between calls and nothing has to be cleared: every kernel writes what it reads.
 */
#define METOK_STATIC_SCRATCH_BYTES (8u << 20)

METOK_API size_t metok_static_scratch_bytes(void);

METOK_API int metok_prefill_prune_static(const void* hidden, int64_t S, int D, int dtype,
                               const void* q_text, const void* k_all, int Hq, int Hkv, int dh, int Tq,
                               int score_mode, int vis_start, int n_vis,
                               const int32_t* token_seg, const int32_t* token_event,
                               const float* event_weight, int n_events,
                               int n_seg, const int32_t* seg_quota,
                               const int32_t* orig_idx_in,
                               float* scores, int32_t* kept_idx, void* hidden_out,
                               int32_t* token_seg_out, int32_t* token_event_out, int32_t* orig_idx_out,
                               void* stream);

/* ---------------------------------------------------------------------------------------------
 * Stage 3 -- KV-cache compaction to the retained rows (Sec. 3.3), in place.
 *
 *   k_layers, v_layers  host arrays of L device pointers; layer l holds K (resp. V) as
 *                [B, Hkv, S_cap, dh] of `dtype` (Eq. 3 per layer, head-major).
 *   idx          host array of L device pointers; idx[l] is [B, n_keep[l]] int32, strictly
 *                ascending positions 0 <= p < S_cap inside the current cache for each video b,
 *                including the text rows that stay.  idx[l] == NULL: layer l is left untouched.
 *                The paper's rule is "NULL below l_1, the text rows from l_1 on"; per-layer
 *                retained sets of stage 2 are passed the same way.
 *   n_keep       host, [L] int32 (ignored where idx[l] is NULL).
 *   new_len      device out, [L] int32 or NULL: n_keep[l], or S_cap for untouched layers.
 *   Effect: for every (l, b, head) and for K and V, row i <- row idx[l][b][i], i < n_keep[l].
 *   Rows >= n_keep[l] are unspecified afterwards.  Positions that are not >= their rank or not
 *   below S_cap are skipped (never dereferenced).  dh * sizeof(dtype) must be a multiple of 16.
 *   workspace    device, at least metok_kv_compact_workspace_bytes() bytes, 16-byte aligned: progress
 *                flags of the row tiles, cleared by the call itself (its contents on entry do not
 *                matter).  After the call its first 32-bit word is 0; a 1 there means that a wait between
 *                two tiles of a slab expired and the cache was not compacted completely.  The waits are
 *                bounded (about 2^24 polls) and by construction always end much earlier; an expiry has
 *                never been observed and would mean that the GPU stopped running resident workgroups.
 * ------------------------------------------------------------------------------------------- */
METOK_API size_t metok_kv_compact_workspace_bytes(int L, int B, int Hkv, int64_t S_cap, int dh, int dtype);

METOK_API int metok_kv_compact(void* const* k_layers, void* const* v_layers, int L, int B, int Hkv,
                     int64_t S_cap, int dh, int dtype,
                     const int32_t* const* idx, const int32_t* n_keep, int32_t* new_len,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same compaction for a paged cache (Sec. 3.3).  Layer l holds K (resp. V) as a pool
 * [n_pages_pool, Hkv, page_size, dh] of `dtype`; logical row p of video b is slot p % page_size of page
 * page_table[b][p / page_size].
 *   page_table   device, [B, pages_per_seq] int32, shared by all layers; the pages of the table must be
 *                pairwise distinct (no page shared between or inside sequences), else rows alias and the
 *                in-place move is not defined.  Entries outside [0, n_pages_pool) are never dereferenced
 *                (rows that would touch them are skipped).
 *   idx, n_keep, new_len  as in metok_kv_compact, positions being logical rows below
 *                pages_per_seq * page_size.
 *   workspace    as in metok_kv_compact, sized by metok_kv_compact_workspace_bytes(L, B, Hkv,
 *                pages_per_seq * page_size, dh, dtype).
 * Afterwards the pages from ceil(n_keep[l] / page_size) on hold no live rows of layer l; the table itself is
 * not modified (page ids are shared by the layers, whose lengths now differ: the caller keeps one length
 * per layer, new_len, and may release a page once no layer needs it).
 */
METOK_API int metok_kv_compact_paged(void* const* k_pools, void* const* v_pools, int L, int B, int Hkv,
                           int64_t n_pages_pool, int page_size, int dh, int dtype,
                           const int32_t* page_table, int pages_per_seq,
                           const int32_t* const* idx, const int32_t* n_keep, int32_t* new_len,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Stage 3 on a paged cache by relinking pages (Sec. 3.3): the same compaction as metok_kv_compact_paged -- new
 * logical row i of (layer l, video b) holds old logical row idx[l][b][i] -- but instead of moving every kept
 * row, every layer gets a page table of its own:
 *   - a new page whose rows are exactly one whole old page (in order, from that page's first slot) takes over
 *     that page's physical page: nothing is copied;
 *   - the other new pages are filled by row copies into physical pages the sequence already owns (the k-th
 *     such new page takes the k-th old page, in table order, that no relinked page took over);
 *   - the old pages that are left are released.
 * With the paper's rule (from l_1 on only the text rows stay) and a visual span that ends on a page boundary
 * every new page is relinked: no row moves at all and all visual pages are released.
 *
 *   page_table_in   device, int32: the tables the rows are read through, [B, pages_per_seq] shared by all layers
 *                   (table_in_layer_stride = 0) or [L, B, pages_per_seq] (stride = B * pages_per_seq).  Pages of
 *                   the tables must be pairwise distinct inside a layer; entries outside [0, n_pages_pool) are
 *                   never dereferenced.
 *   len_in          host, [L] int32 or NULL (= pages_per_seq * page_size): rows each layer holds now; the old
 *                   pages of a layer are its first ceil(len_in[l] / page_size) table entries.
 *   idx, n_keep     as in metok_kv_compact: idx[l] [B, n_keep[l]] strictly ascending logical rows below
 *                   len_in[l]; idx[l] == NULL leaves the layer alone (its table is copied to the output).
 *   page_table_out  device out, [L, B, pages_per_seq] int32: new table of every layer and video; entries from
 *                   ceil(n_keep[l] / page_size) on are -1.  Must not overlap page_table_in.
 *   free_pages      device out, [L, B, pages_per_seq] int32: physical pages layer l releases for video b, in the
 *                   order of the old table, padded with -1;  n_free  device out, [L, B] int32: how many.
 *   rows_copied     device out, [L, B] int32: rows whose physical place changed (per kv head and for K and V the
 *                   same rows move).
 *   new_len         device out, [L] int32 or NULL.
 *   workspace       metok_kv_relink_paged_workspace_bytes(); its first word reports an expired wait as in
 *                   metok_kv_compact.
 */
METOK_API size_t metok_kv_relink_paged_workspace_bytes(int L, int B, int Hkv, int page_size, int pages_per_seq, int dh, int dtype);

METOK_API int metok_kv_relink_paged(void* const* k_pools, void* const* v_pools, int L, int B, int Hkv,
                          int64_t n_pages_pool, int page_size, int dh, int dtype,
                          const int32_t* page_table_in, int64_t table_in_layer_stride, int pages_per_seq,
                          const int32_t* len_in,
                          const int32_t* const* idx, const int32_t* n_keep,
                          int32_t* page_table_out, int32_t* free_pages, int32_t* n_free, int32_t* rows_copied,
                          int32_t* new_len,
                          void* workspace, size_t workspace_bytes, void* stream);

/* Test hook (not part of the method): number of polls after which a tile of the row mover gives a wait up.
 * 0 makes every wait that does not succeed at once expire, which exercises the error word of the workspace
 * without stalling anything; the default is 2^24. */
METOK_API int metok_debug_set_move_spin_limit(int polls);

/* ---------------------------------------------------------------------------------------------
 * Measurement helper (not part of the method): times one kernel family inside the library calls.
 * While armed on the calling thread, every launch of the named kernel is bracketed by hipEventRecord of
 * ev_begin and ev_end (hipEvent_t passed as void*, created by the caller with timing enabled) on the
 * stream of the call, so hipEventElapsedTime(ev_begin, ev_end) after the call is the duration of that
 * kernel alone, without the small planning kernels around it.  If a call launches the kernel more than
 * once the events bracket the last launch.  kernel == METOK_TRACE_NONE (or NULL events) disarms.  Do not
 * arm while a stream is being captured into a graph.
 * ------------------------------------------------------------------------------------------- */
enum {
    METOK_TRACE_NONE = 0,
    METOK_TRACE_FRAME_STATS = 1,        /* Eq. 4 / Eq. 5 pass over the frame features */
    METOK_TRACE_POOL = 2,               /* adaptive pooling pass */
    METOK_TRACE_FRAME_STATS_POOL2 = 3,  /* both in one pass (uniform stride 2) */
    METOK_TRACE_SEGMENT = 4,
    METOK_TRACE_PLAN = 5,
    METOK_TRACE_ROW_STATS = 6,          /* attention pass 1 (softmax statistics) */
    METOK_TRACE_COL_SUMS = 7,           /* attention pass 2 (probability mass per key) */
    METOK_TRACE_SELECT = 8,
    METOK_TRACE_WRITE_INDEX = 9,
    METOK_TRACE_GATHER_ROWS = 10,       /* hidden-state compaction */
    METOK_TRACE_MOVE_ROWS = 11          /* in-place row mover (KV compaction, in-place hidden compaction) */
};

METOK_API int metok_trace_kernel(int kernel, void* ev_begin, void* ev_end);

/* ---------------------------------------------------------------------------------------------
 * Measurement helper (not part of the method): a plain device-to-device copy kernel with the
 * same access width as the streaming kernels.  The bench uses it to calibrate the profiler's
 * HBM byte counters against a transfer of known size.  bytes must be a multiple of 16.
 * ------------------------------------------------------------------------------------------- */
METOK_API int metok_calib_copy(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* METOK_H */
