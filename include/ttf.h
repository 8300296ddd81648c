/*
 * ttf.h -- C ABI of the Temporal Token Fusion (TTF) pre-LLM compression pass for AMD
 * Instinct MI355X (gfx950).
 *
 * TTF (paper Section 3, "Temporal Token Fusion") takes the visual tokens of a clip,
 * X in R^{FN x C} viewed as [F, N=H*W, C], and
 *   1. picks an anchor frame a: the frame whose mean token has the largest cosine with the
 *      clip's mean token (anchor-frame-selection equation), or a caller-fixed frame
 *      (ablation A2: first / last frame);
 *   2. for every token (k,i) of every other ("source") frame searches the (2r+1)x(2r+1)
 *      neighbourhood of its grid cell in the anchor frame, clamped to the grid with
 *      duplicate cells counted once, for the anchor token of largest cosine similarity:
 *      best similarity s^(k,i) and anchor flat index dst(k,i) (pointwise matching with
 *      local window search: projection, flat-index map, similarity, arg max, s^/dst);
 *   3. fuses the token (drops it; the anchor token at dst stands for it) iff s^ > t, keeps
 *      it iff s^ <= t (threshold-gating equation);
 *   4. emits the compressed sequence X' = [N anchor rows ; P kept source rows in ascending
 *      flat order k*N+i] as bit-exact copies of input rows (no averaging), together with
 *      each row's original position triple (k, y, x) (stacked-X' equation, positional
 *      alignment: mask, gather of X and P) and the compressed length L' = N + P that
 *      cache-aware decode alignment needs.
 *
 * A batch holds B independent clips: every clip gets its own anchor, matches, mask and
 * L'; outputs are packed clip after clip.  (The paper's tied-batch rule -- one offset from
 * the batch-mean similarity, keep = union over the batch -- is a different mode, offered by
 * ttf_compress_tied.)
 *
 * General conventions
 *   - All data pointers are DEVICE pointers unless a field says HOST.  Every buffer is
 *     owned by the caller, before, during and after the call.  The library allocates and
 *     frees no device memory.
 *   - Work is enqueued on the caller's stream and the call returns without synchronising.
 *     Buffers must stay alive until the stream has drained.  Calls that share a workspace
 *     must be ordered by the caller (same stream, or events).
 *   - Every function returns a ttf_status.  On any status other than TTF_OK no kernel has
 *     been launched and no output has been written, except TTF_ERR_HIP, which reports a
 *     failed launch or copy part-way through the sequence (outputs are then undefined).
 *   - Same inputs give bit-identical outputs on every call (no floating-point atomics, fixed
 *     reduction orders).
 *   - Input values are not scanned.  A candidate whose cosine is NaN (a NaN or infinite entry in
 *     the source token or in that anchor token) wins no comparison.  A source token all of whose
 *     candidates are like that is kept and reports best_sim = -inf, best_idx = -1, fuse_map = -1.
 *     A NaN or infinite entry anywhere in a clip makes every anchor score NaN; the automatic
 *     rule then picks frame 0.  Dot products and squared norms are accumulated in fp32: token rows
 *     whose squared norm overflows fp32 (entries around 1e17 and beyond) behave like rows with
 *     infinite entries.  Only an exactly zero norm gives cosine 0.
 */
#ifndef TTF_H
#define TTF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TTF_OK = 0,
    TTF_ERR_INVALID_ARG = 1,          /* NULL required pointer, size <= 0, r < 0, non-finite t, ... */
    TTF_ERR_UNSUPPORTED = 2,          /* unknown dtype, misaligned features / tokens_out            */
    TTF_ERR_WORKSPACE_TOO_SMALL = 3,  /* workspace_bytes < ttf_workspace_size()                     */
    TTF_ERR_HIP = 4                   /* a HIP call failed; see ttf_last_hip_error()                */
} ttf_status;

typedef enum { TTF_BF16 = 0, TTF_F32 = 1 } ttf_dtype;

typedef enum { TTF_ANCHOR_AUTO = 0, TTF_ANCHOR_FIXED = 1 } ttf_anchor_mode;

/* Problem description.  B*F*ceil(H*W/64)*64 (the token count with every frame rounded up to whole
 * 64-token groups) must be below 2^25 = 33 554 432, and H*W below 2^31. */
typedef struct {
    int32_t B, F, H, W, C;    /* clips, frames, token-grid height and width, channels; all >= 1 */
    int32_t dtype;            /* ttf_dtype of `features` and `tokens_out`                        */
    int32_t r;                /* search radius >= 0, window (2r+1)^2; r >= max(H,W)-1 = whole grid */
    float   t;                /* cosine threshold; fused iff s^ > t (strict).  Any finite value.  */
    int32_t anchor_mode;      /* ttf_anchor_mode                                                  */
    int32_t anchor_index;     /* FIXED only: frame in [-F, F); negative counts from the last     */
} ttf_params;

/*
 * Outputs.  cap = B*F*H*W rows is the capacity the row-indexed buffers must have; rows at
 * and beyond row_offsets[B] are left untouched.  N = H*W.
 */
typedef struct {
    void*    tokens_out;    /* [cap, C] dtype.  Clip b owns rows row_offsets[b] .. row_offsets[b+1)-1:
                               first its N anchor rows, then its kept source rows (stacked-X' equation). */
    int32_t* pos_ids;       /* [3, cap] planes k (frame), y, x of every output row (plane stride cap). */
    int32_t* src_index;     /* [cap]    flat index k*N+i inside its clip of every output row (I_keep). */
    int32_t* row_offsets;   /* [B+1]    exclusive prefix sum of kept_count.                            */
    int32_t* kept_count;    /* [B]      L'_b = N + P_b.                                                */
    int32_t* anchor_index;  /* [B]      anchor frame chosen (or given) per clip.                       */
    int32_t* fuse_map;      /* [B,F,N]  dst(k,i) in [0,N) if the token was fused, else -1
                                        (anchor-frame tokens: -1).                                     */
    float*   best_sim;      /* [B,F,N]  s^(k,i); 1.0f on anchor-frame tokens.  May be NULL.            */
    int32_t* best_idx;      /* [B,F,N]  dst(k,i) for every source token whether fused or not;
                                        i on anchor-frame tokens.  May be NULL.                        */
    int32_t* host_counts;   /* HOST, pinned, [2B+1]: kept_count[0..B) then row_offsets[0..B]; filled by
                               an asynchronous copy on the stream.  May be NULL.                       */
} ttf_outputs;

/* Bytes of device workspace ttf_compress needs for these sizes (depends on B,F,H,W,C and dtype only).
 * The workspace must be 256-byte aligned.  INVALID_ARG on bad sizes or NULL pointers. */
ttf_status ttf_workspace_size(const ttf_params* params, size_t* bytes);

/*
 * The whole pass (Section 3: anchor frame selection, pointwise matching with local window
 * search, threshold gating and token compression, positional alignment).
 *   features   DEVICE [B,F,H,W,C] contiguous, dtype per params, 16-byte aligned; read only.
 *   workspace  DEVICE scratch of at least ttf_workspace_size() bytes, 256-byte aligned; its
 *              contents on entry do not matter and are garbage afterwards.
 *   out        see ttf_outputs; all but the three optional fields are required.
 *   hip_stream hipStream_t (NULL = the default stream).
 * Errors: INVALID_ARG (NULL params/features/workspace/out or required output, a size < 1,
 * more than 2^25 tokens (frames rounded up to 64), r < 0, t not finite, anchor_index outside [-F,F) in FIXED mode, unknown
 * anchor_mode), UNSUPPORTED (unknown dtype; features, tokens_out or workspace misaligned),
 * WORKSPACE_TOO_SMALL, HIP.  Any C, grid and radius work.  Fast paths: bf16 and fp32 input with
 * C % 32 == 0 and r <= 2 runs the window search on the matrix cores (fp32 as three bf16 pieces
 * per value, 24 significant bits) (any grid; grids exactly 16
 * or 32 tokens wide with H*W % 64 == 0 are the best case); rows whose byte length is a multiple
 * of 16 are read and copied with 16-byte accesses.
 */
ttf_status ttf_compress(const ttf_params* params, const void* features,
                        void* workspace, size_t workspace_bytes,
                        const ttf_outputs* out, void* hip_stream);

/*
 * ttf_compress for callers that cannot allocate device memory or hand over a workspace: code
 * running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, outputs, kernels and errors as ttf_compress, but the workspace is a fixed array of
 * TTF_STATIC_WORKSPACE_BYTES that lives in the library's device image (every GPU the library is
 * used on holds its own copy from the first use until the process ends).  The call allocates and
 * frees nothing.
 *   - Problems whose ttf_workspace_size() exceeds TTF_STATIC_WORKSPACE_BYTES are refused with
 *     TTF_ERR_WORKSPACE_TOO_SMALL before anything is launched.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race and give undefined outputs; order them on one stream or with events.
 *     The array keeps the previous call's contents; nothing in it needs to start at zero.
 *   - The first call on a device looks up the array's device address (hipGetSymbolAddress); make
 *     that call outside any stream capture.  TTF_ERR_HIP if the lookup fails.
 */
#define TTF_STATIC_WORKSPACE_BYTES (16u << 20)
ttf_status ttf_compress_static(const ttf_params* params, const void* features,
                               const ttf_outputs* out, void* hip_stream);

/*
 * One segment of a stream (the streaming use sketched in Discussion D3): video arrives in pieces, and
 * each piece is matched not against a frame of its own but against the frame that closed the
 * previous piece, so that earlier context never has to be encoded again.
 * Every one of the F frames of `features` is a source frame matched against `anchor_frame`; the
 * output holds only the preserved source rows, in ascending flat order k*N+i, so it is what
 * ttf_compress gives for the (F+1)-frame clip [anchor_frame ; features] with its anchor fixed to
 * frame 0, without the N anchor rows.  To chain segments pass the previous segment's last frame
 * (features + (F-1)*N*C elements of each clip, gathered to [B,H,W,C]) as the next anchor_frame.
 *   anchor_frame  DEVICE [B,H,W,C] dtype, 16-byte aligned, read only; may alias no output
 *   frame_offset  added to the temporal plane of pos_ids: frame k of the segment reports
 *                 frame_offset + k (its index in the stream); frame_offset + F must fit int32
 *   out           as for ttf_compress, except: kept_count[b] = P_b (no anchor rows),
 *                 anchor_index[b] = -1, best_idx / fuse_map index cells of anchor_frame,
 *                 src_index = k*N+i inside the segment
 * params->anchor_mode and anchor_index are not used.  Errors as for ttf_compress; a NULL or
 * misaligned anchor_frame is INVALID_ARG / UNSUPPORTED.  ttf_restore_map does not apply to
 * segment outputs (their anchor rows live in an earlier segment's output).
 */
ttf_status ttf_compress_segment(const ttf_params* params, const void* features, const void* anchor_frame,
                                int32_t frame_offset, void* workspace, size_t workspace_bytes,
                                const ttf_outputs* out, void* hip_stream);

/*
 * Tied-batch mode (Section 3, the remark on B > 1 after the s^/dst equations, and the gating
 * paragraph): the B elements are treated as views of one sequence.  For every source position the
 * candidate cell is scored by the average of the B elements' cosines and one cell is picked for all of
 * them; each element reports its own cosine at that shared cell; a position is dropped only when
 * every element's cosine exceeds t.  All B elements therefore keep the same index set and the
 * output is rectangular.  Choices the text leaves open: the anchor frame is
 * shared -- under the automatic rule the frame with the largest batch-mean anchor score (lowest
 * k on ties), else the fixed frame; the mean is the arithmetic mean of the B cosines of one
 * candidate cell; first maximum in row-major offset order.  Radius r <= 3 (UNSUPPORTED beyond).
 *
 * cap = F*N rows.
 */
typedef struct {
    void*    tokens_out;    /* [B, cap, C] dtype: element b's rows start at row b*cap; rows
                               0..L'-1 of every element are valid, the rest untouched            */
    int32_t* pos_ids;       /* [3, cap] planes k, y, x of the shared rows                         */
    int32_t* src_index;     /* [cap] flat k*N+i of the shared rows                                */
    int32_t* kept_count;    /* [1] L' = N + P                                                     */
    int32_t* anchor_index;  /* [B] every entry = the shared anchor frame                          */
    int32_t* fuse_map;      /* [F,N] shared: dst(k,i) if every element has s^ > t, else -1        */
    float*   best_sim;      /* optional [B,F,N]: s^ of every element at the shared offset (1 on
                               anchor rows)                                                      */
    int32_t* best_idx;      /* optional [F,N]: shared dst(k,i) (i on anchor rows)                 */
    float*   mean_sim;      /* optional [F,N]: the maximal batch-mean similarity (1 on anchor
                               rows)                                                             */
    int32_t* host_counts;   /* optional HOST pinned [1]: copy of kept_count                       */
} ttf_tied_outputs;

/* Workspace bytes of ttf_compress_tied (depends on B,F,H,W,C,dtype and r). */
ttf_status ttf_tied_workspace_size(const ttf_params* params, size_t* bytes);

/* Arguments and errors as for ttf_compress; workspace of ttf_tied_workspace_size() bytes. */
ttf_status ttf_compress_tied(const ttf_params* params, const void* features, void* workspace,
                             size_t workspace_bytes, const ttf_tied_outputs* out, void* hip_stream);

/*
 * Restoration (Discussion D4, token restoration through the map dst(k,i) of the matching step).
 *
 * ttf_restore_map: for every original token, the row of the compressed sequence that stands for
 * it -- its own row if it was retained (anchor tokens included), the anchor row
 * row_offsets[b] + dst(k,i) if it was fused.
 *   fuse_map, row_offsets, src_index   DEVICE, as written by ttf_compress for the same params
 *   restore_map                        DEVICE int32 [B,F,N], every entry written
 * ttf_restore: the full layout rebuilt from the compressed rows,
 *   restored[b,k,i,:] = tokens[restore_map[b,k,i], :]   (bit-exact row copies).
 *   tokens       DEVICE [rows, C] dtype, 16-byte aligned (ttf_compress's tokens_out, or rows of the
 *                same shape computed from it, e.g. after further layers)
 *   rows         number of valid rows in `tokens`; map entries outside [0, rows) give a zero row
 *   restored     DEVICE [B,F,N,C] dtype, 16-byte aligned
 * Errors: INVALID_ARG (NULL pointer, bad sizes, rows < 0), UNSUPPORTED (dtype, alignment), HIP.
 */
ttf_status ttf_restore_map(const ttf_params* params, const int32_t* fuse_map, const int32_t* row_offsets,
                           const int32_t* src_index, int32_t* restore_map, void* hip_stream);
ttf_status ttf_restore(const ttf_params* params, const void* tokens, int64_t rows,
                       const int32_t* restore_map, void* restored, void* hip_stream);

/*
 * Cache-aware decode alignment (Section 3; prefill-length and decode-position equations), host
 * arithmetic on HOST integers: with L' compressed visual tokens and T text tokens the cache holds
 * L_pre = L' + T pairs; decode step l = 0,1,... gets position L_pre + l and an attention mask of
 * length L_pre + l + 1.  Output pointers may be NULL.  INVALID_ARG on a negative input.
 */
ttf_status ttf_decode_alignment(int64_t l_prime, int64_t text_tokens, int64_t step,
                                int64_t* l_pre, int64_t* position, int64_t* mask_length);

/*
 * Video-adaptive threshold (Discussion D1: t calibrated from the empirical distribution of the
 * best-match similarities of the current clip).  The paper leaves the rule open; this library
 * uses an order statistic.  For a requested fused fraction phi in [0,1] of the M = (F-1)*N source
 * tokens of a clip:  rank = clamp(ceil((1 - phi) * M), 1, M)  (formed in double precision), and
 * thresholds[b] = the rank-th smallest s^ of clip b.  Tokens strictly above it fuse, so at most
 * floor(phi*M) do, exactly that many when the values next to the rank are distinct.  F = 1 gives
 * thresholds[b] = 1.  Values are ordered as real numbers (-0 just below +0; a NaN with the sign
 * bit clear sorts above +inf, with it set below -inf).  Outputs of ttf_compress_segment
 * (anchor_index[b] = -1) work too: all F frames are then source frames, M = F*N.
 *   best_sim, anchor_index   DEVICE, as written by ttf_compress (best_sim requested there)
 *   thresholds               DEVICE float [B]
 * Errors: INVALID_ARG (NULL pointer, bad sizes, phi outside [0,1] or NaN), HIP.
 */
ttf_status ttf_select_threshold(const ttf_params* params, const float* best_sim,
                                const int32_t* anchor_index, float fused_fraction,
                                float* thresholds, void* hip_stream);

/*
 * Gate, offsets and row emission redone from stored matches (threshold-gating equation and the
 * compaction that follows it), without a window search: the result is what ttf_compress gives
 * for the same features with clip b gated at thresholds[b] (or at params->t for every clip when
 * thresholds is NULL) and its anchor fixed to anchor_index[b].
 *   out->anchor_index, out->best_sim, out->best_idx   INPUTS here: DEVICE arrays a previous
 *       ttf_compress on the same features and params (r included) wrote; all three required
 *   out->fuse_map, tokens_out, pos_ids, src_index, row_offsets, kept_count, host_counts   written
 *   thresholds   DEVICE float [B] or NULL
 * params->anchor_mode / anchor_index / r are not used.  Workspace as for ttf_compress.
 */
ttf_status ttf_regate(const ttf_params* params, const void* features, const float* thresholds,
                      void* workspace, size_t workspace_bytes, const ttf_outputs* out, void* hip_stream);

/* Static, NUL-terminated description of a status code (never NULL). */
const char* ttf_status_string(ttf_status status);

/* hipError_t (as int) behind the calling thread's last TTF_ERR_HIP; 0 if none. */
int ttf_last_hip_error(void);

/*
 * How ttf_compress evaluates the automatic anchor rule (the anchor-frame-selection equation needs the
 * mean of every frame, i.e. a pass over the whole input before the search can start).
 *   two-pass      frame sums over the whole input, then the search.
 *   speculative   the rule is first evaluated on 256 of the C channels (four runs of 64 channels,
 *                 run j starting at channel (2j+1)*C/8 rounded down to a multiple of 64).  A clip
 *                 whose guessed best frame beats the runner-up by at least 0.1 in that cosine is
 *                 searched against the guess at once, the search adds up the exact sums of every
 *                 frame on the side, and the exact rule is evaluated from them afterwards: it
 *                 confirms the guess, or the clip is searched again against the exact anchor.
 *                 A clip without a clear guess sits out the first search and takes the two-pass
 *                 route together with the refuted clips.  Outputs are those of the
 *                 exact rule in every case; only the time differs (one pass over the input instead
 *                 of two when the guesses hold, one extra search for a clip whose trusted guess
 *                 was wrong).
 *                 Available for bf16 input on grids whose rows fill at least 70 % of the 32-cell
 *                 strips the search cuts them into (12..16, 23..32, 45..64, ... columns; any
 *                 height), C % 128 == 0, C >= 1024, r <= 2, F >= 2, automatic anchor.
 * mode  0 (default): speculative for inputs of 256 MiB and more in clips of at most 128 frames
 *       where available, else two-pass;
 *       1: speculative wherever available;  -1: always two-pass.
 * Process-wide; takes effect for calls made after it returns.  INVALID_ARG for other values.
 */
ttf_status ttf_set_speculation(int mode);

/*
 * Which window-search kernels a problem takes (Section 3, "Pointwise Matching with Local Window
 * Search"): a host-side query, no GPU work.  Results never depend on the route, only the time does.
 *   params  host; checked as in ttf_compress.
 *   route   host, out: one of the TTF_ROUTE_* values.
 * Errors: INVALID_ARG (NULL pointer, bad params), UNSUPPORTED (unknown dtype).
 */
#define TTF_ROUTE_GENERAL      0   /* wave-per-token kernels (any C, any radius) */
#define TTF_ROUTE_MFMA_BF16    1   /* matrix cores, bf16, grid exactly 16 or 32 wide with whole keep words */
#define TTF_ROUTE_MFMA_BF16_PADDED 2   /* matrix cores, bf16, any other grid (tile rows padded to 16 columns) */
#define TTF_ROUTE_MFMA_F32     3   /* matrix cores, fp32 as three bf16 pieces per value, any grid */
ttf_status ttf_search_route(const ttf_params* params, int* route);

/*
 * Per-stage timing, for benchmarks.  Stages, in launch order:
 *   0 frame sums (speculative route: over the guess channels only)   1 anchor scores (two-pass
 *     route only)   2 anchor choice + norms   3 window search + gate
 *   4 anchor verification (speculative route only: exact rule from the search's sums, repeated
 *     search of refuted clips)   5 offsets scan   6 row emission
 * ttf_profile_enable(slots), 1 <= slots <= TTF_PROFILE_MAX_SLOTS, makes every following
 * ttf_compress on the calling thread record HIP events around each stage on the call's
 * stream; successive calls use `slots` event sets round-robin (created once, reused), so up to
 * `slots` calls can be in flight or waiting to be read.  ttf_profile_enable(0) turns it off.
 * Enabling resets the call counter.  ttf_profile_read(call, ms_out, n) waits for profiled call
 * number `call` (0-based since enabling; must be one of the last `slots` calls) and writes its
 * stage durations in milliseconds to ms_out[0..min(n, TTF_NUM_STAGES)); stages that did not
 * run report ~0.  Event records sit between the kernels; profiling is off by default.
 * This is a measurement hook, not part of the pass: it is the one place where the library creates
 * HIP objects (events, at most TTF_PROFILE_MAX_SLOTS sets per thread, created by the first
 * ttf_profile_enable that needs them and kept until the process ends); ttf_compress and
 * ttf_compress_segment record into them only while profiling is enabled on the calling thread,
 * the other entry points never do.  Do not enable it around a stream capture.
 * Errors: INVALID_ARG (bad slot count, NULL, call not available), HIP.
 */
#define TTF_NUM_STAGES 7
#define TTF_PROFILE_MAX_SLOTS 256
ttf_status ttf_profile_enable(int slots);
ttf_status ttf_profile_read(int call, float* ms_out, int n);
const char* ttf_stage_name(int stage);

#ifdef __cplusplus
}
#endif
#endif /* TTF_H */
