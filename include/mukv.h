/*
 * mukv.h -- C ABI of the MuKV hot path for AMD MI355X (gfx950).
 *
 * MuKV ("Multi-Grained KV Cache Compression for Long Streaming Video
 * Question-Answering") keeps a compact multi-grained KV cache of a video stream
 * offline and retrieves question-relevant parts of it online.  This library is
 * the data-parallel part of that method, as HIP kernels:
 *
 *   offline, per chunk of frames  : mukv_compress_chunk   (Sec. 3.3, Eq. 1-5)
 *   online, per batch of questions: mukv_retrieve          (Sec. 3.4, Eq. 6-8)
 *                                   mukv_gather_kv         (Sec. 3.5, Eq. 9 context)
 *
 * The Video-LLM itself is not part of the library: the caller hands over the
 * K/V tensors of a prefill, the scoring layer's query states (or the attention
 * it already computed) and, online, the question's query states.
 *
 * General rules
 *  - Every function returns MUKV_OK (0) or a negative mukv_status.  No C++
 *    exception crosses this boundary.  Arguments are validated on the host
 *    before anything is launched, so a failed call has no device side effects.
 *  - "device" pointers are HIP device pointers valid on the context's device;
 *    "host" pointers are ordinary process memory.  The caller owns every buffer
 *    it passes in; the context owns the cache.  Inputs may be reused as soon as
 *    the stream has passed the call (batch_chunks and overlap_copy lengthen
 *    that for mukv_compress_chunk: see there).
 *  - Work is enqueued on the hipStream_t passed as `stream` (void*, NULL = the
 *    default stream) and is never synchronised by the library.  Calls on one
 *    context must be issued in stream order; the context is not thread-safe.
 *  - After mukv_create no device memory is allocated or freed until
 *    mukv_destroy.  A call makes the context's device current while it runs
 *    and gives the caller's current device back.
 *  - MUKV_ERR_HIP from a call that launches kernels leaves the cache in an
 *    unspecified state: destroy the context.  Every other error leaves it as
 *    it was.
 *  - Inputs must be finite.  Non-finite values give unspecified selections.
 */
#ifndef MUKV_H
#define MUKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mukv_ctx mukv_ctx;

typedef enum mukv_status {
    MUKV_OK = 0,
    MUKV_ERR_INVALID_ARG = -1, /* null pointer, value out of range            */
    MUKV_ERR_SHAPE = -2,       /* sizes inconsistent with the configuration   */
    MUKV_ERR_CAPACITY = -3,    /* more frames / questions than reserved       */
    MUKV_ERR_UNSUPPORTED = -4, /* shape or alignment no kernel is built for   */
    MUKV_ERR_HIP = -5          /* a HIP runtime call failed                   */
} mukv_status;

typedef enum mukv_dtype { MUKV_BF16 = 0, MUKV_F32 = 1 } mukv_dtype;

/* Retrieval strategies compared in the paper's retrieval ablation (Sec. 4.3):
 * SEMI is the method of Sec. 3.4 (parallel stage 1 + Eq. 8 rerank), PARALLEL
 * returns the stage-1 ranking, HIER searches frames only inside the chosen
 * segments with the question as query at both levels. */
typedef enum mukv_mode { MUKV_SEMI = 0, MUKV_HIER = 1, MUKV_PARALLEL = 2 } mukv_mode;

typedef enum mukv_order { MUKV_TEMPORAL = 0, MUKV_AS_GIVEN = 1 } mukv_order;

typedef enum mukv_att_path { MUKV_ATT_AUTO = 0, MUKV_ATT_GENERIC = 1, MUKV_ATT_MFMA = 2 } mukv_att_path;

/*
 * Static description of the stream and the cache (Sec. 3.2-3.3 notation:
 * L layers, P tokens per frame, F frames per segment, S super-patches per
 * frame, rho keep ratio, alpha signal mix).
 */
enum { MUKV_FREQ_FEATURE = 0, MUKV_FREQ_TOKEN = 1 };

typedef struct mukv_config {
    int32_t n_layers;               /* L                                               */
    int32_t n_q_heads;              /* H_q, a multiple of n_kv_heads                   */
    int32_t n_kv_heads;             /* H_kv                                            */
    int32_t head_dim;               /* D: a power of two in 16..128                    */
    int32_t tokens_per_frame;       /* P, 1..256: the unit of Eq. 4.  257..8192 declares
                                       a unit of several frames (up to a segment, Sec. 3.3
                                       at the coarsest granularity) that is ranked as one:
                                       S can then count its frames; alpha > 0 needs  
                                       att_signal and freq_axis must be FEATURE           */
    int32_t frames_per_segment;     /* F >= 1                                          */
    int32_t superpatches_per_frame; /* S, 1..P: index-contiguous groups of floor(P/S)
                                       tokens, the last one takes the remainder        */
    int32_t dtype;                  /* mukv_dtype of K, V, Q payloads                  */
    double keep_ratio;              /* rho in (0,1]; kappa = floor(rho*P + 1e-9) >= 1  */
    double alpha;                   /* weight of the attention signal in Eq. 4, [0,1]  */
    int32_t causal;                 /* 1: query i attends keys j <= i inside its frame */
    int32_t score_layer;            /* layer that supplies Eq. 1-3, 5-7; -1 = last     */
    int32_t max_frames;             /* capacity of the cache in frames                 */
    int32_t max_chunk_frames;       /* largest n_frames of one mukv_compress_chunk     */
    int32_t max_questions;          /* largest batch of one mukv_retrieve / gather     */
    int32_t device_id;              /* HIP device ordinal                              */
    int32_t att_path;               /* mukv_att_path; AUTO picks MFMA when supported   */
    int32_t batch_chunks;           /* 0 or 1: every mukv_compress_chunk enqueues its kernels at
                                       once.  N > 1 (at most 64): the library gathers N chunks
                                       and processes them with one chain of launches; see
                                       mukv_compress_chunk for what that asks of the caller    */
    double refine_margin;           /* frames whose selection margin (gap between the
                                       last kept and first dropped fused score) is
                                       below this are re-scored in fp64 before the
                                       keep; < 0 = library default, 0 = never          */
    int32_t overlap_copy;           /* 0: a call that enqueues kernels enqueues all of them.
                                       1: the keep of a batch runs on a stream of the library's
                                       own beside the next batch's kernels, and the copy of its
                                       kept rows is put off until the batch after next arrives
                                       and then shares ONE launch with that batch's signals
                                       (HBM-bound and arithmetic-bound workgroups side by side on
                                       every compute unit).
                                       See mukv_compress_chunk for what that asks of the caller */
    int32_t freq_axis;              /* axis of the transform in Eq. 2, which the text leaves open:
                                       MUKV_FREQ_FEATURE (0, default) along the D features of each
                                       token's key; MUKV_FREQ_TOKEN (1) along the P tokens of the
                                       frame, feature by feature (row m of the signal is then the
                                       m-th frequency of the frame; rows m and P-m are equal) */
} mukv_config;

/* Element strides (not bytes) of a [layer][head][token][dim] tensor; dim is
 * contiguous.  `layer` is ignored for the single-layer q_last tensor. */
typedef struct mukv_strides {
    int64_t layer;
    int64_t head;
    int64_t token;
} mukv_strides;

/* Optional per-chunk outputs of the scoring stage, device float [n_frames][P]
 * each, any may be NULL: raw Eq. 1 signal, raw Eq. 3 signal, fused Eq. 4 score
 * (as used for the keep, i.e. after fp64 re-scoring where that happened). */
typedef struct mukv_signals_out {
    float *att;
    float *fft;
    float *fused;
} mukv_signals_out;

typedef struct mukv_retrieve_params {
    int32_t mode;             /* mukv_mode                                            */
    int32_t k_seg;            /* k_g at segment level, 1..512                         */
    int32_t k_frame;          /* k_g at frame level, 1..512                           */
    int32_t n_global;         /* N segments averaged into the global query; 0 = k_seg */
    int32_t n_visible_frames; /* question timestamp: only frames < this are searched;
                                 < 0 = every ingested frame                           */
    int32_t reserved0;
    double lambda_frame;      /* lambda_g of Eq. 8 for frames (segments use 0)        */
} mukv_retrieve_params;

/* Read-only view of the context's state; device pointers stay valid until
 * mukv_destroy.  Tables are valid for frames < n_frames once the stream has
 * passed the calls that produced them. */
typedef struct mukv_state {
    int64_t n_frames;          /* frames submitted (tables cover them once the gathered
                                  chunks have been flushed and the stream has run)    */
    int64_t n_segments;        /* ceil(n_frames / F); the last may be partial         */
    int64_t n_kept_tokens;     /* n_frames * kappa                                    */
    int64_t store_token_capacity; /* max_frames * kappa                               */
    int32_t kappa;
    int32_t c_kv;              /* H_kv * D                                            */
    const void *store_k;       /* [L][H_kv][store_token_capacity][D], payload dtype   */
    const void *store_v;
    const int32_t *kept_idx;   /* [max_frames][kappa] kept positions, ascending       */
    const float *rep_frame_k;  /* [max_frames][c_kv] Eq. 5 block keys, float32        */
    const float *rep_frame_v;  /* same pooling applied to V                           */
    const float *rep_patch_k;  /* [max_frames*S][c_kv]; zero rows where count is 0    */
    const float *rep_patch_v;
    const int32_t *cnt_patch;  /* [max_frames*S] kept tokens in each super-patch      */
    const float *rep_seg_k;    /* [ceil(max_frames/F)][c_kv]                          */
    const float *rep_seg_v;
    const float *margin;       /* [max_frames] selection margin of each frame         */
    const int32_t *refined;    /* [max_frames] 1 where the fp64 re-scoring ran        */
    int32_t patch_cap;         /* most kept tokens a super-patch can hold:
                                  min(kappa, longest super-patch)                     */
} mukv_state;

/* Allocates the cache on cfg->device_id.  *out is set only on success. */
int mukv_create(const mukv_config *cfg, mukv_ctx **out);

/* Frees everything the context owns.  The caller must have synchronised the
 * streams it used.  NULL is accepted. */
int mukv_destroy(mukv_ctx *ctx);

/* Forgets the stream (n_frames = 0, gathered chunks and a copy that was put off
 * are dropped) without freeing memory.  Kernels of earlier calls may still be
 * running: later calls on the same stream are ordered after them as usual. */
int mukv_reset(mukv_ctx *ctx);

/* Enqueues the kernels of the chunks gathered so far (batch_chunks > 1) and, with
 * overlap_copy, the copy that was put off; the stream of the last compress call is
 * then ordered after everything the library has enqueued.  A no-op when there is
 * neither.  Does not synchronise the host. */
int mukv_flush(mukv_ctx *ctx);

/*
 * Offline step for n_frames new frames (Sec. 3.3).  For every frame: Eq. 1
 * attention received (from q_last and the scoring layer's K, softmax over the
 * frame's own keys, scale 1/sqrt(D)) or the caller's att_signal; Eq. 2-3
 * frequency score (length-D DFT of each token's key per KV head, mean
 * magnitude); Eq. 4 min-max fusion; keep of the kappa best tokens (ties: lowest
 * position; emitted ascending); copy of the kept K and V rows of all L layers
 * into the store; Eq. 5 block keys (and the same means of V) per super-patch,
 * frame and segment.  Frames are appended at the context's current time.
 *
 *   k, v        device, logical [L][H_kv][n_frames*P][D] with kv_strides
 *   q_last      device, logical [H_q][n_frames*P][D] with q_strides, or NULL
 *   att_signal  device float [n_frames][P], or NULL
 *               alpha > 0 needs exactly one of q_last / att_signal;
 *               alpha == 0 ignores both
 *   sig         optional outputs, may be NULL
 *
 * With batch_chunks > 1 the call only records the chunk until batch_chunks
 * chunks are gathered (or mukv_flush, mukv_retrieve or mukv_gather_kv is
 * called); the kernels for all of them are then enqueued together on the
 * stream the chunks were submitted with.  The caller must keep the chunk's
 * input buffers (and `sig` outputs) alive and unchanged until the stream has
 * passed that later call.  A chunk whose stream, strides or attention source
 * differ from the gathered ones flushes them first.  Capacity errors are
 * reported by the call that submits the chunk, launch errors by the call that
 * flushes.
 *
 * With overlap_copy = 1 the rows of a batch are copied out of the input buffers
 * only by the SECOND call after it that enqueues compress kernels, or by a
 * mukv_flush, retrieve, gather, attend or snapshot call.  The inputs (and `sig`
 * outputs) of a batch must then stay alive and unchanged until the stream has
 * passed that call.  Results are the same bit for bit.
 *
 * Errors: INVALID_ARG (null k/v, missing or doubled attention source),
 * SHAPE (n_frames < 1), CAPACITY (n_frames > max_chunk_frames or the cache is
 * full), UNSUPPORTED (strides or pointers not 16-byte aligned, a query
 * token stride of 16 MiB or more, or q_last for units of more than 256 tokens).
 */
int mukv_compress_chunk(mukv_ctx *ctx, const void *k, const void *v, const mukv_strides *kv_strides,
                        const void *q_last, const mukv_strides *q_strides, const float *att_signal,
                        int32_t n_frames, void *stream, const mukv_signals_out *sig);

/*
 * Online retrieval for a batch of B questions (Sec. 3.4).  Eq. 6 mean of each
 * question's query tokens; Eq. 7 cosine with every visible segment and frame
 * key (keys expanded over their query-head group); stage-1 top-2k; global query
 * = mean of the top-N segment keys; Eq. 8 rerank of the frame candidates;
 * final top-k.  Scores are evaluated in fp64 from the float32 key tables.
 *
 *   q_tokens   device, [sum of lengths][H_q][D] dense, payload dtype
 *   q_offsets  device int32 [B+1], question b owns tokens q_offsets[b] ..
 *              q_offsets[b+1]-1
 *   outputs    device; indices in rank order (best first; ties: lowest index),
 *              padded with -1 / score 0 when fewer blocks are visible:
 *              seg_idx_out [B][k_seg], seg_score_out [B][k_seg] (Eq. 7),
 *              frame_idx_out [B][k_frame], frame_score_out [B][k_frame]
 *              (Eq. 8 score in SEMI mode, Eq. 7 otherwise).  Score outputs may
 *              be NULL.
 *
 * Errors: INVALID_ARG, CAPACITY (B > max_questions), UNSUPPORTED (k > 512).
 */
int mukv_retrieve(mukv_ctx *ctx, const void *q_tokens, const int32_t *q_offsets, int32_t B,
                  const mukv_retrieve_params *params, int32_t *seg_idx_out, float *seg_score_out,
                  int32_t *frame_idx_out, float *frame_score_out, void *stream);

/*
 * The same search with the super-patch as the fine level (the patch granularity
 * of Sec. 3.2 / 3.4): Eq. 7 against every visible super-patch key, stage-1
 * top-2k, Eq. 8 against the global query of the top-N segments, final top-k.
 * params->k_frame and params->lambda_frame are read as k_g and lambda_g of the
 * patch level; k_seg, n_global, mode and n_visible_frames keep their meaning
 * (HIER: super-patches inside the k_seg chosen segments).  A patch is named
 * frame * S + s.  Super-patches without a kept token are never returned.
 *
 *   patch_idx_out    device int32 [B][k_frame], rank order, padded with -1
 *   patch_score_out  device float [B][k_frame] or NULL
 *
 * Errors as for mukv_retrieve.
 */
int mukv_retrieve_patches(mukv_ctx *ctx, const void *q_tokens, const int32_t *q_offsets, int32_t B,
                          const mukv_retrieve_params *params, int32_t *patch_idx_out, float *patch_score_out,
                          void *stream);

/*
 * The search for questions asked at different times (the streaming setting of
 * Sec. 3.1: a question is answered from the content before its timestamp).
 * Question b sees frames < n_visible[b] (device int32 [B]; a negative value or
 * one past the ingested frames means all of them); params->n_visible_frames
 * is ignored.  A segment cut by a question's timestamp is re-pooled from its
 * visible frames for that question.  level 0: frames are the fine level
 * (mukv_retrieve), 1: super-patches (mukv_retrieve_patches).  seg_idx_out /
 * seg_score_out may be NULL.  Everything else as in mukv_retrieve.
 */
int mukv_retrieve_at(mukv_ctx *ctx, const void *q_tokens, const int32_t *q_offsets, const int32_t *n_visible, int32_t B,
                     const mukv_retrieve_params *params, int32_t level, int32_t *seg_idx_out, float *seg_score_out,
                     int32_t *fine_idx_out, float *fine_score_out, void *stream);

/*
 * Packs the stored K,V of the selected super-patches of each question into a
 * dense decode context: for every patch the kept rows whose position lies in it
 * (a dense run inside its frame's rows), patches in ascending id (MUKV_TEMPORAL)
 * or list order, rows back to back.
 *
 *   patch_idx     device int32 [B][k_patch]; -1 and ids >= n_frames*S are skipped
 *   k_out, v_out  device [B][L][H_kv][k_patch*patch_cap][D] (patch_cap from
 *                 mukv_get_state), payload dtype; rows past the last copied one
 *                 are zero-filled
 *   n_tokens_out  device int32 [B] = rows copied per (layer, head), may be NULL
 *
 * Errors: INVALID_ARG, CAPACITY (B > max_questions), UNSUPPORTED (k_patch > 1024).
 */
int mukv_gather_patches(mukv_ctx *ctx, const int32_t *patch_idx, int32_t B, int32_t k_patch, int32_t order,
                        void *k_out, void *v_out, int32_t *n_tokens_out, void *stream);

/*
 * Attention of new tokens over the retrieved context at one layer (Sec. 3.5,
 * Eq. 9): the step after the retrieval.  For question b, query token i and
 * head h the keys are [R_k, W_K X]: the kept rows of the frames listed in
 * frame_idx[b] (entries -1 or out of range are skipped; the rows are read in
 * place from the cache, no gathered copy is needed) followed by the
 * question's own "local" rows (question tokens, tokens generated so far, the
 * current token), and the values [R_v, W_V X] likewise.  Scores are
 * q.k / sqrt(D), the softmax runs over all visible keys, head h uses KV head
 * h / (Hq / Hkv).  Every retrieved row is visible to every token.  The n_q
 * query tokens are the LAST n_q local rows: with causal_local = 1 token i sees
 * local row j only if j <= n_local_b - n_q + i; with 0 it sees all of them.
 * A token that sees no key at all gets zeros.
 *
 *   layer          0 .. n_layers-1: which layer's kept rows are read
 *   q              device, payload dtype, [B][n_q][Hq][D] contiguous
 *   n_q            query tokens per question, 1 .. 16 (1 = decode)
 *   frame_idx      device int32 [B][k_frame] (e.g. mukv_retrieve's output), or
 *                  null with k_frame = 0
 *   k_local,       device, payload dtype, [n_local_total][Hkv][D]: the local
 *   v_local        rows of all questions back to back
 *   local_offsets  device int32 [B+1]: question b owns local rows
 *                  local_offsets[b] .. local_offsets[b+1]-1.  k_local,
 *                  v_local and local_offsets are given together or all null.
 *   out            device, payload dtype, [B][n_q][Hq][D]
 *
 * Arithmetic in fp32 (dot products, exp2, sums in a fixed order); the output
 * is rounded to the payload dtype.  Uses scratch owned by the context: calls
 * on one context must not overlap.
 * Errors: INVALID_ARG, CAPACITY (B > max_questions), UNSUPPORTED (n_q > 16,
 * k_frame > 1024, pointers not 16-byte aligned).
 */
int mukv_attend(mukv_ctx *ctx, int32_t layer, const void *q, int32_t n_q, const int32_t *frame_idx, int32_t k_frame,
                const void *k_local, const void *v_local, const int32_t *local_offsets, int32_t B, int32_t causal_local,
                void *out, void *stream);

/*
 * The prefill of new tokens at one layer, which also yields the attention the
 * new tokens receive (Sec. 3.2: each step's tokens attend to the past cache of
 * their granularity and to themselves; Sec. 3.3, Eq. 1: the compression takes
 * its attention signal from that prefill at no extra cost).  The attention is
 * that of mukv_attend -- same arguments, same visibility rules -- for up to
 * 8192 query tokens per question; the new tokens are the LAST n_q local rows
 * of the question (local rows before them, if any, are older context).  A
 * question should own at least n_q local rows; new tokens without a row of
 * their own (fewer local rows than n_q) receive a signal of zero and are
 * attended to by nobody.
 *
 *   att_signal_out  device float [B][n_q]: for new token j of question b the
 *                   mean over the Hq heads and the n_q query tokens of the
 *                   softmax weight put on it, the softmax being normalised over
 *                   everything the query sees (retrieved rows, older local rows,
 *                   new tokens).  With B = 1 and n_q = n_frames * P it is the
 *                   att_signal argument of mukv_compress_chunk (Eq. 4 min-max
 *                   normalises it per unit, so the common factor is immaterial).
 *   workspace       device scratch of at least mukv_prefill_workspace_size()
 *                   bytes, 16-byte aligned, owned by the caller; contents are
 *                   undefined afterwards.  The call allocates nothing.
 *
 * Arithmetic in fp32, sums in a fixed order; `out` is rounded to the payload
 * dtype.  For bf16 payloads with D = 128 both products run on the matrix
 * cores: the softmax weights enter the value product rounded to bf16 (the
 * normaliser and att_signal_out use the unrounded fp32 weights).
 * Errors: INVALID_ARG (null pointers: here the local rows and both
 * outputs are required), CAPACITY (B > max_questions, workspace too small),
 * UNSUPPORTED (n_q > 8192, k_frame > 1024, n_q * Hq > 524 280, alignment).
 */
int mukv_prefill_workspace_size(const mukv_ctx *ctx, int32_t n_q, int32_t k_frame, int32_t B, int64_t *bytes_out);
int mukv_prefill_attend(mukv_ctx *ctx, int32_t layer, const void *q, int32_t n_q, const int32_t *frame_idx,
                        int32_t k_frame, const void *k_local, const void *v_local, const int32_t *local_offsets,
                        int32_t B, int32_t causal_local, void *out, float *att_signal_out, void *workspace,
                        int64_t workspace_bytes, void *stream);

/*
 * mukv_prefill_attend for callers that cannot allocate device memory and so
 * have no workspace to hand over: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments without the
 * workspace, same kernels, same results.  The scratch is a fixed array of
 * MUKV_STATIC_SCRATCH_BYTES in the library's device image, one copy per GPU,
 * held until the process ends; the call allocates and frees nothing.
 *
 * A call whose mukv_prefill_workspace_size() exceeds MUKV_STATIC_SCRATCH_BYTES
 * returns MUKV_ERR_CAPACITY and launches nothing (in the 7B head layout one
 * frame of 196 new tokens over 32 retrieved frames needs 23 MB, a chunk of
 * 1568 tokens 5 MB).  Every call on a GPU -- of any context, on any stream --
 * uses that GPU's one array: calls that overlap in time on one GPU race and
 * must be ordered by the caller (one stream, or events).  Nothing in the
 * array has to start at zero; it keeps the last call's contents.
 * Errors otherwise as for mukv_prefill_attend.
 */
#define MUKV_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
int mukv_prefill_attend_static(mukv_ctx *ctx, int32_t layer, const void *q, int32_t n_q, const int32_t *frame_idx,
                               int32_t k_frame, const void *k_local, const void *v_local,
                               const int32_t *local_offsets, int32_t B, int32_t causal_local, void *out,
                               float *att_signal_out, void *stream);

/*
 * Snapshot of the cache (the offline memory of Sec. 3.3 is persistent state):
 * the kept K/V rows, kept positions, block keys and running segment sums of
 * the frames ingested so far, in one host buffer, so that a stream can be
 * resumed in another context of the same configuration.  These three calls
 * are for set-up and tear-down, not for the hot path: save and load copy
 * between device and host on `stream` and SYNCHRONISE it before returning.
 *
 *   mukv_snapshot_size  bytes a snapshot of the current content needs
 *   mukv_snapshot_save  host_dst: host buffer of at least that size.  Gathered
 *                       chunks are launched first.  CAPACITY if too small.
 *   mukv_snapshot_load  host_src: a buffer written by mukv_snapshot_save.  The
 *                       context's content is replaced (after a wait for all
 *                       work on the device); afterwards the stream
 *                       continues at the snapshot's frame count.  SHAPE if
 *                       the configurations differ (layers, heads, D, P, F, S,
 *                       dtype, kappa, scoring layer), CAPACITY if the
 *                       snapshot holds more than max_frames frames,
 *                       INVALID_ARG if the buffer is not a snapshot.
 */
int mukv_snapshot_size(const mukv_ctx *ctx, int64_t *bytes_out);
int mukv_snapshot_save(mukv_ctx *ctx, void *host_dst, int64_t bytes, void *stream);
int mukv_snapshot_load(mukv_ctx *ctx, const void *host_src, int64_t bytes, void *stream);

/*
 * Combined gather over the three granularities of Sec. 3.4: the kept rows of
 * every frame of the selected segments, of the selected frames and of the
 * selected super-patches, every row once, in temporal order (ascending frame,
 * ascending position), packed into one dense decode context per question.
 *
 *   seg_idx, frame_idx, patch_idx  device int32 [B][k_*]; a list may be NULL
 *                 with its k 0; -1 and out-of-range entries are skipped
 *   rows_cap      rows per (layer, head) the outputs have room for
 *   k_out, v_out  device [B][L][H_kv][rows_cap][D], payload dtype; rows past the
 *                 last copied one are zero-filled
 *   n_tokens_out  device int32 [B]: rows the union holds; when it exceeds
 *                 rows_cap only the first rows_cap rows were copied.  May be NULL.
 *
 * Needs superpatches_per_frame <= 32.  Calls on one context must not overlap
 * (the plan of the union lives in the context).
 * Errors: INVALID_ARG, CAPACITY (B > max_questions), UNSUPPORTED.
 */
int mukv_gather_union(mukv_ctx *ctx, const int32_t *seg_idx, int32_t k_seg, const int32_t *frame_idx, int32_t k_frame,
                      const int32_t *patch_idx, int32_t k_patch, int32_t B, int32_t rows_cap, void *k_out, void *v_out,
                      int32_t *n_tokens_out, void *stream);

/*
 * Retrieval over several independently compressed stores (Sec. 3.3,
 * granularity-adaptive compression: the patch-, frame- and segment-level caches
 * are pruned on their own, each with its rho and alpha; Sec. 3.4: the question
 * is scored against every cache, and stage 2 applies the global query taken
 * from the segment-level cache to the candidates of the finer ones; Sec. 4.1:
 * k_g = 20 / 32 / 12 and lambda_g = 0.3 / 0.3 / 0 for patch / frame / segment).
 * A store is a context whose unit of compression (tokens_per_frame) is that
 * granularity's block -- a segment of F*P tokens, a frame of P, a super-patch of
 * floor(P/S) -- fed by its own mukv_compress_chunk calls.  The blocks searched
 * here are the store's units, each with its Eq. 5 key; the store's own segment
 * level takes no part.
 *
 * mukv_retrieve_units scores the visible units of ONE store against the
 * questions (Eq. 6-7) and selects k of them per question:
 *   global_query_in == NULL  (the coarsest store, lambda_g = 0): the k best by
 *       the stage-1 score.  If global_query_out != NULL it receives, per
 *       question, the mean of the keys of the first n_global of them (0: all
 *       k; fewer if fewer units exist) -- the global query of stage 2.
 *   global_query_in != NULL  (a finer store): stage 1 keeps the 2k best units,
 *       stage 2 gives each gamma = cos(its key, the question's global query)
 *       and s~ = (1 - lambda_g) s + lambda_g gamma (Eq. 8); the k best by s~
 *       are returned (equal s~: the lower unit number).
 *
 *   q_tokens, q_offsets, B    as for mukv_retrieve
 *   n_visible_units           units that precede the questions (timestamp); < 0: all
 *   global_query_in / _out    device double [B][H_kv*D], 8-byte aligned; at most
 *                             one of them non-NULL
 *   idx_out                   device int32 [B][k], rank order, padded with -1
 *   score_out                 device float [B][k] (s, or s~), may be NULL
 *
 * The calls for the stores of one question batch are ordered by the stream:
 * first the store that writes the global query, then those that read it.
 * Errors: INVALID_ARG, CAPACITY (B > max_questions), UNSUPPORTED (2k > 1024,
 * alignment).
 */
int mukv_retrieve_units(mukv_ctx *ctx, const void *q_tokens, const int32_t *q_offsets, int32_t B, int32_t k,
                        double lambda_g, int32_t n_visible_units, const double *global_query_in, int32_t n_global,
                        double *global_query_out, int32_t *idx_out, float *score_out, void *stream);

/*
 * One decode context from several stores (Sec. 3.5: the retrieved blocks of
 * all granularities are loaded as the context of Eq. 9): the kept rows of the
 * chosen units of every store, in temporal order -- ascending time step, unit u
 * of store i belonging to step u / units_per_step[i]; within a step the stores
 * in the order given (coarse to fine) and a store's units ascending.  A unit
 * listed twice is copied once; entries that name no unit of their store (-1
 * padding, numbers past the units held) are skipped.
 *
 *   ctxs            host array of n_ctx (1..4) contexts with the same n_layers,
 *                   n_kv_heads, head_dim, dtype and device
 *   unit_idx        host array of n_ctx device pointers, int32 [B][k[i]] each
 *   k               host int32 [n_ctx]; the k[i] add up to at most 3072
 *   units_per_step  host int32 [n_ctx], >= 1 (the paper's stores: 1, 1, S)
 *   rows_cap        rows of the output per (layer, head)
 *   k_out, v_out    device [B][L][H_kv][rows_cap][D], payload dtype; rows past
 *                   the context are zero-filled, rows past rows_cap dropped
 *   n_tokens_out    device int32 [B]: rows of the whole context.  May be NULL.
 *
 * The plan lives in ctxs[0]: calls that share it must not overlap.
 * Errors: INVALID_ARG, SHAPE (stores of different models), CAPACITY
 * (B > max_questions of ctxs[0]), UNSUPPORTED.
 */
int mukv_gather_multi(mukv_ctx *const *ctxs, int32_t n_ctx, const int32_t *const *unit_idx, const int32_t *k,
                      const int32_t *units_per_step, int32_t B, int32_t rows_cap, void *k_out, void *v_out,
                      int32_t *n_tokens_out, void *stream);

/*
 * Packs the stored K,V of the selected frames of each question into a dense
 * decode context (the retrieved part of R_k, R_v in Eq. 9).
 *
 *   frame_idx     device int32 [B][k_frame]; -1 entries are skipped
 *   order         MUKV_TEMPORAL: ascending frame number; MUKV_AS_GIVEN
 *   k_out, v_out  device [B][L][H_kv][k_frame*kappa][D], payload dtype; slots
 *                 past the last selected frame are zero-filled
 *   n_tokens_out  device int32 [B] = selected frames * kappa, may be NULL
 *
 * Frame numbers must be < n_frames (larger ones are skipped like -1).
 * Errors: INVALID_ARG, CAPACITY (B > max_questions), UNSUPPORTED (k_frame > 1024).
 */
int mukv_gather_kv(mukv_ctx *ctx, const int32_t *frame_idx, int32_t B, int32_t k_frame, int32_t order,
                   void *k_out, void *v_out, int32_t *n_tokens_out, void *stream);

/* Fills *out (host).  Does not synchronise. */
int mukv_get_state(const mukv_ctx *ctx, mukv_state *out);

/* Static, never-NULL description of a status code. */
const char *mukv_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* MUKV_H */
