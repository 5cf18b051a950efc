/*
 * w2v.h -- C ABI of the MI355X-native SGNS (skip-gram, negative sampling) trainer.
 *
 * The library trains the two word2vec matrices with the window scheme of the FULL-W2V
 * paper: the N negatives are drawn once per context window and shared by all of its
 * context words, the N+1 output rows (target + negatives) live in registers for the
 * window, the context rows live in an on-chip ring for as long as the window can reach
 * them, sentences are independent lock-free units (Sections 2.1, 3.1, 3.2, 4.2).
 *
 * Conventions
 *   - C99; no C++ types and no exceptions cross this boundary.
 *   - Every function returns W2V_OK (0) or a negative W2V_E* code; the text of the last
 *     error of a context is available from w2v_last_error().
 *   - "device" pointers are HIP device memory valid on cfg.device; "host" pointers are
 *     ordinary process memory.  The CALLER owns every device buffer and the stream; the
 *     library owns only the host-side context object and never allocates device memory.
 *   - All argument validation happens before the first HIP call, so every W2V_EINVAL /
 *     W2V_ESTATE / W2V_ENOMEM path can be exercised on a machine without a GPU.
 *   - One context is used by one host thread at a time.  Work is enqueued on cfg.stream;
 *     functions documented as "asynchronous" return before the GPU has finished.
 */
#ifndef W2V_H
#define W2V_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define W2V_OK      0
#define W2V_EINVAL -1   /* null pointer, value out of range, struct_size mismatch           */
#define W2V_ESTATE -2   /* call out of order (training before the unigram table was built) */
#define W2V_ENOMEM -3   /* caller-provided workspace too small                              */
#define W2V_EHIP   -4   /* a HIP runtime call failed; see w2v_last_error()                   */

#define W2V_MAX_DIM        512u        /* largest supported embedding size d                  */
#define W2V_MAX_WINDOW     16u         /* largest W                                           */
#define W2V_MAX_NEGATIVES  20u         /* largest N (the paper's range is N in [2,20], Sec. 2.1) */
#define W2V_MAX_VOCAB      (1u << 27)  /* word ids must fit 27 bits                           */

typedef struct w2v_ctx w2v_ctx;        /* opaque */

/* Hyper-parameters follow the problem statement of Section 2.1 (vocabulary V, dimension
 * d, window W, negatives N); learning-rate schedule and subsampling are the conventional
 * word2vec ones the evaluation section refers to. */
typedef struct w2v_config {
    uint32_t struct_size;         /* = sizeof(w2v_config)                                               */
    uint32_t vocab;               /* V in [1, W2V_MAX_VOCAB]                                            */
    uint32_t dim;                 /* d in [1, W2V_MAX_DIM]                                              */
    uint32_t window;              /* W in [1, W2V_MAX_WINDOW]; dim*window must not exceed 512*10        */
    uint32_t negatives;           /* N in [0, W2V_MAX_NEGATIVES]                                        */
    uint32_t window_mode;         /* 0: width of each window drawn uniformly from [1,W] (Sec. 3.2,
                                     "traditional"); 1: fixed width ceil(W/2) (Sec. 3.2, the paper's) */
    uint32_t total_epochs;        /* E >= 1, length of the learning-rate decay                          */
    uint32_t sentences_in_flight; /* 0: as many wavefronts at once as the GPU holds, but at most one per
                                     2,048 * ((N+1)/6)^2 tokens that survive subsampling in an epoch, with
                                     summed updates also at most 0.5 / (rows a wavefront holds * sum over
                                     words of the squared shares of the kept tokens), and at least 64
                                     (lock-free sentences, Sec. 2.2 / 2.3);
                                     k >= 1: at most k at once; 1 = strict corpus order, deterministic     */
    uint64_t tokens_per_epoch;    /* T >= 1, corpus tokens per epoch before subsampling                 */
    uint64_t seed;                /* keys every random decision and the weight initialisation          */
    double   lr0;                 /* starting learning rate (0.025)                                     */
    double   lr_min_frac;         /* floor of the decay as a fraction of lr0 (1e-4)                     */
    double   subsample_t;         /* frequent-word subsampling threshold t; 0 switches it off           */
    void    *syn0;                /* device, float[vocab*ld] (uint16 if storage = 1): input (context-word) embeddings */
    void    *syn1neg;             /* device, float[vocab*ld]: output (target / negative) weights          */
    uint32_t ld;                  /* row stride in floats, >= dim and a multiple of 4; columns
                                     dim..ld-1 are never read or written by training                    */
    int32_t  device;              /* HIP device ordinal                                                 */
    void    *stream;              /* hipStream_t owned by the caller (NULL = the default stream)        */
    void    *workspace;           /* device scratch, 256-byte aligned, owned by the caller              */
    uint64_t workspace_bytes;     /* >= w2v_query_workspace()                                           */
    uint32_t negative_block;      /* 0 or 1: N fresh negatives for every window (Sec. 3.1, the paper's
                                     method).  B in {2,4,8,16,32,64}: reuse over more than one window
                                     (Sec. 7, future work): the windows centred in one stretch of B
                                     consecutive tokens of a sentence (offsets before subsampling) share
                                     the N negatives drawn at the stretch's first position; a negative
                                     equal to a window's own target is skipped for that window only      */
    uint32_t update_mode;         /* How lock-free wavefronts write rows back (Sec. 2.2 / 2.3 leave the
                                     conflicts between sentences unresolved):
                                     1: overwrite -- a row goes back as the wavefront's copy of it (a context
                                        row's copy lives for up to 2W+1 windows), so of the updates several
                                        wavefronts make to one row at the same time only the last writer's
                                        survives;
                                     2: summed -- a row goes back as (what memory holds now) + (the change the
                                        wavefront made to its copy), and rows are stored at system scope, so
                                        wavefronts on different XCDs see each other's updates.  Exists
                                        for dim <= 256, 5 <= N <= 11 and windows of at most 10 as they occur;
                                        W2V_EINVAL otherwise.  Needs the snapshot space that
                                        w2v_query_workspace() then adds;
                                     0: automatic -- summed where such a kernel exists and the word counts
                                        say that the rows one L2 can hold carry under 30 % of the tokens
                                        (walks over a large graph), overwrite otherwise (text).
                                     Strict order (sentences_in_flight = 1) always overwrites: there is
                                     nothing to sum                                                      */
    uint32_t storage;             /* 0: the tables hold float (the paper's precision, Sec. 5.1).
                                     1 (extension): the tables hold bfloat16 -- uint16[vocab*ld], the upper halves
                                     of floats -- which halves the bytes every window moves.  All arithmetic stays
                                     in fp32 on the on-chip copies (a context row for as long as the window span
                                     holds it, Sec. 3.2; target and negative rows for one window, Sec. 3.1); a copy
                                     that goes back is rounded STOCHASTICALLY, with bits from the counter-based
                                     generator keyed by the token position that writes (nearest rounding would
                                     undo most steps, which are far smaller than a bfloat16's last place).  Exists
                                     for dim <= 320 that are multiples of 4 (or <= 128 and even, or <= 64),
                                     5 <= N <= 11, windows of at most 10 as they occur, update_mode 0 or 1
                                     (always overwriting); W2V_EINVAL otherwise                           */
    uint32_t reserved;            /* 0                                                                  */
} w2v_config;

/* Row stride (in floats) that keeps every row aligned to 128-byte memory lines. */
int w2v_query_ld(uint32_t dim, uint32_t *ld_out);

/* Bytes of device workspace needed for a sampling table of table_size slots.  Reads cfg->vocab, and
 * cfg->dim, window, window_mode, negatives and update_mode for the snapshot space of summed updates
 * (none if update_mode is 1 or the configuration has no such kernel; cfg->ld may be 0 = w2v_query_ld()). */
int w2v_query_workspace(const w2v_config *cfg, uint32_t table_size, uint64_t *bytes_out);

/* Validates cfg, copies it, and (init_weights != 0) fills syn0 with U(-0.5/d, 0.5/d) values
 * keyed by cfg->seed and syn1neg with zeros (asynchronous).  With init_weights == 0 the
 * caller's buffers are used as they are.  *out receives the context on success. */
int w2v_create(const w2v_config *cfg, int init_weights, w2v_ctx **out);

/* Frees the context.  Waits for the stream; never frees caller-owned buffers. */
int w2v_destroy(w2v_ctx *ctx);

/* Builds the negative-sampling table (the "weighted distribution" of Sec. 2.1: word i owns a
 * share count_i^0.75 of table_size slots) and the subsampling thresholds from the host array
 * counts_host[vocab], and uploads both into the workspace.  table_size in [1, 2^31].
 * Synchronous.  Must precede training. */
int w2v_build_unigram_table(w2v_ctx *ctx, const uint64_t *counts_host, uint32_t table_size);

/* One pass over n_sent sentences (Sec. 4.2: one sentence per execution unit, windows in strict
 * order inside a sentence).  tokens_dev: device int32 word ids (ids outside [0,V) are skipped like
 * subsampled words); sent_off_dev: device uint64[n_sent+1], sentence s is
 * tokens[sent_off[s] .. sent_off[s+1]).  first_token_global_pos is the position of tokens_dev[0]
 * inside the epoch (0 unless the epoch is fed in several calls); it enters the random-number key
 * and the learning rate.  epoch < total_epochs.  Asynchronous. */
int w2v_train_epoch(w2v_ctx *ctx, const int32_t *tokens_dev, const uint64_t *sent_off_dev,
                    uint64_t n_sent, uint64_t first_token_global_pos, uint32_t epoch);

/* w2v_train_epoch for callers that cannot allocate or be handed extra memory at the time of the call: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  It allocates no memory (no
 * hipMalloc / hipFree, no allocating library call) and uses none of the caller's workspace as scratch: its accumulators, its work-queue
 * head and (summed updates) its ring snapshots live in an array of W2V_STATIC_SCRATCH_BYTES that is part of the
 * library's code object (every GPU the library runs on holds one copy until the process ends).  The workspace is
 * only read (sampling table, thresholds).  Trains exactly like w2v_train_epoch (same kernels, same draws).
 * loss_sum_dev / pairs_dev: device locations that receive the loss sum and the number of (context, target) pairs of
 * THIS call (either may be NULL); the context's own accumulators (w2v_loss, w2v_counters) are not touched.
 * With summed updates the array holds the snapshots of (W2V_STATIC_SCRATCH_BYTES - 256) / (4 * (2W+2) * row floats
 * per wavefront) wavefronts: automatic concurrency is limited to that, an explicit cfg.sentences_in_flight beyond
 * it is W2V_EINVAL.  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two contexts) race and give wrong counts; calls on one stream do not.  Asynchronous. */
#define W2V_STATIC_SCRATCH_BYTES (32u << 20)
int w2v_train_epoch_static(w2v_ctx *ctx, const int32_t *tokens_dev, const uint64_t *sent_off_dev,
                           uint64_t n_sent, uint64_t first_token_global_pos, uint32_t epoch,
                           double *loss_sum_dev, uint64_t *pairs_dev);

/* The same pass for a corpus that lives in host memory (the batching pipeline of Sec. 4.1 without
 * the CPU-side sampling: only word ids cross the bus).  tokens_host / sent_off_host: host arrays
 * laid out as for w2v_train_epoch.  The sentences are cut into batches that fit one half of
 * staging_dev (caller-owned device memory, staging_bytes >= 2 * (room for the longest sentence),
 * 256-byte aligned); while one half is trained on, the other is filled over a copy stream the
 * context owns, so transfers hide behind the kernel.  Every random draw and the learning rate are
 * keyed by global token positions, so the result equals that of w2v_train_epoch on a resident copy
 * (bit for bit with sentences_in_flight = 1).  Returns when the last batch has been queued on the
 * context's stream (the call itself waits until all but the last two batches have been trained):
 * the host arrays must stay valid until that stream has been synchronised (pinned host memory
 * gives truly asynchronous copies, pageable memory works and blocks this call while each batch is
 * staged).  Every batch is a launch of its own, whose last wavefronts leave part of the GPU idle:
 * large halves (tens of MiB) keep that loss small.  The sentences are spread over as few batches as
 * fit, of nearly equal size, and the halves alternate across calls, so the first batch of an epoch
 * is copied while the previous epoch still trains.
 * W2V_EINVAL if a sentence does not fit half of the staging buffer. */
int w2v_train_epoch_host(w2v_ctx *ctx, const int32_t *tokens_host, const uint64_t *sent_off_host,
                         uint64_t n_sent, uint64_t first_token_global_pos, uint32_t epoch,
                         void *staging_dev, uint64_t staging_bytes);

/* Same arithmetic without any on-chip reuse: every (target, context) pairing re-reads and
 * re-writes its context row, and the window's N+1 output rows go through global memory per
 * context word.  Exists only as the memory-traffic comparator for w2v_train_epoch (the role
 * the pre-existing GPU kernels play in Table 4).  A sentence longer than 1,024 tokens is handled in
 * pieces of 1,024 tokens whose windows do not reach across the cut, so only sentences up to that
 * length (the corpus preparation rule of Table 3 allows 1,000) train as w2v_train_epoch does.
 * Asynchronous. */
int w2v_train_epoch_naive(w2v_ctx *ctx, const int32_t *tokens_dev, const uint64_t *sent_off_dev,
                          uint64_t n_sent, uint64_t first_token_global_pos, uint32_t epoch);

/* Copies matrix `which` (0 = syn0, 1 = syn1neg) as a dense [vocab][dim] float array (widened if storage = 1) into dst
 * (device memory if dst_is_device != 0, else host memory), dst_floats >= vocab*dim.
 * Waits for the stream. */
int w2v_get_embeddings(w2v_ctx *ctx, int which, float *dst, uint64_t dst_floats, int dst_is_device);

/* Sum of the SGNS log-loss over all windows trained since the last reset (each window's loss is
 * evaluated with the weights it started from) and the number of (context, target) pairs.
 * Mean loss = *loss_sum / *positive_pairs.  Either output may be NULL.  Waits for the stream. */
int w2v_loss(w2v_ctx *ctx, double *loss_sum, uint64_t *positive_pairs, int reset);

/* Token counters since the last reset: kept_tokens = tokens that survived subsampling (= context
 * windows processed), invalid_tokens = ids outside [0, vocab).  Either output may be NULL.
 * Waits for the stream. */
int w2v_counters(w2v_ctx *ctx, uint64_t *kept_tokens, uint64_t *invalid_tokens, int reset);

/* Test surface: writes, for every token t of the given range, the integer decisions the trainer
 * takes for it: keep_dev[t] (1 kept / 0 dropped), width_dev[t] (window width, 0 if dropped),
 * neg_dev[t*N + k] (k-th negative word id, -1 if dropped).  Device outputs.  Asynchronous. */
int w2v_debug_draws(w2v_ctx *ctx, const int32_t *tokens_dev, const uint64_t *sent_off_dev,
                    uint64_t n_sent, uint64_t first_token_global_pos, uint32_t epoch,
                    uint8_t *keep_dev, uint8_t *width_dev, int32_t *neg_dev);

/* Test surface: w2v_train_epoch with the window kernel itself writing out the integer decisions it
 * takes (the subsampling, width and negative draws of Sec. 2.1 / 3.1 / 3.2 as the hot path computes
 * them, not a second implementation): same outputs and layout as w2v_debug_draws, for every token
 * that gets a context window in this call.  Trains like w2v_train_epoch.  Asynchronous after one
 * wait for the stream. */
int w2v_debug_train_draws(w2v_ctx *ctx, const int32_t *tokens_dev, const uint64_t *sent_off_dev,
                          uint64_t n_sent, uint64_t first_token_global_pos, uint32_t epoch,
                          uint8_t *keep_dev, uint8_t *width_dev, int32_t *neg_dev);

/* Test surface: fixes the update mode of every later launch, strict order included (update = 0
 * overwrite, 1 summed, -1 back to cfg.update_mode's rules). */
int w2v_debug_set_update(w2v_ctx *ctx, int update);

/* Test surface: the work plan of the last launch (sentences before coarse_sentences were handed out as
 * 2^unit_shift units each, the others as 2^fine_shift; units in all), its update mode (0 overwrite,
 * 1 summed) and the wavefronts it was given.  Any output may be NULL.  Waits for the stream. */
int w2v_debug_get_plan(w2v_ctx *ctx, uint32_t *unit_shift, uint32_t *fine_shift,
                       uint64_t *coarse_sentences, uint64_t *units, uint32_t *update,
                       uint64_t *wavefronts);

/* Test surface: fixes the granularity of the work queue.  w2v_train_epoch hands a sentence out as
 * 2^unit_shift stretches of its tokens (each reads the W kept tokens on either side as context
 * only, so the windows are those of the whole sentence); by default the library picks the
 * exponent on the device from the sizes of the call (0 when one wavefront runs alone).  unit_shift in [0, 16]
 * fixes it, -1 restores the default. */
int w2v_debug_set_units(w2v_ctx *ctx, int unit_shift);

/* Test surface: fixes how the work queue ends.  By default lock-free launches cut the last eighth of
 * their sentences into smaller stretches than the rest, so that the wavefronts finish close
 * together.  fine_shift in [0, 16]: the sentences from index coarse_sentences on (all of them if
 * it is 0, none if it is >= n_sent) are handed out as 2^fine_shift stretches each, the ones before
 * as w2v_debug_set_units or the default says; fine_shift = -1 restores the default. */
int w2v_debug_set_unit_tail(w2v_ctx *ctx, int fine_shift, uint64_t coarse_sentences);

/* Test surface: runs the window kernel's cross-lane reduction on its own.  in_dev: device
 * float[60*64], value m of lane l at in_dev[m*64 + l]; out_dev: device float[64], out_dev[l] =
 * sum over lanes of value l for l < 60.  stream: hipStream_t or NULL.  Asynchronous. */
int w2v_debug_reduce(const float *in_dev, float *out_dev, void *stream);

/* Library-owned text of the last error of ctx (or of the last failed w2v_create when ctx is
 * NULL); valid until the next call on the same context. */
const char *w2v_last_error(const w2v_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* W2V_H */
