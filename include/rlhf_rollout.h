/*
 * rlhf_rollout.h -- C ABI of the MI355X (gfx950) rollout library.
 *
 * The library covers the experience-generation step of PPO stage 3 as the
 * paper frames it (Section 2.1, "RLHF Training"): the actor generates a
 * response token by token against a key/value cache, and the generated
 * positions are then scored by the actor and the reference model to obtain
 * per-token log-probabilities and the penalty on policy deviation.  The cache
 * lives in ONE preallocated arena cut into fixed pages, which is this
 * library's answer to the paper's finding that the inference phases of RLHF
 * leave an allocator full of cached blocks of assorted sizes that later
 * requests cannot reuse (Section 3.1; Appendix A): nothing is ever taken from
 * or returned to the driver between create and destroy, so the paper's
 * fragmentation event (Section 3, first paragraph; Appendix B: reserved minus
 * allocated at the moment the allocator must call the driver) cannot occur.
 *
 * Conventions
 *   - Every function returns an rlhf_status.  No C++ exception crosses the
 *     boundary.  rlhf_last_error_string() gives text for the last failure on
 *     the calling thread.
 *   - "dev" pointers are device memory owned by the caller (for example a
 *     torch tensor's data_ptr()); "host" pointers are ordinary host memory and
 *     are fully read before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls that launch work enqueue it on that stream and return without
 *     synchronising, except where stated.
 *   - One arena may be used by one host thread at a time, and the calls that
 *     pass it a stream must be ordered with respect to each other on the
 *     device (one stream, or streams the caller orders with events): the
 *     arena's device mirrors and its append scratch change in that order.
 *     A workspace serves one call at a time in the same sense.  Several host
 *     threads may call the compute entry points at once, each with outputs and
 *     a workspace of its own; no call's result depends on an earlier call.
 *     (rlhf_decode_attention keeps a few counters in device memory of the
 *     library's own, one set per calling stream, zero between calls: see there.)
 *   - The compute entry points (decode and prefill attention, log-prob/KL,
 *     the draws, the probes) allocate nothing, issue no memset or copy and
 *     never synchronise: they may be recorded into a HIP graph on the stream
 *     they are given and replayed; a replay reads the buffers' contents of
 *     that moment.  rlhf_kv_arena_append and rlhf_kv_arena_free_seq may not
 *     be recorded (their bookkeeping runs on the host at call time).
 *   - Compute entry points fail with RLHF_ERR_DEVICE when no HIP device is
 *     usable; there is no CPU fallback.
 *   - One kernel launch holds fewer than 2^32 lanes per grid dimension.  The
 *     row-wise entry points (log-prob/KL, the draws) spread rows over two
 *     dimensions and take any int32 row count; the others return
 *     RLHF_ERR_UNSUPPORTED, before anything has changed, for a call whose one
 *     launch would not fit (the limits are stated with each: all are beyond
 *     what fits the device's memory at the paper's model shapes).
 */
#ifndef RLHF_ROLLOUT_H
#define RLHF_ROLLOUT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RLHF_OK = 0,
    RLHF_ERR_INVALID = -1,     /* NULL pointer, bad shape, id out of range, misaligned buffer */
    RLHF_ERR_OOM = -2,         /* arena has too few free pages; state unchanged */
    RLHF_ERR_DEVICE = -3,      /* a HIP call failed */
    RLHF_ERR_UNSUPPORTED = -4  /* dtype / head_dim / page size outside what the kernels cover, or a
                                  call too large for one launch (split it) */
} rlhf_status;

typedef enum { RLHF_F16 = 0, RLHF_BF16 = 1, RLHF_F32 = 2 } rlhf_dtype;

/* Tokens per page.  The kernels are written for this value only. */
#define RLHF_PAGE_TOKENS 16

/* ------------------------------------------------------------------------
 * KV arena
 *
 * Storage.  The arena holds n_pages K pages followed by n_pages V pages.  A
 * page holds RLHF_PAGE_TOKENS tokens of every KV head; the part of a page that
 * belongs to one head is a "block" of 16*head_dim elements, and block
 * (page, head) starts at element (page*n_kv_heads + head)*16*head_dim of the K
 * (or V) half.  Inside a block the elements are stored in the order in which
 * one 64-lane wavefront consumes them, so that every 1 KiB a wavefront loads
 * is contiguous and is already a matrix-core operand:
 *
 *   K block: element (slot s, dim d) at offset ((d/8)*16 + s)*8 + d%8
 *            -- 16-byte granules of 8 consecutive dims, granules of the 16
 *            slots adjacent, then the next 8 dims;
 *   V block: element (slot s, dim d) at offset ((s/4)*head_dim + d)*4 + s%4
 *            -- 8-byte granules of 4 consecutive slots at one dim, granules of
 *            consecutive dims adjacent, then the next 4 slots.
 *
 * Callers never need this layout: rlhf_kv_arena_append writes it and
 * rlhf_kv_arena_gather reads it back in plain [token][head][dim] order.
 *
 * Bookkeeping (all integer, exact).  Pages are popped from the head of a free
 * list that starts as initial_free_order.  A sequence takes a new page exactly
 * when its length is a multiple of 16.  rlhf_kv_arena_free_seq pushes the
 * sequence's pages to the tail of the free list in logical order;
 * rlhf_kv_arena_reset restores initial_free_order.  reset is the arena's
 * counterpart of the cache release the paper inserts after each phase
 * (Section 3.3), at the cost of host integer work and two small fill kernels.
 * ------------------------------------------------------------------------ */

typedef struct rlhf_kv_arena rlhf_kv_arena; /* opaque, library-owned */

/* flags for rlhf_kv_arena_desc.flags */
#define RLHF_ARENA_HOST_ONLY 1u /* bookkeeping only: no device is touched, append ignores
                                   k_new/v_new, views/gather are unavailable */

typedef struct {
    int32_t max_seqs;          /* sequence ids are 0 .. max_seqs-1 */
    int32_t n_kv_heads;
    int32_t head_dim;          /* 64 or 128 */
    int32_t page_tokens;       /* must be RLHF_PAGE_TOKENS */
    int32_t n_pages;           /* pages in the arena (each has a K part and a V part) */
    int32_t max_pages_per_seq; /* row length of the page table */
    int32_t kv_dtype;          /* RLHF_F16 or RLHF_BF16 */
    uint32_t flags;
    void *device_buffer;       /* dev, 256-byte aligned, caller-owned; NULL: the library
                                  makes the one allocation itself */
    size_t device_buffer_bytes;/* must be >= rlhf_kv_arena_bytes_required */
    const int32_t *initial_free_order; /* host, a permutation of 0..n_pages-1; NULL: identity */
} rlhf_kv_arena_desc;

/* Bytes of K/V storage the description needs (2 * n_pages * page bytes). */
int rlhf_kv_arena_bytes_required(const rlhf_kv_arena_desc *desc, size_t *out_bytes);

/* Creates the arena.  Besides the K/V storage it allocates, once, the device
 * page table [max_seqs][max_pages_per_seq] (int32, unused entries -1), the
 * device lengths [max_seqs] (int32) and a small pinned command ring.  Nothing
 * is allocated afterwards.  Synchronises the device once. */
int rlhf_kv_arena_create(const rlhf_kv_arena_desc *desc, rlhf_kv_arena **out);

/* Waits for the device, then frees everything the library allocated. */
int rlhf_kv_arena_destroy(rlhf_kv_arena *arena);

/* Appends n_new[i] tokens to sequence seq_ids[i], i = 0 .. n_seqs-1, in that
 * order.  k_new / v_new (dev) hold the new rows packed as [sum n_new][n_kv_heads]
 * [head_dim] in the arena's dtype, sequence after sequence.  A sequence id may
 * appear once per call.  All-or-nothing: if the free list is too short the call
 * returns RLHF_ERR_OOM, and if a sequence would outgrow max_pages_per_seq it
 * returns RLHF_ERR_INVALID; a call of more than 2^26 - 4 (token, head) pairs
 * (sum n_new * n_kv_heads) returns RLHF_ERR_UNSUPPORTED; in all three cases
 * nothing has changed.  The host
 * mirrors are updated before return; the device page table, lengths and K/V
 * pages are updated in stream order.
 *
 * Waiting.  Each append and free_seq hands its changes to the device through
 * one of four pinned command slots.  A call whose slot is still being read --
 * that is, when the fourth-previous append/free_seq on this arena has not yet
 * run on the device -- waits for that one (hipEventSynchronize) before it
 * touches anything; otherwise the call does not synchronise.
 *
 * Device errors.  RLHF_ERR_DEVICE from that wait, or from a kernel launch the
 * device refuses before any of the call's work was enqueued, leaves host and
 * device mirrors unchanged (the host bookkeeping is taken back).  If an error
 * strikes after part of the call was enqueued (a later launch of a multi-token
 * append, or the event that guards the slot), the device will still apply what
 * it was given: the call returns RLHF_ERR_DEVICE, the arena refuses append and
 * free_seq from then on, and rlhf_kv_arena_reset (which rewrites both mirrors)
 * makes it usable again.
 *
 * Neither append nor free_seq may be recorded into a HIP graph: their
 * bookkeeping runs on the host at call time and the kernels read a pinned slot
 * whose contents belong to that one call. */
int rlhf_kv_arena_append(rlhf_kv_arena *arena, const int32_t *seq_ids /*host*/,
                         const int32_t *n_new /*host*/, int32_t n_seqs,
                         const void *k_new /*dev*/, const void *v_new /*dev*/, void *stream);

/* Returns the pages of one sequence to the free-list tail; length becomes 0.
 * Device mirrors are updated in stream order.  Waiting, device errors and graph
 * capture: as for rlhf_kv_arena_append. */
int rlhf_kv_arena_free_seq(rlhf_kv_arena *arena, int32_t seq_id, void *stream);

/* Testing aid, not a step of the method: the next n_calls calls of
 * rlhf_kv_arena_append / rlhf_kv_arena_free_seq on this arena that pass
 * validation behave as if the device had refused their first kernel: they take
 * their bookkeeping back through the same path a real refusal takes, enqueue
 * nothing and return RLHF_ERR_DEVICE, so that "nothing has changed" can be
 * checked (host mirrors, and device mirrors on a real arena) without a failing
 * device.  Works on host-only arenas too.  n_calls = 0 switches it off. */
int rlhf_kv_arena_fail_next_submissions(rlhf_kv_arena *arena, int32_t n_calls);

/* Phase boundary: every page free again in initial_free_order, every length 0. */
int rlhf_kv_arena_reset(rlhf_kv_arena *arena, void *stream);

/* The paper's allocator counters (Section 2.2) for the arena. */
typedef struct {
    uint64_t reserved_bytes;    /* K/V storage taken at create; constant */
    uint64_t allocated_bytes;   /* pages in use * page bytes, K and V */
    uint64_t live_token_bytes;  /* bytes of tokens actually cached */
    uint64_t driver_allocations;/* calls to the driver for K/V storage since create: 1 if the
                                   library allocated the buffer, 0 if the caller brought it */
    int32_t pages_free;
    int32_t pages_in_use;
    int32_t peak_pages_in_use;  /* since create or the last reset */
    int32_t live_seqs;          /* sequences with length > 0 */
} rlhf_kv_arena_stats_t;

int rlhf_kv_arena_stats(const rlhf_kv_arena *arena, rlhf_kv_arena_stats_t *out);

/* Device views for rlhf_decode_attention.  Pointers stay valid until destroy. */
int rlhf_kv_arena_views(const rlhf_kv_arena *arena, const void **k_arena, const void **v_arena,
                        const int32_t **page_table /*dev [max_seqs][max_pages_per_seq]*/,
                        const int32_t **seq_lens /*dev [max_seqs]*/);

/* Host mirrors of the bookkeeping (valid until the next call on the arena):
 * page table [max_seqs][max_pages_per_seq] with -1 in unused entries, lengths
 * [max_seqs], and the free list (free_count entries, head first). */
int rlhf_kv_arena_host_state(const rlhf_kv_arena *arena, const int32_t **page_table,
                             const int32_t **seq_lens, const int32_t **free_list,
                             int32_t *free_count);

/* Reads tokens [start, start+n) of a sequence back as plain rows: k_out / v_out
 * (dev) receive [n][n_kv_heads][head_dim] in the arena's dtype.  More than
 * 2^26 - 4 (token, head) pairs in one call: RLHF_ERR_UNSUPPORTED. */
int rlhf_kv_arena_gather(const rlhf_kv_arena *arena, int32_t seq_id, int32_t start, int32_t n,
                         void *k_out /*dev*/, void *v_out /*dev*/, void *stream);

/* ------------------------------------------------------------------------
 * Decode attention (Section 2.1: the actor generating one token per step).
 *
 * For every sequence b and query head h, with kv head h / (n_q_heads /
 * n_kv_heads) and L = seq_lens[b] cached tokens (the current token's K/V has
 * been appended already, so causality needs no mask):
 *     s_j = softmax_scale * <q[b,h,:], K_j>,  j = 0 .. L-1
 *     out[b,h,:] = sum_j softmax(s)_j * V_j
 * computed as a split over the token range with an online softmax per split
 * and a log-sum-exp merge; fp32 accumulation.  L = 0 gives zeros.  Lengths
 * above max_seq_len are treated as max_seq_len.
 *
 *   q          dev [batch][n_q_heads][head_dim], qkv_dtype
 *   k_arena    dev, K half of an arena in the block layout above
 *   v_arena    dev, V half
 *   page_table dev [batch][max_pages_per_seq] int32
 *   seq_lens   dev [batch] int32
 *   out        dev [batch][n_q_heads][head_dim], out_dtype (round to nearest even)
 *   workspace  dev, >= rlhf_decode_attention_workspace_bytes, 16-byte aligned;
 *              scratch for split partials, contents undefined afterwards
 * q, k_arena, v_arena and out must be 16-byte aligned.  batch may not exceed
 * 8192 per call, nor batch * n_q_heads 2^26 - 4 (RLHF_ERR_UNSUPPORTED; split
 * larger batches).
 *
 * Launches.  With one query head per KV head the call is one kernel launch
 * when it can be: the wavefront that completes a (sequence, head) unit merges
 * the unit's split partials itself.  That needs one arrival counter per unit,
 * which cannot live in a workspace whose contents are undefined; the counters
 * are device memory of the library's (zero when loaded, and every call leaves
 * them zero), one set for each of the first 8 streams that call on a device,
 * since calls on one stream never overlap.  The call takes two launches (split
 * kernel, merge kernel; no state at all) with grouped-query heads (where the
 * merge kernel's wavefront per query head is faster), while its stream is
 * being captured into a graph, on further streams, above 32768 (sequence, head)
 * units per call, and when the units are so few that one wavefront would have
 * to merge dozens of partials (a call whose caches cannot exceed 8 MiB in all
 * -- batch * heads * max_seq_len * head_dim * 4 bytes, so a tight max_seq_len
 * helps -- is cut into fewer pieces instead, so that it still takes one launch:
 * it is bound by latencies, not bytes).  Both forms give bit-identical results; each is
 * deterministic for given inputs, and neither depends on which physical pages
 * a sequence owns.  A stream destroyed while a call on it is still running
 * must not be replaced by a new stream that calls at once (the new one could
 * be given the same handle and so the same counters).
 * ------------------------------------------------------------------------ */
typedef struct {
    int32_t batch;
    int32_t n_q_heads;
    int32_t n_kv_heads;        /* divides n_q_heads */
    int32_t head_dim;          /* 64 or 128 */
    int32_t page_tokens;       /* RLHF_PAGE_TOKENS */
    int32_t max_pages_per_seq; /* row length of page_table */
    int32_t max_seq_len;       /* upper bound on seq_lens; 0: max_pages_per_seq*page_tokens.
                                  Sizes the launch and the workspace. */
    int32_t qkv_dtype;         /* RLHF_F16 or RLHF_BF16 */
    int32_t out_dtype;         /* qkv_dtype or RLHF_F32 */
    float softmax_scale;       /* 0: 1/sqrt(head_dim) */
} rlhf_attn_params;

int rlhf_decode_attention_workspace_bytes(const rlhf_attn_params *params, size_t *out_bytes);

int rlhf_decode_attention(const rlhf_attn_params *params, const void *q, const void *k_arena,
                          const void *v_arena, const int32_t *page_table, const int32_t *seq_lens,
                          void *out, void *workspace, size_t workspace_bytes, void *stream);

/* rlhf_decode_attention for callers that cannot allocate device memory and so
 * cannot bring a workspace (code under graph capture, serving loops, harnesses
 * that forbid allocation): the split partials go to a 16 MiB scratch array
 * that is part of the library's device image (one per device, held until the
 * process ends).  Same arguments, results and limits otherwise; a shape whose
 * workspace (rlhf_decode_attention_workspace_bytes) would exceed 16 MiB is
 * RLHF_ERR_UNSUPPORTED (the largest configuration of the paper's model shapes,
 * 128 sequences x 64/8 heads x 128, needs 8.5 MB).  The call allocates nothing,
 * issues no memset or copy and does not synchronise.  All calls on a device
 * share that one array and one set of arrival counters, whatever their stream:
 * calls that may overlap on the device race and must be ordered by the caller
 * (one stream, or events). */
int rlhf_decode_attention_static(const rlhf_attn_params *params, const void *q, const void *k_arena,
                                 const void *v_arena, const int32_t *page_table, const int32_t *seq_lens,
                                 void *out, void *stream);

/* ------------------------------------------------------------------------
 * Fused token log-probability and actor-vs-reference KL (Section 2.1: actor
 * and reference inferences over the generated tokens; the KL term is what
 * keeps the trained policy near the reference).  For each position i, in one pass over the two logit rows:
 *     logp_out[i] = log softmax(actor[i,:])[tokens[i]]
 *     kl_out[i]   = KL( softmax(actor[i,:]) || softmax(ref[i,:]) )   (nats, >= 0 up to rounding)
 * fp32 accumulation.  tokens[i] outside [0, vocab) marks padding: both
 * outputs are 0 for that position (negative ids are the padding convention;
 * an id >= vocab is scored the same way, and rlhf_token_logprobs_kl_rewards
 * can report it through a device flag).  Logits are finite or -infinity (a masked
 * entry); a NaN logit gives NaN outputs for its row.  The outputs carry the
 * fp32 rounding of the logits' own magnitude (about 1.2e-7 * max |logit|) on
 * top of the error of the sums, which stays far below 1e-3.
 *
 *   actor_logits, ref_logits  dev [n_positions][row_stride_elems], logits_dtype
 *                             (RLHF_F32 or RLHF_BF16 or RLHF_F16); first `vocab` entries of a row used
 *   tokens                    dev [n_positions] int32
 *   logp_out, kl_out          dev [n_positions] float
 *   row_stride_elems          0: vocab
 *   n_positions               0 .. 2^31 - 1 (above: RLHF_ERR_INVALID)
 * Rows that start 16-byte aligned take the vectorised path; others a slower
 * element-wise one with the same results up to summation order.
 * ------------------------------------------------------------------------ */
int rlhf_token_logprobs_kl(const void *actor_logits, const void *ref_logits, const int32_t *tokens,
                           float *logp_out, float *kl_out, int64_t n_positions, int32_t vocab,
                           int64_t row_stride_elems, int32_t logits_dtype, void *stream);

/* ------------------------------------------------------------------------
 * The same pass with per-token reward shaping (Section 2.1: the reference
 * model is there to keep the reward from running away, the reward model
 * supplies the sequence return).  Besides logp_out and kl_out, and at no extra HBM traffic:
 *     ref_logp_out[i] = log softmax(ref[i,:])[tokens[i]]
 *     reward_out[i]   = -kl_coef * penalty_i + terminal_scores[i]
 * with penalty_i = kl_out[i] (RLHF_PENALTY_FULL_KL) or the sampled estimate
 * logp_out[i] - ref_logp_out[i] (RLHF_PENALTY_SAMPLED), whose expectation over
 * tokens drawn from the actor is kl_out[i].  terminal_scores (dev [n_positions]
 * or NULL) is what the caller wants added per position: the sequence's score at
 * its last generated position, 0 elsewhere.  Padded positions get 0 in every
 * output.  ref_logp_out and reward_out may each be NULL.
 *
 * token_error_flag (dev int32 or NULL) tells a corrupted token id from padding:
 * the kernel stores 1 there when some tokens[i] >= vocab, and never stores
 * anything else, so the flag is sticky across calls until the caller clears it
 * (a 4-byte fill or copy on the same stream); it is read like any device
 * buffer, after the stream has reached the call.  Negative ids never set it.
 * ------------------------------------------------------------------------ */
#define RLHF_PENALTY_FULL_KL 0
#define RLHF_PENALTY_SAMPLED 1

typedef struct {
    float *ref_logp_out;          /* dev [n_positions] or NULL */
    float *reward_out;            /* dev [n_positions] or NULL */
    const float *terminal_scores; /* dev [n_positions] or NULL */
    float kl_coef;
    int32_t penalty;              /* RLHF_PENALTY_FULL_KL or RLHF_PENALTY_SAMPLED */
    int32_t *token_error_flag;    /* dev int32 or NULL: becomes 1 if some tokens[i] >= vocab */
} rlhf_reward_shaping;

int rlhf_token_logprobs_kl_rewards(const void *actor_logits, const void *ref_logits, const int32_t *tokens,
                                   float *logp_out, float *kl_out, int64_t n_positions, int32_t vocab,
                                   int64_t row_stride_elems, int32_t logits_dtype,
                                   const rlhf_reward_shaping *shaping, void *stream);

/* ------------------------------------------------------------------------
 * Next-token sampling in one pass over the logits (Section 2.1, experience
 * generation by the actor: this is the step between a decode step's logits and
 * the append of the next token).
 *     temperature > 0: tokens_out[i] = argmax_v ( logits[i,v]/T + G_iv ), with
 *         G_iv = -ln(-ln u_iv): an exact draw from softmax(logits[i,:]/T)
 *         (Gumbel-max).  u_iv = (k + 1/2) / 2^23 with k the top 23 bits of word
 *         v%4 of Philox4x32-10( counter = (v/4, i, offset low, offset high),
 *         key = (seed low, seed high) ).  No noise is read from memory; use a
 *         new offset for every decode step.
 *     temperature == 0: greedy argmax.
 *   Ties go to the lowest index.  logp_out (dev [n_rows] or NULL) receives
 *   log softmax(logits[i,:]/T)[token] (T = 1 for greedy).
 *   logits      dev [n_rows][row_stride_elems], F32 / BF16 / F16
 *   tokens_out  dev [n_rows] int32
 *   n_rows      0 .. 2^31 - 1 (above: RLHF_ERR_INVALID); the row index is a 32-bit
 *               counter word of the generator
 * ------------------------------------------------------------------------ */
int rlhf_sample_tokens(const void *logits, int32_t *tokens_out, float *logp_out, int64_t n_rows,
                       int32_t vocab, int64_t row_stride_elems, int32_t logits_dtype, float temperature,
                       uint64_t seed, uint64_t offset, void *stream);

/* The same draw with the rows cut into segments, for calls that bring fewer rows
 * than the chip has room for (a decode step: one row per sequence).  Each row is
 * read by up to eight workgroups and a second small kernel merges their records;
 * tokens_out is identical to rlhf_sample_tokens' for the same arguments (the
 * noise depends on (row, index) only), logp_out agrees to rounding.
 *   workspace  dev, >= rlhf_sample_tokens_workspace_bytes(n_rows, vocab),
 *              16-byte aligned, caller-owned scratch, contents irrelevant
 * With 512 rows or more it does what rlhf_sample_tokens does. */
int rlhf_sample_tokens_workspace_bytes(int64_t n_rows, int32_t vocab, size_t *out_bytes);
int rlhf_sample_tokens_split(const void *logits, int32_t *tokens_out, float *logp_out, int64_t n_rows,
                             int32_t vocab, int64_t row_stride_elems, int32_t logits_dtype, float temperature,
                             uint64_t seed, uint64_t offset, void *workspace, size_t workspace_bytes,
                             void *stream);

/* Top-k variant of the draw (Section 2.1, the same generation step with the
 * usual truncation of the sampling distribution).  With tau_i the top_k-th
 * largest logit of row i, only the entries with logits[i,v] >= tau_i take part:
 * every entry tied with the top_k-th stays, so at least top_k entries survive.
 * Each survivor gets the noise G_iv it would get in rlhf_sample_tokens (same
 * seed, offset, row and index), the token is the argmax of logits/T + G over the
 * survivors, and logp_out is the log of the softmax over the survivors only.
 * tau is found exactly (comparisons of the stored values, no rounding), so the
 * survivor set does not depend on the temperature.  top_k >= vocab is the plain
 * draw; top_k = 1 leaves the row maximum and whatever ties with it; top_k < 1
 * is RLHF_ERR_INVALID.  Rows holding NaN give unspecified tokens (in range).
 * One workgroup per row: meant for decode steps (hundreds of rows). */
int rlhf_sample_tokens_topk(const void *logits, int32_t *tokens_out, float *logp_out, int64_t n_rows,
                            int32_t vocab, int64_t row_stride_elems, int32_t logits_dtype, float temperature,
                            int32_t top_k, uint64_t seed, uint64_t offset, void *stream);

/* ------------------------------------------------------------------------
 * Prefill attention (Section 2.1: generation starts from the prompts; this is
 * the step that brings a prompt, or a chunk of it, into the cache before the
 * one-token-per-step loop).  The new tokens' K/V rows have been appended to the
 * arena already (rlhf_kv_arena_append takes any number of tokens per
 * sequence).  Sequence b brings n_b = cu_q[b+1] - cu_q[b] query rows, the last
 * n_b of its L_b = seq_lens[b] cached tokens; row i sits at position
 * p = L_b - n_b + i and attends causally to keys 0 .. p:
 *     s_j = softmax_scale * <q_i[h,:], K_j>,  out_i[h,:] = sum_{j<=p} softmax(s)_j V_j
 * with kv head h / (n_q_heads / n_kv_heads).  Matrix-core products, fp32
 * accumulation, one pass with a running softmax reference.  The softmax weights
 * enter the second product rounded to fp16, and so does V: an output element is
 * within 2^-11 * sum_j softmax(s)_j |V_j| of the exact one (plus fp32 rounding),
 * and a BF16 cache must keep |V| below 65536 (larger entries turn into
 * infinities in the result; BF16 magnitudes under 2^-14 are rounded to fp16
 * subnormals, an absolute error under 2^-25).
 *
 *   params     shapes as for decode attention (max_seq_len: as there)
 *   q          dev [cu_q[batch]][n_q_heads][head_dim], qkv_dtype, rows packed
 *              sequence after sequence
 *   cu_q       dev [batch+1] int32, non-decreasing, cu_q[0] = 0
 *   max_q_len  host: an upper bound on n_b.  It sizes the launch: a
 *              sequence's rows at or beyond max_q_len may be left untouched
 *              (those the launch's last block of positions still covers are
 *              computed, the others are not).
 *   out        dev, same shape as q, out_dtype
 * A sequence with n_b = 0 is skipped; one with n_b > L_b (more query rows than
 * cached tokens) is skipped too and its rows of out are left untouched.
 * q, k_arena, v_arena and out must be 16-byte aligned.  n_q_heads / n_kv_heads
 * may not exceed 256 (RLHF_ERR_UNSUPPORTED).
 * ------------------------------------------------------------------------ */
int rlhf_prefill_attention(const rlhf_attn_params *params, const void *q, const int32_t *cu_q,
                           int32_t max_q_len, const void *k_arena, const void *v_arena,
                           const int32_t *page_table, const int32_t *seq_lens, void *out, void *stream);

/* The same call with the workgroup size chosen by the caller.  A workgroup
 * covers a block of (32 * wavefronts / (n_q_heads / n_kv_heads)) positions of
 * one sequence and KV head: 12 wavefronts (three per SIMD) copy each K/V block
 * into LDS for more rows and hide more latency, 8 give more, smaller
 * workgroups when the call is small.  0 = the library's choice (12 once that
 * still leaves some 4096 workgroups), which is what rlhf_prefill_attention
 * uses; any other value is RLHF_ERR_INVALID.  Results are the same up to fp32
 * summation order. */
int rlhf_prefill_attention_wg(const rlhf_attn_params *params, const void *q, const int32_t *cu_q,
                              int32_t max_q_len, const void *k_arena, const void *v_arena,
                              const int32_t *page_table, const int32_t *seq_lens, void *out,
                              int32_t wavefronts_per_workgroup, void *stream);

/* Measurement aid, not a step of the method: reads `bytes` (rounded down to
 * 16) of `buffer` (dev, 16-byte aligned) once with the 16-byte streaming loads
 * the kernels above use and does nothing else, so that its duration gives the
 * device's practical read ceiling to set beside the published HBM peak.  sink
 * (dev uint32 or NULL) only keeps the loads alive.  Asynchronous on stream. */
int rlhf_probe_stream_read(const void *buffer, size_t bytes, uint32_t *sink, void *stream);

/* Measurement aid, not a step of the method: n_workgroups workgroups of 768
 * threads (three wavefronts per SIMD, as the prefill kernel runs) each take
 * sixteen 16-byte operand registers per lane from `operands` (dev, 16-byte
 * aligned, `bytes` >= 16, read modulo its length: bf16 values, the caller's
 * choice) and issue iterations x 8 of the 32x32x16 bf16 matrix products the
 * prefill kernel is made of, nothing else.  Flops = n_workgroups * 12 *
 * iterations * 8 * 32768; the caller times the call.  ticks (dev, three
 * uint64) receives, for workgroup 0's first wavefront, the duration of its
 * loop in ticks of the 100 MHz wall clock ([0]) and in shader cycles ([1]):
 * their ratio is the clock the device held, which under matrix load depends
 * on the operand data; [2] is scratch.  Keep operand magnitudes small enough
 * that iterations * 16 * max|a| * max|b| stays finite in fp32.  Asynchronous
 * on stream. */
int rlhf_probe_matrix_rate(const void *operands, size_t bytes, int32_t iterations, int32_t n_workgroups,
                           uint64_t *ticks, void *stream);

/* Text for the most recent failure on this thread ("" if none). */
const char *rlhf_last_error_string(void);

/* Library version, for the binding's sanity check. */
int rlhf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RLHF_ROLLOUT_H */
