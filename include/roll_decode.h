/*
 * roll_decode.h - C ABI of the rollout decode step for MI355X (gfx950).
 *
 * One decode step of an LLM rollout worker over a ragged, continuously
 * refilled batch: paged grouped-query decode attention over per-sequence
 * KV lengths, then temperature / top-p sampling that records the log-prob
 * of the sampled token under the distribution it was drawn from.
 *
 * Where this sits in ROLL Flash (arXiv 2510.11345): Section 4.2 describes
 * the serving worker's event loop, whose "step-wise inference" service
 * advances the engine by one decode step over the running batch and whose
 * ADD / ABORT commands make requests join and leave that batch at step
 * granularity; Section 1 states that decoding is memory-bandwidth bound
 * and that response lengths are long-tailed; Section 5.1 (queue
 * scheduling) hands a freed slot the next prompt at once; Appendix A.1
 * fixes the sampling parameters (temperature, top_p, top_k off, one beam)
 * and uses the engine's token probability as the denominator of the
 * truncated importance weight.  The paper treats the engine step as a
 * black box; the definitions below are the standard ones it relies on.
 *
 * Conventions
 *   - Every pointer is tagged HOST or DEVICE.  DEVICE pointers belong to
 *     the one visible GPU; the caller owns them and the stream.
 *   - Calls that take a stream enqueue work on it (a hipStream_t passed as
 *     void*, NULL = the default stream) and return without waiting for it; the
 *     exceptions say so (roll_kv_commit when the host runs 8 commits ahead,
 *     the diagnostic and profiling calls marked SYNCHRONISES).
 *   - Return value: ROLL_OK (0) or a negative roll_status.  On error no
 *     output buffer has been written and no allocator state has changed.
 *     roll_last_error() returns a thread-local description.
 *   - bf16 = upper 16 bits of an IEEE-754 binary32, stored as uint16.
 *
 * KV page layout (both pools hold num_pages pages of page_size tokens for
 * num_kv_heads heads of head_dim elements, bf16).  The layouts are chosen
 * so that the matrix-core operands of the attention kernel are 16-byte
 * contiguous per lane and every load instruction of a wave covers whole
 * 128-byte lines; the writer (roll_kv_append_tokens) pays the transposition
 * once, the reader (every later decode step) never does.
 *   K:  k_pages[page][h][d / 8][kpos(t)][d % 8]   shape [N, Hkv, D/8, P, 8]
 *   V:  v_pages[page][h][t / 8][d][t % 8]         shape [N, Hkv, P/8, D, 8]
 * with t the token's position inside the page, d the head-dim index, and
 * kpos a fixed permutation of the token order inside blocks of W = min(P, 32)
 * tokens: for t = W * blk + u,
 *   kpos(t) = W * blk + (u & 3) + 4 * (u >> 3) + (W / 2) * ((u >> 2) & 1)
 * i.e. of every 8 consecutive tokens the first four go to the first half of
 * the block and the last four to the second half.  (The score tile of the
 * attention kernel hands each lane four consecutive tokens of either half;
 * with this order the K rows of one tile are contiguous in memory.)
 *
 * Page stride.  A page of a pool is Hkv * P * D elements; consecutive pages
 * are page_stride elements apart, the same for both pools (0 = dense, the
 * page size itself; otherwise a multiple of P * D that is >= Hkv * P * D).
 * The stride lets K and V share ONE allocation with the two blocks of a page
 * side by side, which is the layout to prefer:
 *   kv[page][0 = K, 1 = V][...],  k_pages = kv,  v_pages = kv + Hkv * P * D,
 *   page_stride = 2 * Hkv * P * D.
 * A decode step then reads one contiguous 2 * Hkv * P * D * 2 bytes per page
 * instead of two regions in different allocations, and DRAM serves fewer,
 * longer runs: measured 4-5 % more KV bandwidth on the 7B-class shapes.
 */
#ifndef ROLL_DECODE_H
#define ROLL_DECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum roll_status {
    ROLL_OK = 0,
    ROLL_ERR_INVALID_ARG = -1,  /* NULL / misaligned pointer, bad shape or parameter */
    ROLL_ERR_NO_PAGES = -2,     /* free list cannot cover the request; state unchanged */
    ROLL_ERR_SLOT_EMPTY = -3,   /* release of a slot that holds no sequence */
    ROLL_ERR_SLOT_RANGE = -4,   /* slot index outside [0, num_slots) */
    ROLL_ERR_SEQ_TOO_LONG = -5, /* sequence would need more than max_pages_per_seq pages */
    ROLL_ERR_WORKSPACE = -6,    /* workspace NULL, misaligned or too small */
    ROLL_ERR_HIP = -7,          /* a HIP runtime call failed (message has the HIP error) */
    ROLL_ERR_BUFFER_FULL = -8,  /* SampleBuffer: (1 + alpha) * batch samples are outstanding */
    ROLL_ERR_WOULD_BLOCK = -9   /* SampleBuffer: the call must wait for generation to finish */
} roll_status;

typedef enum roll_dtype { ROLL_BF16 = 0, ROLL_F32 = 1 } roll_dtype;

/* HOST. Thread-local text of the last error on this thread ("" if none). */
const char* roll_last_error(void);

/* HOST. Library version, e.g. "0.5". */
const char* roll_version(void);

/* ------------------------------------------------------------------ */
/* Page-table KV-cache allocator (Section 4.2: ADD enqueues a request, */
/* ABORT or completion reclaims it; Section 5.1: a freed slot is given */
/* the next prompt immediately).                                       */
/* ------------------------------------------------------------------ */

typedef struct roll_kv_pool roll_kv_pool;

typedef struct roll_kv_config {
    int32_t num_pages;          /* physical pages in each of k_pages / v_pages */
    int32_t page_size;          /* tokens per page: 16, 32 or 64 */
    int32_t num_slots;          /* rows of the running batch (B) */
    int32_t max_pages_per_seq;  /* row length of page_table */
    int32_t run_pages;          /* pages handed out together: 0 or 1 = single pages; 2, 4 or 8 = aligned
                                   runs of that many physically consecutive pages (see roll_kv_pool_create) */
} roll_kv_config;

/*
 * Create a pool.  The authoritative state (free-page stack, per-slot page
 * lists and lengths) lives in host memory owned by the pool.
 *   page_table_dev  DEVICE int32 [num_slots, max_pages_per_seq], borrowed for
 *                   the pool's lifetime; the pool fills it with -1 on the
 *                   first roll_kv_commit and keeps it in step afterwards.
 *   seq_lens_dev    DEVICE int32 [num_slots], borrowed likewise.
 * Both may be NULL together: the pool is then host-only (allocator logic,
 * schedulers, tests) and roll_kv_commit is an error.
 * Free pages are handed out as a LIFO stack whose initial pop order is
 * 0, 1, 2, ...; no result of the decode step depends on that order.
 * With run_pages = R > 1 the stack holds runs of R consecutive pages
 * (R k .. R k + R - 1; num_pages is used up to a multiple of R): a slot
 * takes a run when it needs page number 0, R, 2R, ... of its sequence and
 * the following R - 1 pages come from the same run, so that R consecutive
 * logical pages are physically adjacent however fragmented the pool has
 * become; at most R - 1 pages per slot are held unused.  With 16-token pages
 * R = 2 makes every 32-token step of the attention kernel one contiguous
 * region (with K and V side by side: 2 * Hkv * 32 * D * 2 bytes), which DRAM
 * serves 3-4 % faster than two scattered pages.  roll_kv_free_pages counts
 * the pages of the free runs.
 */
int roll_kv_pool_create(roll_kv_pool** pool, const roll_kv_config* cfg,
                        int32_t* page_table_dev, int32_t* seq_lens_dev);
int roll_kv_pool_destroy(roll_kv_pool* pool);

/*
 * HOST state only.  Grow slot's sequence by n_tokens (>= 1), taking pages
 * from the free stack when a page boundary is crossed.  A slot with length
 * 0 becomes live (ADD / refill).  All-or-nothing: on ROLL_ERR_NO_PAGES or
 * ROLL_ERR_SEQ_TOO_LONG nothing has changed.
 */
int roll_kv_alloc(roll_kv_pool* pool, int32_t slot, int32_t n_tokens);

/*
 * HOST state only.  roll_kv_alloc for count distinct slots in one call (the
 * per-step "every live row grows by one token").  slots and n_tokens are HOST
 * arrays of count entries.  All-or-nothing over the whole batch: on any error
 * (a repeated slot is ROLL_ERR_INVALID_ARG) nothing has changed.
 */
int roll_kv_alloc_batch(roll_kv_pool* pool, const int32_t* slots,
                        const int32_t* n_tokens, int32_t count);

/*
 * HOST state only.  Finish or ABORT: every page of the slot goes back on
 * the free stack and its length becomes 0 (the KV of an aborted request is
 * discarded and recomputed later, Section 4.2).  ROLL_ERR_SLOT_EMPTY if the
 * slot holds nothing.
 */
int roll_kv_release(roll_kv_pool* pool, int32_t slot);

/*
 * Publish every change made since the last commit to page_table_dev and
 * seq_lens_dev, as one small block of pinned host memory that one scatter
 * kernel, enqueued on stream, reads.  Work enqueued on the same stream
 * afterwards sees the new tables.  The call does not wait for the stream, with
 * one exception: the pool owns a ring of 8 such blocks, and a host that is 8
 * commits ahead of the GPU waits (hipEventSynchronize) for the oldest block to
 * have been consumed before it reuses it.
 */
int roll_kv_commit(roll_kv_pool* pool, void* stream);

/*
 * roll_kv_commit and, in the same kernel launch, the K/V append of a decode
 * step: the vectors k_new[slot], v_new[slot] are written at the last position
 * (seq_len - 1) of every slot that holds a sequence; empty slots are skipped.
 * The target page of each slot is taken from the pool's host state, so the
 * write does not depend on the device tables being published first.
 *   k_new, v_new    DEVICE bf16 [num_slots, num_kv_heads, head_dim], row-major
 *   k_pages,v_pages DEVICE bf16 pools of cfg.num_pages pages
 *   page_stride     elements between pages (0 = dense), see the top of this header
 */
int roll_kv_commit_append(roll_kv_pool* pool, const void* k_new, const void* v_new,
                          void* k_pages, void* v_pages, int32_t num_kv_heads,
                          int32_t head_dim, int64_t page_stride, void* stream);

/* HOST introspection. */
int roll_kv_free_pages(const roll_kv_pool* pool);               /* count, or < 0 */
int roll_kv_seq_len(const roll_kv_pool* pool, int32_t slot);    /* tokens, or < 0 */
/* Copies up to cap page ids of the slot to pages_out (HOST); returns the
 * number of pages the slot owns, or < 0. */
int roll_kv_slot_pages(const roll_kv_pool* pool, int32_t slot,
                       int32_t* pages_out, int32_t cap);
/* Decode steps that roll_decode_step_attn published in its single launch
 * (the others took the two-launch route), or < 0. */
int64_t roll_kv_fused_steps(const roll_kv_pool* pool);

/*
 * Write the K/V vectors of n_tokens tokens into the paged pools in the page
 * layout given at the top of this header.  Token i goes to position
 * positions[i] of the sequence in slot slots[i]; the page is looked up in
 * page_table on the device, so a roll_kv_commit covering that position must
 * precede this call on the same stream.  The decode step appends one token
 * per live row (positions[i] = seq_len - 1); a refilled prompt writes all
 * its tokens with one call.
 *   k_new, v_new   DEVICE bf16 [n_tokens, num_kv_heads, head_dim], row-major
 *   slots          DEVICE int32 [n_tokens], or NULL for slot i = i
 *   positions      DEVICE int32 [n_tokens] (entries < 0 are skipped), or NULL
 *                  for "the last token of the slot": seq_lens[slot] - 1
 *   seq_lens       DEVICE int32 [num_slots]; read only when positions is NULL
 *   k_pages,v_pages DEVICE bf16 pools
 *   page_table     DEVICE int32 [num_slots, max_pages_per_seq]
 *   page_stride    elements between pages (0 = dense), see the top of this header
 */
int roll_kv_append_tokens(const void* k_new, const void* v_new,
                          const int32_t* slots, const int32_t* positions,
                          const int32_t* seq_lens,
                          int32_t n_tokens, void* k_pages, void* v_pages,
                          const int32_t* page_table, int32_t max_pages_per_seq,
                          int32_t num_pages, int32_t page_size,
                          int32_t num_kv_heads, int32_t head_dim, int64_t page_stride, void* stream);

/* ------------------------------------------------------------------ */
/* Paged GQA decode attention (the bandwidth-bound part of the step,   */
/* Section 1).  For every row b with L = seq_lens[b] >= 1 and query    */
/* head h (KV head h / (Hq/Hkv)):                                      */
/*   s_j = scale * <q[b,h,:], K_j>,  p = softmax_j(s),  j in [0, L)    */
/*   out[b,h,:] = sum_j p_j V_j                                        */
/* seq_lens counts the token being decoded: its K/V is appended before */
/* the call, so no mask is needed.  Rows with L == 0 give zeros.       */
/* ------------------------------------------------------------------ */

typedef struct roll_attn_desc {
    int32_t batch;              /* B rows of q / page_table / seq_lens / out; <= 8192, B * Hkv <= 65536 */
    int32_t num_q_heads;        /* Hq */
    int32_t num_kv_heads;       /* Hkv; Hq % Hkv == 0 and Hq / Hkv <= 16 */
    int32_t head_dim;           /* D: 64 or 128 */
    int32_t page_size;          /* P: 16, 32 or 64 */
    int32_t max_pages_per_seq;  /* row length of page_table */
    int32_t num_pages;          /* pages in each pool (bounds the page ids) */
    int32_t out_dtype;          /* ROLL_BF16 or ROLL_F32 */
    float softmax_scale;        /* 0 => 1 / sqrt(D) */
    int64_t page_stride;        /* elements between pages of a pool; 0 = dense (Hkv * P * D) */
} roll_attn_desc;

/* HOST. Bytes of DEVICE workspace roll_decode_attn needs for this desc. */
size_t roll_decode_attn_workspace_bytes(const roll_attn_desc* desc);

/*
 * HOST, introspection for tests and schedulers: how roll_decode_attn would
 * cut a batch with these lengths across `workgroups` persistent workgroups
 * (a launch uses one per compute unit).  The rows' 32-token steps, laid end
 * to end, are cut into ranges that are equal in cost, a row counting one step
 * more than it has (what starting a row costs a wave); range c owns the steps
 * first_step_out[c] .. first_step_out[c + 1] - 1.  Arithmetic shared with the
 * kernel.  Long-tailed lengths: Section 1 of the paper.
 *   seq_lens_host   HOST int32 [B], clamped as the kernel clamps them
 *   first_step_out  HOST int32 [capacity]; num_ranges + 1 entries are written
 *   num_ranges_out  HOST; written also when capacity is too small (then the
 *                   call returns ROLL_ERR_INVALID_ARG and writes nothing else)
 * Touches no device.
 */
int roll_decode_attn_ranges(const roll_attn_desc* desc, const int32_t* seq_lens_host, int32_t workgroups,
                            int32_t* first_step_out, int32_t capacity, int32_t* num_ranges_out);

/*
 * Prepare a workspace: enqueues a kernel on stream that zeroes the arrival
 * counters at its start and writes a tag word that marks the buffer as
 * prepared.  Call once after allocating the buffer (and again if anything else
 * has written to it, or after a call that failed on the device); every
 * roll_decode_attn leaves the counters zero again.  A workspace prepared once
 * serves any later desc it is large enough for.
 * The attention kernel reads the tag before it writes anything: on a buffer
 * that was never prepared it leaves `out`, the pools and the tables untouched
 * and records the refusal in the workspace, where roll_decode_attn_workspace_check
 * finds it.
 */
int roll_decode_attn_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/*
 * Diagnostic, SYNCHRONISES: waits for stream, then inspects the workspace header.
 * ROLL_OK if the buffer is prepared, no launch has refused it and every arrival
 * counter is zero (as between any two calls); ROLL_ERR_WORKSPACE otherwise, the
 * message saying which: never prepared, refused by a launch (whose results were
 * therefore not written), or counters left over from a launch that did not
 * finish.  Prepare the buffer again after any of these.
 */
int roll_decode_attn_workspace_check(const void* workspace, size_t workspace_bytes, void* stream);

/*
 *   q           DEVICE bf16 [B, Hq, D]
 *   k_pages     DEVICE bf16 [num_pages, Hkv, D/8, P, 8], pages desc->page_stride apart
 *   v_pages     DEVICE bf16 [num_pages, Hkv, P/8, D, 8], likewise
 *   page_table  DEVICE int32 [B, max_pages_per_seq]; entries past a row's
 *               last page are never read
 *   seq_lens    DEVICE int32 [B]; values outside [0, max_pages*P] are
 *               clamped into that range
 *   out         DEVICE [B, Hq, D] of out_dtype
 *   workspace   DEVICE, 256-byte aligned, >= roll_decode_attn_workspace_bytes,
 *               prepared with roll_decode_attn_workspace_init
 * All pointers 16-byte aligned.  Enqueues one kernel on stream: the persistent
 * stream-K attention kernel, which also merges the rows it cut across workgroups.
 * The workspace size does not depend on the sequence lengths.  Two calls that
 * share a workspace must be ordered on one stream.
 */
int roll_decode_attn(const void* q, const void* k_pages, const void* v_pages,
                     const int32_t* page_table, const int32_t* seq_lens,
                     void* out, const roll_attn_desc* desc,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * roll_decode_attn for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and kernel as roll_decode_attn; the
 * scratch for the pieces of cut rows is a buffer inside the library's device
 * image (48 MiB, held on every GPU the library runs on until the process ends).
 * The call allocates nothing and frees nothing.  A shape whose scratch does not
 * fit (it grows with num_kv_heads * num_q_heads / num_kv_heads * head_dim; the
 * 7B- and 32B-class shapes of this header's benchmarks need 15 and 34 MiB) is
 * refused with ROLL_ERR_WORKSPACE before anything is launched.  The first call
 * on a device also enqueues, on stream and ahead of the attention kernel, the
 * small kernel that prepares the buffer.  All calls on one GPU share that
 * GPU's buffer: calls that overlap on one GPU race, so order them (one stream,
 * or events between streams).
 */
int roll_decode_attn_static(const void* q, const void* k_pages, const void* v_pages,
                            const int32_t* page_table, const int32_t* seq_lens,
                            void* out, const roll_attn_desc* desc, void* stream);

/*
 * One launch for the memory-side of a decode step (Section 4.2, the engine's
 * step over the whole running batch): what roll_kv_commit_append followed by
 * roll_decode_attn on the pool's own device tables would do.  Publishes the
 * allocator changes made since the last commit, writes the newest token of
 * every live slot (k_new / v_new, DEVICE bf16 [num_slots, Hkv, D]) into the
 * pages, and attends over all tokens including that one, which is taken from
 * k_new / v_new directly.
 *   pool        created with device tables; desc->batch, page_size,
 *               max_pages_per_seq and num_pages must equal the pool's
 *   k_pages, v_pages  DEVICE, written (one token per live slot) and read
 *   q, out, desc, workspace  as for roll_decode_attn
 * The single launch applies when the changes since the last commit are exactly
 * one decode step: every live slot grew by one token, empty slots stayed
 * empty, and at most 128 slots started a new page.  Anything else (refills,
 * releases, the first use of a pool) is still handled, by the two launches
 * named above, with the same results.  HOST-side effects are those of
 * roll_kv_commit.  Errors as for the two calls it replaces.
 */
int roll_decode_step_attn(roll_kv_pool* pool, const void* k_new, const void* v_new, const void* q,
                          void* k_pages, void* v_pages, void* out, const roll_attn_desc* desc,
                          void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------ */
/* Chunked prefill attention into pages (Section 4.2: a request that   */
/* joins the running batch, or a slot refilled by queue scheduling,    */
/* Section 5.1.1, is prefilled before it is decoded step by step).     */
/* Chunk c is the n_c = chunk_offset[c+1] - chunk_offset[c] consecutive */
/* tokens of slot chunk_slot[c] at positions chunk_start[c] + j.       */
/*   1. every chunk token's K/V is written into the slot's pages;      */
/*   2. token (c, j) attends causally over its slot's positions        */
/*      0 .. chunk_start[c] + j (tokens cached before the chunk and    */
/*      the chunk itself): out = softmax(scale * q K^T) V.             */
/* ------------------------------------------------------------------ */
typedef struct roll_prefill_desc {
    int32_t num_chunks;         /* C >= 0                                 */
    int32_t num_tokens;         /* T = chunk_offset[C] >= 0               */
    int32_t num_q_heads;        /* Hq, a multiple of num_kv_heads         */
    int32_t num_kv_heads;       /* Hkv                                    */
    int32_t head_dim;           /* D: 64 or 128                           */
    int32_t page_size;          /* P: 16, 32 or 64                        */
    int32_t max_pages_per_seq;  /* row stride of page_table               */
    int32_t num_pages;          /* pages in the pools                     */
    int32_t num_slots;          /* rows of page_table                     */
    int32_t out_dtype;          /* ROLL_BF16 or ROLL_F32                  */
    float   softmax_scale;      /* 0 = 1/sqrt(head_dim)                   */
    int64_t page_stride;        /* elements between pages; 0 = dense      */
} roll_prefill_desc;

/*
 *   q                DEVICE bf16 [T, Hq, D], chunks back to back
 *   k_new, v_new     DEVICE bf16 [T, Hkv, D]
 *   chunk_slot       DEVICE int32 [C]
 *   chunk_start      DEVICE int32 [C]  tokens the slot holds before the chunk
 *   chunk_offset     DEVICE int32 [C + 1], non-decreasing, chunk_offset[0] = 0
 *   k_pages, v_pages DEVICE bf16 pools in the layouts of roll_decode_attn; written
 *   page_table       DEVICE int32 [num_slots, max_pages_per_seq]; must already map
 *                    every position of every chunk (roll_kv_alloc + roll_kv_commit)
 *   out              DEVICE [T, Hq, D] of out_dtype
 * q, k_new, v_new, the pools and out 16-byte aligned.  Chunks of one call must
 * not overlap in (slot, position); several chunks of one slot are fine.  A
 * chunk whose slot or positions are out of range is skipped (nothing written
 * for it, its rows of out unspecified).  Enqueues two kernels on stream: the
 * writer of the chunk tokens, then the attention.  The device sequence lengths
 * of the allocator are not read: the chunk arrays say how far each token sees.
 */
int roll_prefill_attn(const void* q, const void* k_new, const void* v_new,
                      const int32_t* chunk_slot, const int32_t* chunk_start,
                      const int32_t* chunk_offset, void* k_pages, void* v_pages,
                      const int32_t* page_table, void* out,
                      const roll_prefill_desc* desc, void* stream);

/* ------------------------------------------------------------------ */
/* Sampling with log-prob recording (Appendix A.1).  Per row r:        */
/*   z_i = logits[r,i] / temperature                                   */
/*   kept = all i                       if top_p >= 1                  */
/*        = { i : logits[r,i] >= x_cut } otherwise, x_cut = the first  */
/*          value, going down the distinct logit values, at which the  */
/*          mass of softmax(z) on values >= it reaches top_p           */
/*   u_i  = uniform from Philox4x32-10, key = philox_seed,             */
/*          counter = (i >> 2, row_id, step_lo, step_hi), word i & 3,  */
/*          u = ((word >> 9) + 0.5) * 2^-23                            */
/*   token   = argmax_{i in kept} z_i - log(-log u_i)   (lowest i wins */
/*             exact ties)                                             */
/*   logprob = z_token - log sum_{i in kept} exp(z_i)                  */
/* At temperature 1 and top_p 1 (the setting the paper enforces) the   */
/* log-prob is log_softmax(logits)[token], the behaviour-policy        */
/* probability that the truncated importance weight divides by.        */
/* ------------------------------------------------------------------ */

typedef struct roll_sample_desc {
    int32_t batch;          /* B rows */
    int32_t vocab;          /* V */
    int64_t row_stride;     /* elements between rows of logits (>= V) */
    int32_t logits_dtype;   /* ROLL_BF16 or ROLL_F32 */
    int32_t policy_version; /* version n of the weights that produced these logits */
    const int32_t* row_ids; /* DEVICE int32 [B] Philox row ids, or NULL for 0..B-1 */
    float* raw_logprob_out; /* DEVICE fp32 [B] or NULL: log_softmax(logits)[token] at temperature 1
                             * with no truncation, for the token that was drawn.  Appendix A.1 forces
                             * temperature 1 and top_p 1 because an engine returns one distribution
                             * only; with both values recorded any sampling setting keeps the raw
                             * probability available to the trainer. */
    int32_t* policy_version_out; /* DEVICE int32 [B] or NULL: policy_version, written beside every
                             * log-prob.  A trajectory that was aborted and resumed (Section 4.2) holds
                             * tokens of several policy versions; the per-token tag tells the trainer
                             * which pi_old each recorded log-prob belongs to, and the oldest tag of a
                             * sample is what the asynchronous-ratio freshness rule bounds. */
} roll_sample_desc;

size_t roll_sample_logprob_workspace_bytes(const roll_sample_desc* desc);

/*
 *   logits       DEVICE [B, row_stride] bf16 or fp32, 16-byte aligned rows
 *   temperature  > 0
 *   top_p        in (0, 1]
 *   tokens_out   DEVICE int32 [B]
 *   logprob_out  DEVICE fp32 [B]
 * Entries of -inf are masked tokens (probability 0).  A row without any finite entry has no
 * distribution to draw from: its token is -1 and its log-probs are NaN.
 */
int roll_sample_logprob(const void* logits, float temperature, float top_p,
                        uint64_t philox_seed, uint64_t step,
                        int32_t* tokens_out, float* logprob_out,
                        const roll_sample_desc* desc,
                        void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------ */
/* Consumer of logprob_out: the off-policy objectives of Section 3.2   */
/* and the truncated importance weight of Appendix A.1, per token of a */
/* batch of ragged responses.  With r = pi_theta / pi_old (pi_old = the */
/* rollout's recorded probability), R the learning signal (reward or    */
/* advantage) and clip(x, lo, hi):                                      */
/*   PPO            min(R r, R clip(r, 1 - eps_low, 1 + eps_high))      */
/*   DECOUPLED_PPO  min(R r, R (pi_prox / pi_old)                       */
/*                          clip(pi_theta / pi_prox, 1 - eps_low, 1 + eps_high)) */
/*   TIS            sg(clip(r, 0, c)) R log pi_theta                    */
/*   CISPO          sg(clip(r, 1 - eps_low, 1 + eps_high)) R log pi_theta */
/*   TOPR           (R > 0 ? 1 : sg(clip(r, 0, c))) R log pi_theta      */
/* sg() terms carry no derivative.                                      */
/* ------------------------------------------------------------------ */

typedef enum roll_loss_kind {
    ROLL_LOSS_PPO = 0, ROLL_LOSS_DECOUPLED_PPO = 1, ROLL_LOSS_TIS = 2, ROLL_LOSS_CISPO = 3, ROLL_LOSS_TOPR = 4
} roll_loss_kind;

typedef struct roll_loss_desc {
    int32_t kind;      /* roll_loss_kind */
    int32_t num_seqs;  /* responses in the batch */
    float eps_low;     /* lower clip offset (PPO, Decoupled PPO, CISPO) */
    float eps_high;    /* upper clip offset */
    float c;           /* truncation threshold (TIS, TOPR, is_weight_out) */
} roll_loss_desc;

/* HOST. Bytes of DEVICE workspace roll_policy_loss needs (partial sums of the responses that are
 * spread over several waves); 0 for a bad desc. */
size_t roll_policy_loss_workspace_bytes(const roll_loss_desc* desc);

/*
 * All pointers DEVICE.  Tokens of response s are seq_offsets[s] .. seq_offsets[s+1]-1.
 *   logp_theta, logp_old, signal  fp32 [T]; logp_prox fp32 [T] (Decoupled PPO only, else NULL)
 *   seq_offsets    int64 [num_seqs + 1], non-decreasing, seq_offsets[0] = 0
 *   value_out      fp32 [T] or NULL: the objective per token
 *   grad_out       fp32 [T] or NULL: its derivative with respect to log pi_theta
 *   is_weight_out  fp32 [T] or NULL: min(pi_theta / pi_old, c)
 *   seq_mean_out   fp32 [num_seqs]: (1/|o|) sum_t value (0 for an empty response)
 *   batch_mean_out fp32 [1]: mean of seq_mean_out over the non-empty responses
 *   workspace      8-byte aligned, >= roll_policy_loss_workspace_bytes; needs no preparation;
 *                  two calls that share it must be ordered on one stream
 * Enqueues two kernels on stream.  The batch's tokens are dealt to the waves in equal shares
 * whatever the lengths of the responses, so a long-tailed batch runs as fast as an even one.
 */
int roll_policy_loss(const float* logp_theta, const float* logp_old, const float* logp_prox,
                     const float* signal, const int64_t* seq_offsets, float* value_out,
                     float* grad_out, float* is_weight_out, float* seq_mean_out,
                     float* batch_mean_out, const roll_loss_desc* desc,
                     void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------ */
/* SampleBuffer with the asynchronous ratio (Section 4.3), HOST only.  */
/* alpha = largest allowed gap between the current policy version n and */
/* the version that initiated a sample.  A sample is outstanding from   */
/* begin until a batch takes it; one batch is taken per version.        */
/* Guarantees, for any interleaving of the calls: at most               */
/* floor((1 + alpha) * batch) samples outstanding;                      */
/* every sample taken at version n was initiated at a version >= n -    */
/* alpha; every sample begun is eventually taken (none is dropped).     */
/* Not thread-safe: one controller thread calls it.                     */
/* ------------------------------------------------------------------ */

typedef struct roll_sample_buffer roll_sample_buffer;

int roll_sample_buffer_create(roll_sample_buffer** buffer, int32_t batch_size, double alpha);
int roll_sample_buffer_destroy(roll_sample_buffer* buffer);
/* Start generating a new sample under the current version.  ROLL_ERR_BUFFER_FULL when the
 * earliest batch that could take it lies more than alpha versions ahead (with alpha = 0:
 * while the trainer runs, or once a batch worth of samples is outstanding). */
int roll_sample_buffer_begin(roll_sample_buffer* buffer, int64_t* ticket, int64_t* init_version);
/* Generation finished; payload is the caller's handle of the trajectory. */
int roll_sample_buffer_complete(roll_sample_buffer* buffer, int64_t ticket, uint64_t payload);
/* ABORT (Section 4.2): the running request is interrupted and reclaimed; it stays outstanding
 * with its initiating version and is resumed later, possibly under a newer policy. */
int roll_sample_buffer_abort(roll_sample_buffer* buffer, int64_t ticket);
int roll_sample_buffer_resume(roll_sample_buffer* buffer, int64_t ticket, int64_t* version_now);
/* One training batch: batch_size samples, those that cannot wait another version first, then
 * the oldest.  ROLL_ERR_WOULD_BLOCK if fewer are complete or a due sample is still generating.
 * tickets / init_versions / payloads: HOST arrays of batch_size entries (the last two may be NULL). */
int roll_sample_buffer_take_batch(roll_sample_buffer* buffer, int64_t* tickets, int64_t* init_versions,
                                  uint64_t* payloads);
/* After the train step: n -> n + 1.  ROLL_ERR_WOULD_BLOCK while a sample would become too old. */
int roll_sample_buffer_advance_version(roll_sample_buffer* buffer);
int64_t roll_sample_buffer_version(const roll_sample_buffer* buffer);
int64_t roll_sample_buffer_outstanding(const roll_sample_buffer* buffer);
int64_t roll_sample_buffer_capacity(const roll_sample_buffer* buffer);

/* ------------------------------------------------------------------ */
/* Profiling helpers: HIP events around the attention kernel.          */
/* ------------------------------------------------------------------ */
/* HOST, per calling thread: the next roll_decode_attn / roll_decode_step_attn
 * launches made by this thread record `begin` right before and `end` right
 * after the stream-K attention kernel, on the launch's stream (hipEvent_t
 * handles from roll_prof_event_create).  NULL, NULL switches it off again. */
int roll_prof_attn_events(void* begin, void* end);
/* The same for roll_prefill_attn: the events bracket its attention kernel (the
 * launch after the K/V writer). */
int roll_prof_prefill_events(void* begin, void* end);
/*
 * A prefill workgroup computes U units, one per wave, where a unit is (span of 32
 * query tokens of a chunk, query head of the KV head's group) and a chunk's units
 * are dealt out span after span.  U is chosen per launch from its size (7
 * computing waves and a copying one for a large launch with a bf16 result, fewer
 * for a small one); this fixes it for the calling thread's roll_prefill_attn
 * calls: units = 1 .. 8, or 0 for the choice per launch (for tests and
 * measurements; results are the same to rounding order).  HOST;
 * ROLL_ERR_INVALID_ARG for any other value.
 */
int roll_prof_prefill_units(int32_t units);
/*
 * Per-wave timestamps of the attention kernel, for a library built with
 * -DROLL_ATTN_TIMELINE only (the product build returns ROLL_ERR_INVALID_ARG).
 * buffer: DEVICE, 8-byte aligned, >= 1024 waves * 8 * 8 bytes, or NULL to switch
 * it off.  Every wave of the following attention launches writes 8 words:
 * the 100 MHz clock at entry, after the row prefix, after its first step,
 * after its last step, at exit; the steps it ran; its XCD; its streams.
 * SYNCHRONISES (a copy to a device symbol).
 */
int roll_prof_attn_timeline(void* buffer, size_t buffer_bytes);
/*
 * Per-workgroup timestamps of the prefill attention kernel, for a library built
 * with -DROLL_ATTN_TIMELINE only (the product build returns ROLL_ERR_INVALID_ARG).
 * buffer: DEVICE, 8-byte aligned, 64 bytes per workgroup to record (workgroups
 * numbered at or above buffer_bytes / 64 record nothing), or NULL to switch it
 * off.  Wave 0 of every workgroup of the following roll_prefill_attn launches
 * that takes the pipelined loop (bf16 result, up to 8 query heads per KV head)
 * writes 8 words: the 100 MHz clock at entry, with its block found, before its
 * first and after its last loop iteration, after its stores; XCC_ID << 32 |
 * HW_ID; its steps; 1.  SYNCHRONISES (copies to device symbols).
 */
int roll_prof_prefill_timeline(void* buffer, size_t buffer_bytes);
/*
 * Bandwidth ceiling of the decode step's access pattern (Section 1: decoding is
 * memory-bandwidth bound): enqueues ONE kernel that reads, through page_table,
 * the K block and the V block (all KV heads) of every page that holds tokens of
 * a row (ceil(seq_lens[b] / page_size) pages of row b), with streaming 16-byte
 * loads and no arithmetic.  Arguments as for roll_decode_attn (desc: batch,
 * num_kv_heads, head_dim, page_size, max_pages_per_seq, num_pages, page_stride).
 *   sink            DEVICE, >= 2048 * 256 * 4 bytes; receives one meaningless word per thread
 *   bytes_per_page  HOST, optional: bytes the kernel reads per page (K + V block)
 * The caller times the launch; bytes read = bytes_per_page * sum_b ceil(L_b / P).
 */
int roll_prof_kv_read_probe(const void* k_pages, const void* v_pages, const int32_t* page_table,
                            const int32_t* seq_lens, const roll_attn_desc* desc, void* sink,
                            size_t sink_bytes, int64_t* bytes_per_page, void* stream);
int roll_prof_event_create(void** event);
int roll_prof_event_destroy(void* event);
int roll_prof_event_record(void* event, void* stream);
/* Waits for end, then writes the milliseconds between the two events. */
int roll_prof_event_elapsed_ms(void* begin, void* end, float* ms);

#ifdef __cplusplus
}
#endif
#endif /* ROLL_DECODE_H */
