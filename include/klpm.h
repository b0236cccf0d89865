/*
 * klpm.h - C ABI of the GPU-resident k-LPM scheduling step (MI355X / gfx950).
 *
 * One scheduling step of the k-LPM scheduler over a RadixAttention-style prefix cache:
 *   match  : for every waiting query, the longest prefix of its prompt already held in the cache
 *   select : the k-LPM batch (Algorithm 1), FCFS and LPM being its k = 1 and k = infinity endpoints
 *   commit : insert the admitted prompts into the radix tree, then LRU-evict down to the KV budget
 *
 * Conventions for every entry point
 *   - Pointers marked DEVICE point to GPU memory owned by the caller; HOST pointers are ordinary
 *     host memory.  The library never allocates or frees device memory: the tree lives inside an
 *     arena the caller provides and keeps alive until kLPM_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call only
 *     enqueues work on that stream and returns; outputs are valid once the stream has been
 *     synchronised.  Only kLPM_snapshot / kLPM_snapshot_bytes / kLPM_read_stats synchronise.
 *   - Return value: KLPM_OK or a negative KLPM_E* code.  Conditions only the device can see
 *     (capacity exhausted, malformed offsets) set bits in the tree's sticky device_error word,
 *     reported through kLPM_stats; the failing commit leaves the tree as it was before the call.
 *   - Calls that use the same tree must be issued on one stream (or be externally ordered).
 */
#ifndef KLPM_H
#define KLPM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KLPM_OK 0
#define KLPM_EINVAL (-1) /* NULL pointer, negative count, inconsistent configuration */
#define KLPM_EARENA (-2) /* arena or workspace too small / misaligned */
#define KLPM_EHIP (-3)   /* a HIP runtime call or kernel launch failed */
#define KLPM_ENOMEM (-4) /* host allocation failed */
#define KLPM_ELIMIT (-5) /* input larger than the fixed maximum of an entry point that brings its own scratch memory */

/* bits of kLPM_stats.device_error */
#define KLPM_DEV_NODES_FULL 1u     /* not enough free node slots for the batch */
#define KLPM_DEV_POOL_FULL 2u      /* edge-token pool cannot take the batch even after compaction */
#define KLPM_DEV_BAD_INPUT 4u      /* a prompt offset/length outside the token buffer or limits */
#define KLPM_DEV_BATCH_OVERFLOW 8u /* *n_selected larger than the capacity given to kLPM_commit */
#define KLPM_DEV_CLOCK_RANGE 16u   /* more prompts admitted than the launch sequence was sized for
                                      (see kLPM_reserve_clock); that commit evicted nothing */
#define KLPM_DEV_INTERNAL 32u      /* the tree and its child table disagree (memory overwritten from outside,
                                      or a defect of the library): the tree is no longer usable */

/* k value that encodes k = infinity (pure longest-prefix-match order); k = 0 means the same. */
#define KLPM_K_INFINITY 0xFFFFFFFFu

typedef void *kLPM_stream;
typedef struct kLPM_tree kLPM_tree; /* opaque host-side handle */

/* A query stream (x_i, t_i), i in [n] (Def. 1): token strings in CSR form plus arrival ticks. */
typedef struct {
    const int32_t *tokens;   /* DEVICE [n_tokens] token pool */
    const int64_t *off;      /* DEVICE [n] start of prompt i in `tokens` */
    const int32_t *len;      /* DEVICE [n] prompt length, 1 <= len <= max_prompt_len */
    const uint64_t *arrival; /* DEVICE [n] arrival time t_i in integer ticks (may be NULL where unused) */
    int64_t n_tokens;        /* size of `tokens`, used for bounds checks */
    int32_t n;               /* number of queries (HOST value; launches are sized for it) */
    const int32_t *n_live;   /* DEVICE [1] or NULL.  When given, only the first
                                min(n, max(0, *n_live)) queries exist: a queue whose length is decided
                                on the device is passed with n = its capacity, and no step of the
                                scheduling loop needs the host to read the length back */
} kLPM_queries;

typedef struct {
    int64_t budget_tokens;  /* KV budget: eviction brings the cached token total down to <= this */
    int64_t pool_tokens;    /* capacity of one half of the edge-token pool (two halves are kept);
                               must hold what stays cached (the budget, or the initial cache if
                               larger) plus one worst-case batch of max_batch * max_prompt_len tokens:
                               the end of a commit compacts the pool when less than that is left */
    int32_t max_nodes;      /* node slots, root included */
    int32_t max_batch;      /* most prompts one kLPM_commit may admit (<= 65536) */
    int32_t max_prompt_len; /* longest prompt accepted */
    uint32_t flags;         /* reserved, 0 */
} kLPM_config;

typedef struct {
    int64_t total_tokens;    /* tokens held by the tree after the call */
    int64_t inserted_tokens; /* new tokens added by this commit */
    int64_t evicted_tokens;  /* tokens removed by this commit */
    int32_t n_nodes;         /* non-root nodes after the call */
    int32_t new_nodes;       /* nodes created by this commit (leaves and splits) */
    int32_t evicted_nodes;
    uint32_t device_error;   /* sticky KLPM_DEV_* bits */
    uint64_t clock;          /* logical LRU clock = prompts admitted so far */
} kLPM_stats;

/* Bytes of device memory the arena needs for `cfg`. */
int kLPM_arena_bytes(const kLPM_config *cfg, size_t *out_bytes);

/*
 * Build the prefix cache (RadixAttention radix tree, Sec. 1) inside `arena` (DEVICE, 256-byte
 * aligned, arena_bytes >= kLPM_arena_bytes) from the prompts already processed.  Equivalent to
 * committing initial[0..n) one by one with ticks 0..n-1 and no eviction; `initial` may be NULL or
 * have n = 0 (the empty cache that Def. 2 starts from).  initial->arrival is ignored.
 * The handle is host memory owned by the library until kLPM_destroy.
 */
int kLPM_build_tree(kLPM_tree **out, const kLPM_config *cfg, void *arena, size_t arena_bytes,
                    const kLPM_queries *initial, kLPM_stream stream);

/*
 * Prefix match of the whole waiting queue: match_len[i] = max over cached strings y of
 * overlap(x_i, y), the length of the maximal common prefix (Sec. 1.2 Notation), token-granular,
 * 0 <= match_len[i] <= len[i].  Read-only on the tree (recency is only touched by commit).
 *   match_len  DEVICE [q->n] out (entries at or beyond *q->n_live are left untouched)
 *   last_node  DEVICE [q->n] out or NULL: opaque id of the deepest node whose edge was entered
 * A query whose span falls outside q->tokens gets match_len = -1 and sets KLPM_DEV_BAD_INPUT.
 */
int kLPM_match(kLPM_tree *tree, const kLPM_queries *q, int32_t *match_len, int32_t *last_node,
               kLPM_stream stream);

/* kLPM_select flag: the caller asserts that arrival[] is non-decreasing in the queue index (a queue
 * kept in arrival order).  Selection then needs no sort of the whole queue (one kernel for up to
 * 8,192 entries, five short ones beyond).  The assertion is checked on the
 * device; if it does not hold, *n_selected is set to -1, nothing is selected and the phase is kept.
 * Two cases sort the queue all the same, and there the flag is only a hint - the promise is neither
 * needed nor checked and the result is the correct batch whatever the arrival order: a tie_key with
 * n <= 4096, and min(batch, n) > 4096. */
#define KLPM_SELECT_FIFO 1u

/* Workspace size for kLPM_select over n waiting queries. */
int kLPM_select_workspace_bytes(int32_t n, size_t *out_bytes);

/*
 * k-LPM batch selection (Algorithm 1, with the processing order cut into bins of B, Sec. 2.1).
 * Slot j of the batch is the oldest remaining query if (phase + j) mod k == 0, otherwise the
 * remaining query with the longest match; ties go to the earlier arrival, then the lower index.
 * k = 1 is FCFS; k = 0 or KLPM_K_INFINITY is pure LPM order (Sec. 4).
 *   arrival, match_len  DEVICE [n] in (a negative match_len counts as 0).  match_len is the score of
 *                       the longest-match picks: the match lengths, or any other int32 score such as
 *                       the hit rate written by kLPM_score_hit_rate
 *   tie_key             DEVICE [n] or NULL: decides between equal scores before the arrival time
 *                       does (smaller key first); kLPM_tie_keys fills it with uniform random numbers
 *                       for the random tie-break that the theory assumes (footnote of Sec. 4.2).
 *                       Oldest picks never look at it
 *   n_live              DEVICE [1] or NULL: as in kLPM_queries, the queue holds min(n, max(0, *n_live))
 *                       entries; n then only sizes the launches and the workspace
 *   k, k_dev            k_dev NULL: k is used.  Otherwise DEVICE [1]: the k that memory holds when
 *                       the selection runs (for a k chosen on the device, see kLPM_adapt_*), and the
 *                       argument k is ignored
 *   flags               0 or KLPM_SELECT_FIFO
 *   max_match           with KLPM_SELECT_FIFO: an upper bound of the match_len values (the longest
 *                       prompt accepted will do); 0 = unknown.  A smaller bound means fewer passes; a
 *                       match_len above it is reported like a broken arrival order (*n_selected = -1)
 *   phase_inout         DEVICE [1]: position in the k-cycle, carried from step to step
 *                       (write 0 before the call to restart the cycle every step)
 *   batch_idx           DEVICE [min(batch, n)] out: queue indices in pick order
 *   n_selected          DEVICE [1] out: min(batch, number of entries)
 *   workspace           DEVICE, >= kLPM_select_workspace_bytes(n), 256-byte aligned; scratch only: its
 *                       contents need not be set before a call and mean nothing after it
 * n = 0 or batch = 0 selects nothing (*n_selected = 0), leaves the phase unchanged and needs no
 * workspace (NULL will do).
 */
int kLPM_select(const uint64_t *arrival, const int32_t *match_len, const uint32_t *tie_key, int32_t n,
                const int32_t *n_live, uint32_t k, const uint32_t *k_dev,
                int32_t batch, uint32_t flags, int32_t max_match, uint32_t *phase_inout, int32_t *batch_idx, int32_t *n_selected,
                void *workspace, size_t workspace_bytes, kLPM_stream stream);

/*
 * kLPM_select for callers that cannot allocate device memory or hand a workspace over: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The arguments and the
 * result are those of kLPM_select without workspace / workspace_bytes; the workspace is a fixed
 * array in the library's own device image (KLPM_SELECT_STATIC_MAX_N * 36 bytes + 1 MiB, about
 * 5.5 MiB, held by every GPU the library runs on until the process ends).  The call allocates
 * nothing and frees nothing.
 *   n > KLPM_SELECT_STATIC_MAX_N returns KLPM_ELIMIT and enqueues nothing.
 *   The first call on a device looks the array's address up (hipGetSymbolAddress); make that call
 *   outside any stream capture.
 *   All calls on one GPU share the one array, whatever their stream: calls that may overlap in time
 *   on a GPU race with each other (keep them on one stream, or order them with events).  Nothing in
 *   the array has to hold a particular value when a call starts; nothing is carried from call to call.
 */
#define KLPM_SELECT_STATIC_MAX_N 131072
int kLPM_select_static(const uint64_t *arrival, const int32_t *match_len, const uint32_t *tie_key, int32_t n,
                       const int32_t *n_live, uint32_t k, const uint32_t *k_dev, int32_t batch, uint32_t flags,
                       int32_t max_match, uint32_t *phase_inout, int32_t *batch_idx, int32_t *n_selected,
                       kLPM_stream stream);

/*
 * k-LPM selection with in-batch rescoring: Algorithm 1 applied to scores that follow the cache
 * inside the bin.  Def. 2 credits a query with its overlap with what was processed before it; with
 * a cache that keeps every processed prompt (Sec. 1) a query picked later in the same bin of B
 * (Sec. 2.1) overlaps with the cached strings and with every prompt picked before it.  After each
 * pick p the score of every remaining query i becomes max(score_i, overlap(x_i, x_p)); each slot
 * is filled by Algorithm 1's rule on the current scores (ties: earlier arrival, lower index).
 * Equivalent to `batch` single-query steps of match -> select -> commit without eviction.
 *   q           the waiting queue, q->arrival required, q->n <= 262144
 *   match_len   DEVICE [q->n] in: match lengths against the cache (kLPM_match)
 *   last_node   DEVICE [q->n] in: the last_node output of the same kLPM_match call
 *   dyn_match   DEVICE [q->n] out: for a picked query its score when it was picked (its overlap
 *               credit: it costs len - dyn_match), for the others their final score
 *   k, k_dev, phase_inout, batch_idx, n_selected   as in kLPM_select
 *   flags, max_match   as in kLPM_select: with KLPM_SELECT_FIFO and a bound max_match > 0 on the match
 *               lengths, a queue of more than 4096 entries is not sorted by arrival and its match
 *               lengths only over the bits the bound needs; a queue that breaks the promise, or a
 *               match length above the bound, gives *n_selected = -1 and leaves the phase alone.
 *               Without them (0, 0) any queue order is accepted
 *   workspace   DEVICE, 256-byte aligned, >= kLPM_select_dynamic_workspace_bytes(q->n)
 */
int kLPM_select_dynamic_workspace_bytes(int32_t n, size_t *out_bytes);
int kLPM_select_dynamic(const kLPM_queries *q, const int32_t *match_len, const int32_t *last_node, uint32_t k,
                        const uint32_t *k_dev, int32_t batch, uint32_t flags, int32_t max_match, uint32_t *phase_inout,
                        int32_t *dyn_match, int32_t *batch_idx, int32_t *n_selected, void *workspace,
                        size_t workspace_bytes, kLPM_stream stream);

/*
 * Prefix-cache hit *rate* (the wording of Algorithm 1) as a score for kLPM_select:
 * score[i] = floor(match_len[i] * 2^scale_bits / len[i]), 1 <= scale_bits <= 30.  It orders the
 * queries exactly like the ratios m/|x| whenever every |x| <= 2^(scale_bits/2); beyond that
 * nearly equal rates may share a score (and then count as tied).  All arrays DEVICE [n].
 */
int kLPM_score_hit_rate(const int32_t *match_len, const int32_t *len, int32_t n, const int32_t *n_live,
                        int32_t scale_bits, int32_t *score, kLPM_stream stream);

/*
 * Uniform 32-bit tie keys, one per query, redrawn for every scheduling step:
 * tie_key[i] = word 0 of Philox-4x32-10 (Salmon et al., SC'11) at counter
 * (id[i], 0, step low, step high) under the key (seed low, seed high); id = NULL uses i itself.
 *   id       DEVICE [n] or NULL     tie_key  DEVICE [n] out
 */
int kLPM_tie_keys(uint64_t seed, uint64_t step, const int32_t *id, int32_t n, const int32_t *n_live,
                  uint32_t *tie_key, kLPM_stream stream);

/*
 * Commit a batch: for each admitted prompt, in pick order, give it the next tick of the logical
 * clock, extend the tree to hold it (splitting an edge where the prompt diverges from it or ends
 * inside it) and stamp the tick on every node of its path; then, while the token total exceeds the
 * budget, remove the least-recently-used leaf (fixed-size cache with LRU eviction, Sec. 1, Sec. 2.1).
 *   batch_idx   DEVICE [batch_cap] indices into q (as written by kLPM_select); entries behind the
 *               first *n_selected may be read but are ignored
 *   n_selected  DEVICE [1] number of valid entries, <= batch_cap <= cfg.max_batch
 *   stats       DEVICE [1] out, or NULL
 * Tokens are copied into the arena, so q's buffers may be recycled once the stream has passed.
 */
int kLPM_commit(kLPM_tree *tree, const kLPM_queries *q, const int32_t *batch_idx, const int32_t *n_selected,
                int32_t batch_cap, kLPM_stats *stats, kLPM_stream stream);

/*
 * kLPM_commit for a caller that has just matched the whole queue: the admitted prompts' prefix
 * matches are taken from that call's results instead of being computed again (within one scheduling
 * step the tree does not change between the match and the commit, Algorithm 1).
 *   match_len, last_node  DEVICE [q->n] as written by kLPM_match for this q on the tree as it is
 *                         now (no commit or budget change with eviction in between)
 * Each entry used is checked against the tree where that is cheap (node alive, match ends inside
 * that node's edge on an equal token, nothing continues it); an entry that fails sets
 * KLPM_DEV_BAD_INPUT and the commit is abandoned.  A stale entry that passes these checks leaves a
 * tree with duplicated paths (never an out-of-bounds access): when in doubt call kLPM_commit.
 * Everything else is as for kLPM_commit.
 */
int kLPM_commit_matched(kLPM_tree *tree, const kLPM_queries *q, const int32_t *match_len, const int32_t *last_node,
                        const int32_t *batch_idx, const int32_t *n_selected, int32_t batch_cap, kLPM_stats *stats,
                        kLPM_stream stream);

/*
 * Eviction protection for prompts in flight: the paths of the `recent_prompts` most recently
 * admitted prompts (the batch of the commit itself included) are never evicted by later commits;
 * eviction then stops early and the token total may stay above the budget (kLPM_stats.total_tokens
 * tells).  0 (the default) protects nothing: plain LRU under the fixed cache size (Sec. 1).
 * Host-side, takes effect at the next kLPM_commit.
 */
int kLPM_set_protect(kLPM_tree *tree, int64_t recent_prompts);

/*
 * Dynamic batch size under a prefill token budget (Sec. 2.1: dynamic batch size with a fixed
 * memory pool): of the picks batch_idx[0 .. *n_selected) keep the longest prefix whose uncached
 * tokens, sum of len - match_len, fit `token_budget`; the first pick always stays.  *n_selected is
 * lowered accordingly and *phase_inout is rewound by the picks handed back, so that the k-cycle
 * continues as if only the kept picks had been made.  Call between kLPM_select and kLPM_commit with
 * the k (and k_dev) that the selection used.  All pointers DEVICE.
 */
int kLPM_batch_token_budget(const kLPM_queries *q, const int32_t *match_len, const int32_t *batch_idx,
                            int32_t *n_selected, int32_t batch_cap, int64_t token_budget, uint32_t k,
                            const uint32_t *k_dev, uint32_t *phase_inout, kLPM_stream stream);

/*
 * Cache slots of a batch's matched prefixes (what the prefix cache returns for attention to read:
 * RadixAttention, Sec. 1).  For pick j (prompt batch_idx[j] of q) and t < n_matched[j],
 * slots[j * stride + t] identifies the cache entry of token t of that prompt: equal prefixes get
 * equal slots, different cached prefixes different ones.  A slot is the position of the token in
 * the tree's token pool; slots stay valid until a commit evicts the entry or compacts the pool, so
 * they are taken after kLPM_match / kLPM_select and used before the next kLPM_commit.
 *   stride     row length, >= the longest match wanted (longer matches are cut at stride)
 *   n_matched  DEVICE [batch_cap] out: matched tokens of pick j (0 beyond *n_selected, -1 bad input)
 *   slots      DEVICE [batch_cap * stride] out
 */
int kLPM_kv_slots(kLPM_tree *tree, const kLPM_queries *q, const int32_t *batch_idx, const int32_t *n_selected,
                  int32_t batch_cap, int32_t stride, int32_t *n_matched, int64_t *slots, kLPM_stream stream);

/* tokens_out[i] = the token held in cache slot slots[i] (-1 for a value that is no slot).  DEVICE arrays [n]. */
int kLPM_gather_slots(kLPM_tree *tree, const int64_t *slots, int64_t n, int32_t *tokens_out, kLPM_stream stream);

/*
 * Every call only enqueues kernels (no memset or copy nodes, no synchronisation), so a scheduling
 * step can be captured into a HIP graph and replayed.  The number of eviction passes a commit
 * enqueues follows from a host-side bound of the LRU clock, which replays do not advance: before
 * capturing, reserve as many admissions as will be replayed (or committed without the host seeing
 * them).  A commit that finds the clock beyond the bound evicts nothing and sets
 * KLPM_DEV_CLOCK_RANGE.  kLPM_read_stats re-reads the clock and renews the bound.
 */
int kLPM_reserve_clock(kLPM_tree *tree, uint64_t extra_prompts);

/* Change the KV budget used by later commits (host-side, takes effect at the next kLPM_commit). */
int kLPM_set_budget(kLPM_tree *tree, int64_t budget_tokens);

/*
 * A device-resident waiting queue kept in arrival order, with the CSR view (off, len) of its
 * prompts inside the token pool of the whole stream.  All pointers DEVICE.
 */
typedef struct {
    int32_t *id;       /* [cap] global query ids */
    uint64_t *arrival; /* [cap] enqueue times */
    int64_t *off;      /* [cap] start of each waiting prompt in the stream's token pool */
    int32_t *len;      /* [cap] prompt lengths */
    int32_t *n;        /* [1]  entries in use */
    uint64_t *clock;   /* [1]  simulated time at which this queue state holds */
    int32_t *n_joined; /* [1]  timed runs: entries of the kLPM_arrivals list that have joined so far
                               (NULL where kLPM_queue_advance_timed is not used) */
    int32_t cap;
} kLPM_queue;

/* Fill q->off / q->len from q->id (off = -1, len = 0 for an id outside `all`). */
int kLPM_queue_gather(const kLPM_queue *q, const kLPM_queries *all, kLPM_stream stream);

/*
 * Waiting-queue bookkeeping of an online run (query stream of Def. 1 served in bins, Sec. 2.1;
 * prefill cost of Def. 2 with c_attn = 0).  Given the batch just selected from `cur`: the simulated
 * time moves from *cur->clock by max(1, sum over the batch of len - match_len); TTFT = new time -
 * arrival is recorded for the admitted entries; `next` (a distinct buffer set: entries, count and
 * clock) receives the surviving entries in their old order followed by the n_new arrivals stamped
 * with the new time, the CSR view of the new queue, its length and the new time.  One launch;
 * nothing of `cur` is written, so the two buffer sets are used in turn.
 *   all         the whole stream's prompts (tokens unused; off/len indexed by global id)
 *   match_len   DEVICE [*cur->n] match lengths of the queue as scored this step
 *   batch_idx   DEVICE [batch_cap]: the first *n_selected entries as written by kLPM_select
 *               (distinct positions in `cur`); the rest is read but ignored
 *   n_selected  DEVICE [1], <= batch_cap
 *   new_id      DEVICE [n_new] global ids of the arrivals joining after this step
 *   ttft        DEVICE [all->n] out (written for admitted ids only)
 *   matched_accum DEVICE [1] or NULL: += sum of match_len over the queue (throughput accounting)
 * Arrivals that do not fit next->cap are dropped and set KLPM_DEV_BATCH_OVERFLOW in *dev_error.
 */
int kLPM_queue_advance(const kLPM_queue *cur, const kLPM_queue *next, const kLPM_queries *all,
                       const int32_t *match_len, const int32_t *batch_idx, const int32_t *n_selected,
                       int32_t batch_cap, const int32_t *new_id, int32_t n_new, int64_t *ttft, int64_t *matched_accum,
                       uint32_t *dev_error, kLPM_stream stream);

/*
 * Arrivals that reach the scheduler at their own times (query stream of Def. 1; the Regular
 * Arrival Shuffled Queue of Def. 3 is one).  All pointers DEVICE.  Times and the simulated clock
 * count units of 1/c_den of one token's linear prefill time.
 */
typedef struct {
    const int32_t *id;    /* [n] global query ids ordered by (arrival time, id) */
    const uint64_t *time; /* [n] their arrival times t_i, non-decreasing */
    int32_t n;
    uint32_t c_num;       /* attention coefficient of Def. 2: c_attn = c_num / c_den */
    uint32_t c_den;       /* >= 1 */
} kLPM_arrivals;

/*
 * The same bookkeeping as kLPM_queue_advance under Def. 2's timeline: the batch costs the sum over
 * its queries of (len - match_len) * (c_den + c_num * len) clock units, i.e.
 * (1 + c_attn |x|)(|x| - overlap) token times each; the clock moves by exactly that; TTFT = new time
 * - arrival time.  Then every pending arrival with time <= clock joins `next` behind the survivors,
 * keeping its own arrival time, as far as next->cap allows (the rest stay pending, in order).  If
 * that leaves the queue empty while arrivals are still pending, the clock jumps to the next
 * arrival time (a query cannot start before it arrives, Def. 2) and the queries arriving then join.
 * How many arrivals have joined is read from *cur->n_joined and left in *next->n_joined; the queue
 * length is left in *next->n for the next step's n_live.  Calling it on an empty queue with
 * *n_selected = 0 performs the initial fill.
 */
int kLPM_queue_advance_timed(const kLPM_queue *cur, const kLPM_queue *next, const kLPM_queries *all,
                             const int32_t *match_len, const int32_t *batch_idx, const int32_t *n_selected,
                             int32_t batch_cap, const kLPM_arrivals *pending, int64_t *ttft, int64_t *matched_accum,
                             uint32_t *dev_error, kLPM_stream stream);

/*
 * Adaptive k.  Sec. 4.2 says that k can be set by back-testing or by an adaptive multi-armed bandit
 * and gives no method; this is the textbook epsilon-greedy rule over a caller's list of k values,
 * with its state in device memory so that a scheduling loop never reads anything back:
 *   - a pull lasts `window` scheduling steps (calls of kLPM_adapt_observe);
 *   - its cost is the largest TTFT among the queries admitted during those steps; a window that
 *     admitted nobody is not a pull and changes nothing;
 *   - after a pull, an arm never pulled goes next (lowest index first); otherwise words w0, w1 of
 *     Philox-4x32-10 at counter (pulls low, pulls high, 0x6B4C504D, 0) under key (seed low, seed high)
 *     decide: arm w1 mod n_arms if w0 < explore (probability explore / 2^32), else the arm with the
 *     smallest mean cost (compared exactly; the lower index on equality).
 *   state    DEVICE, 8-byte aligned, >= kLPM_adapt_state_bytes; owned by the caller, initialised
 *            by kLPM_adapt_init (enqueued on the stream)
 *   k_dev    (kLPM_adapt_k) DEVICE pointer into the state: the current k, to be passed as the
 *            k_dev argument of kLPM_select / kLPM_select_dynamic / kLPM_batch_token_budget
 * kLPM_adapt_observe is called once per scheduling step, after the queue advance that wrote the
 * TTFTs: `served` is the queue the batch was selected from (still intact: the advance writes the
 * other buffer set), batch_idx / n_selected the selection, ttft DEVICE [n_ttft] indexed by query id.
 * An entry that cannot be read (index or id out of range, TTFT < 0) is left out and sets
 * KLPM_DEV_BAD_INPUT in the state.  The sum of an arm's costs must fit 64 bits.
 * kLPM_adapt_read synchronises the stream and copies the counters to HOST memory.
 */
#define KLPM_ADAPT_MAX_ARMS 16
typedef struct kLPM_adapt_config {
    uint32_t arms[KLPM_ADAPT_MAX_ARMS]; /* the k values to choose among (0 or KLPM_K_INFINITY = LPM) */
    int32_t n_arms;                     /* 1 .. KLPM_ADAPT_MAX_ARMS */
    int32_t window;                     /* scheduling steps per pull, >= 1 */
    uint64_t explore;                   /* exploration probability times 2^32, 0 .. 2^32 */
    uint64_t seed;
} kLPM_adapt_config;
typedef struct kLPM_adapt_stats {
    uint64_t count[KLPM_ADAPT_MAX_ARMS]; /* pulls per arm */
    uint64_t cost[KLPM_ADAPT_MAX_ARMS];  /* summed cost per arm */
    uint64_t pulls;
    int32_t arm;                         /* current arm */
    uint32_t k;                          /* its k */
    int32_t steps_in_window;
    uint32_t device_error;
} kLPM_adapt_stats;
int kLPM_adapt_state_bytes(size_t *out_bytes);
int kLPM_adapt_init(void *state, size_t state_bytes, const kLPM_adapt_config *cfg, kLPM_stream stream);
int kLPM_adapt_k(void *state, const uint32_t **k_dev);
int kLPM_adapt_observe(void *state, const kLPM_queue *served, const int32_t *batch_idx, const int32_t *n_selected,
                       int32_t batch_cap, const int64_t *ttft, int32_t n_ttft, kLPM_stream stream);
int kLPM_adapt_read(void *state, kLPM_adapt_stats *host_out, kLPM_stream stream);

/*
 * Measurement helper: one plain streaming read over `bytes` of DEVICE memory at `src` (16-byte
 * aligned).  Nothing is computed; *sink (DEVICE) only keeps the loads alive.  Timing it gives the
 * read bandwidth a kernel can reach on this GPU, the yardstick beside kLPM_match's figures.
 */
int kLPM_probe_read(const void *src, size_t bytes, uint64_t *sink, kLPM_stream stream);

/* Synchronises the stream and copies the tree's counters to HOST memory. */
int kLPM_read_stats(kLPM_tree *tree, kLPM_stats *host_out, kLPM_stream stream);

/*
 * Canonical tree state (synchronises).  Layout of the HOST buffer, little endian:
 *   int64 n_nodes, int64 total_tokens, uint64 clock;
 *   n_nodes records {int32 depth_start, int32 edge_len, uint64 tick, int32 n_children, int32 0}
 *     in depth-first pre-order, children visited by ascending first edge token;
 *   total_tokens int32 edge tokens in the same order.
 * Node ids, pool offsets and hash layout are not part of the state.
 */
int kLPM_snapshot_bytes(kLPM_tree *tree, size_t *out_bytes, kLPM_stream stream);
int kLPM_snapshot(kLPM_tree *tree, void *host_buf, size_t cap, size_t *out_bytes, kLPM_stream stream);

int kLPM_destroy(kLPM_tree *tree);
const char *kLPM_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* KLPM_H */
