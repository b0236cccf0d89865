// Commit: insert the admitted prompts into the flattened radix tree, then LRU-evict to the budget.
//
// The prefix cache keeps what every processed query left behind in a radix tree and evicts the
// least recently used entries under a fixed memory size (Sec. 1; fixed pool, Sec. 2.1).  The serial
// definition is: for each admitted prompt in pick order take the next tick, walk the prompt down
// the tree, split the edge where it diverges or ends, hang the unmatched tail as a new leaf, stamp
// the tick on the path; then repeatedly remove the smallest-tick leaf while over budget.
//
// The device formulation reaches the same tree state in parallel phases:
//   1. match every admitted prompt against the pre-commit tree (the batched match kernel);
//   2. copy every unmatched tail into one freshly reserved block of the token pool;
//   3. structure pass: prompts that stopped at different places of the old tree touch disjoint
//      structure (a split keeps the lower part's id, so an edge's end boundary and its children
//      never move), so one wavefront per "stop place" inserts its prompts serially in pick order
//      while different places proceed concurrently;
//   4. tick pass: the final tick of a node is the largest tick of a prompt whose path contains it,
//      an atomic max walking up from each prompt's end node;
//   5. eviction: removing min-tick leaves one by one equals removing the shortest prefix of the
//      nodes ordered by (tick ascending, depth descending) that frees enough tokens; the cut is
//      found by a most-significant-digit-first search over weighted digit histograms, no sort.
#include "klpm_internal.hpp"
#include "lds_sort.hpp"
#include "wave_ops.hpp"

namespace klpm {

constexpr uint64_t kNoGroup = ~0ull;
// ws.lcp_lead[j]: how many tokens prompt j's unmatched tail shares with the tail of the first prompt
// of its group; kLcpPending until the wavefront of prompt j has worked it out, kLcpNone if it does not apply.
constexpr int32_t kLcpPending = -1;
constexpr int32_t kLcpNone = -2;
constexpr uint32_t kDevInternal = 32u;  // KLPM_DEV_INTERNAL: the tree and its child table disagree
constexpr int kDeepRounds = 6;     // structure pass: rounds in which classes of members that met each other settle among themselves
constexpr int kDeepMinClass = 3;   // ... classes of at least this many members (smaller ones are inserted one after the other)
constexpr int kDeepCompare = 512;  // ... tokens a lane compares by itself before it leaves its member to the slow road
constexpr int kCutRows = 4;  // an old edge is cut for up to 64 * kCutRows prompts of a batch at once (several per lane beyond 64)
constexpr int kEvictDigitBits = 11;  // eviction cut search: bits of the key resolved per pass
constexpr int kEvictBins = 1 << kEvictDigitBits;
constexpr int kPlanThreads = 1024;

__device__ __forceinline__ void flag_error(DevState *st, uint32_t bit) { atomicOr(&st->device_error, bit); }

// What a workgroup barrier does for memory, for code that runs inside one wavefront (the structure
// pass: one wavefront per group, also when it is one part of a larger workgroup): the wavefront's
// earlier stores are complete before its later loads are issued.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// ------------------------------------------------------------------ plan
// True for exactly one workgroup of the grid: the one that finishes last. `slot` picks one of the
// per-commit counters (reset by the plan kernel). Every thread of every workgroup must call it.
__device__ __forceinline__ bool last_block_done(DevState *st, int slot) {
    __shared__ int s_last;
    __syncthreads();
    if (gridDim.x == 1) return true;  // (nobody to wait for, nothing to make visible beyond the workgroup)
    if (threadIdx.x == 0) {
        __threadfence();
        s_last = (atomicAdd(&st->done[slot], 1) == (int)gridDim.x - 1) ? 1 : 0;
    }
    __syncthreads();
    if (s_last) __threadfence();
    return s_last != 0;
}

// Node ids are reserved up front, two per admitted prompt (an insertion makes at most one split
// and at most one leaf), so the structure pass needs no shared allocation counter: reservation a
// comes off the top of the free-id stack while it lasts, then from never-used ids.  Reservations
// that end up unused are pushed back when the inserts are published.
__device__ __forceinline__ int32_t reserved_id_at(const TreeView &tv, int32_t a, int32_t f0, int32_t ns0) {
    int32_t id = (a < f0) ? tv.free_stack[f0 - 1 - a] : ns0 + (a - f0);
    return (id > 0 && id < tv.max_nodes) ? id : -1;
}
__device__ __forceinline__ int32_t reserved_id(const TreeView &tv, int32_t a) {
    return reserved_id_at(tv, a, tv.st->free_cnt0, tv.st->n_slots0);
}

// A commit may take the admitted prompts' matches from queue-wide match results the caller vouches
// for.  The plan kernel checks the ranges that later addressing depends on (index, the prompt's span,
// 0 <= m <= |x|, node id); -1 = refused.
struct PlanIn {  // what the plan reads about one admitted prompt (off, L valid when m >= 0)
    int64_t off;
    int32_t qi, L, m, e;
};

// Reads that need nothing but the batch index, so that the first 1,024 prompts' can be in flight
// while thread 0 is still deciding whether the commit goes ahead.  n_host bounds the index for the
// loads; the device-side queue length is checked in plan_check.
__device__ __forceinline__ PlanIn plan_load(const QView &q, const CommitWs &ws, const int32_t *__restrict__ batch_idx,
                                            const int32_t *__restrict__ hint_len,
                                            const int32_t *__restrict__ hint_node, int32_t j) {
    PlanIn r;
    r.qi = batch_idx[j];
    r.off = 0; r.L = 0; r.m = -1; r.e = kRoot;
    if (hint_len) {
        if (r.qi >= 0 && r.qi < q.n) {
            r.off = q.off[r.qi];
            r.L = q.len[r.qi];
            r.m = hint_len[r.qi];
            r.e = hint_node[r.qi];
        }
    } else {
        r.m = ws.bm_len[j];
        r.e = ws.bm_node[j];
        // (the match inside the commit has checked index and span of every admitted prompt; entries
        // behind them are leftovers and only must not be followed out of bounds)
        if (r.m >= 0 && r.qi >= 0 && r.qi < q.n) {
            r.off = q.off[r.qi];
            r.L = q.len[r.qi];
        } else {
            r.m = -1;
        }
    }
    return r;
}

// Range checks of a match taken from the caller's results; false = refused.
__device__ __forceinline__ bool plan_check(const TreeView &tv, const QView &q, const PlanIn &r) {
    if (r.qi < 0 || r.qi >= live_count(q.n, q.n_live)) return false;
    if (r.off < 0 || r.L < 1 || r.L > tv.max_prompt_len || r.off + (int64_t)r.L > q.n_tokens) return false;
    return r.m >= 0 && r.m <= r.L && r.e >= 0 && r.e < tv.max_nodes;
}

// What else can be checked locally about such a match, done by one lane per admitted prompt beside
// the tail copy: the node is alive, the match ends inside that node's edge (or is empty at the
// root), the last matched token is the edge's token there, and neither the edge nor a child
// continues the prompt.
__device__ __forceinline__ bool hinted_match_ok(const TreeView &tv, const int32_t *__restrict__ x, int32_t L, int32_t m,
                                                int32_t e) {
    if (m == 0) return e == kRoot ? true : false;
    if (e == kRoot) return false;
    const int32_t el = tv.edge_len[e], de = tv.depth_end[e];
    const int64_t eo = tv.edge_off[e];
    if (el <= 0 || m > de || m <= de - el) return false;
    const int64_t at = eo + (int64_t)(m - 1 - (de - el));
    if (tv.pool[at] != x[m - 1]) return false;
    if (m == L) return true;
    if (m < de) return tv.pool[at + 1] != x[m];
    int32_t c, cl;
    int64_t co;
    return slot_find(tv.slots, tv.slot_mask, make_key(e, x[m]), c, cl, co) < 0;
}

// Resets the per-commit scalars, admits the batch (or abandons the commit), then: tail lengths ->
// offsets inside the pool block of this commit; group keys; capacity decision.  With hint_len the
// admitted prompts' matches come from there instead of from a match launch before this kernel
// (range-checked here, verified against the tree by the tail copy).
__global__ __launch_bounds__(kPlanThreads) void k_commit_plan(TreeView tv, QView q,
                                                              const int32_t *__restrict__ batch_idx,
                                                              const int32_t *__restrict__ n_selected,
                                                              int32_t batch_cap, CommitWs ws,
                                                              const int32_t *__restrict__ hint_len,
                                                              const int32_t *__restrict__ hint_node) {
    __shared__ int64_t buf[kPlanThreads / kWave];
    __shared__ int64_t carry;
    __shared__ int bad;
    __shared__ int32_t s_nb;
    DevState *st = tv.st;
    const int tid = threadIdx.x;
    PlanIn first;  // of prompt tid, requested before the admission is known (batch_idx holds batch_cap entries)
    if (tid < batch_cap) first = plan_load(q, ws, batch_idx, hint_len, hint_node, tid);
    if (tid == 0) {
        uint32_t err = 0;
        int32_t nb = commit_gate(tv, n_selected, batch_cap, &err);
        if (err) st->device_error |= err;
        st->skip = err ? 1 : 0;
        st->nb = nb;
        st->need_compact = 0;
        st->need_rebuild = 0;
        st->do_evict = 0;
        st->tail_total = 0;
        st->inserted_tokens = 0;
        st->evicted_tokens = 0;
        st->new_nodes = 0;
        st->evicted_nodes = 0;
        st->free_cnt0 = st->free_cnt;
        st->n_slots0 = st->n_slots;
        st->clock0 = st->clock;
        for (int i = 0; i < 12; ++i) st->done[i] = 0;
        s_nb = nb;
        carry = 0;
        bad = 0;
    }
    __syncthreads();
    const int32_t nb = s_nb;
    for (int32_t base = 0; base < nb; base += kPlanThreads) {
        int32_t j = base + tid;
        int64_t tl = 0;
        if (j < nb) {
            ws.used[j] = 0;
            ws.leaf_tok[j] = 0;
            ws.lcp_lead[j] = kLcpPending;
            // the two node ids this prompt may use (at most one split and one leaf)
            ws.resv_id[2 * j] = reserved_id(tv, 2 * j);
            ws.resv_id[2 * j + 1] = reserved_id(tv, 2 * j + 1);
            PlanIn in = first;
            if (base > 0) in = plan_load(q, ws, batch_idx, hint_len, hint_node, j);
            if (hint_len) {
                if (!plan_check(tv, q, in)) {
                    in.m = -1;
                    in.e = kRoot;
                    atomicOr(&st->device_error, 4u /* KLPM_DEV_BAD_INPUT */);
                }
                ws.bm_len[j] = in.m;
                ws.bm_node[j] = in.e;
            }
            const int32_t m = in.m;
            if (m < 0) {
                atomicOr(&bad, 1);
                ws.gkey[j] = kNoGroup;
                ws.end_node[j] = kRoot;
                ws.next_tok[j] = -1;
            } else {
                const int32_t L = in.L, e = in.e;
                tl = (int64_t)(L - m);
                bool inside = m < tv.depth_end[e];
                const int32_t nxt = (m < L) ? q.tokens[in.off + m] : -1;
                uint64_t g;
                if (!inside && m == L) {
                    g = kNoGroup;  // already present and ending on a node boundary: ticks only
                } else if (inside) {
                    g = (uint64_t)(uint32_t)e << 33;
                } else {
                    g = ((uint64_t)(uint32_t)e << 33) | (1ull << 32) | (uint64_t)(uint32_t)nxt;
                }
                ws.gkey[j] = g;
                ws.end_node[j] = e;
                ws.next_tok[j] = nxt;
            }
        }
        int64_t chunk_total;
        int64_t incl = block_inclusive_scan<int64_t, kPlanThreads>(tl, buf, tid, chunk_total);
        if (j < nb) ws.tail_off[j] = carry + incl - tl;
        __syncthreads();
        if (tid == 0) carry += chunk_total;
        __syncthreads();
    }
    if (tid == 0 && nb > 0) {
        st->tail_total = carry;
        if (bad) {
            st->skip = 1;
        } else {
            // the end of every commit leaves room for a worst-case batch if compaction can make it;
            // tails that still do not fit mean the pool is too small for what must stay cached
            int64_t half_end = ((int64_t)st->active_half + 1) * tv.pool_half;
            if (st->pool_top + carry > half_end) {
                st->device_error |= 2u;  // KLPM_DEV_POOL_FULL
                st->skip = 1;
            }
        }
    }
}

// ------------------------------------------------------------------ end-of-commit maintenance (rare work)
// Pool compaction, one wavefront per node: every live edge span moves into the other half and the
// span kept in the child table is patched.
// Every thread of every workgroup of the launch calls it (blocks of 64 nodes go round the workgroups).
constexpr int kCompactBlock = 64;  // nodes a workgroup takes room for at once
__device__ __forceinline__ void compact_nodes(const TreeView &tv, DevState *st) {
    __shared__ int64_t s_from[kWave], s_to[kWave];
    __shared__ int32_t s_len[kWave];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave, n_wv = (int)blockDim.x / kWave;
    const int32_t n_slots = st->n_slots;
    const int64_t dst_end = (int64_t)(2 - st->active_half) * tv.pool_half;
    // kCompactBlock nodes at a time, one per lane of the workgroup's first wavefront: their lengths are summed across
    // the wavefront so that the block takes its room with a single atomic (one atomic per node on the one
    // cursor would be served one by one, 13 ns each and more under load: a millisecond for a tree of 80,000
    // nodes; blocks of 16 nodes, tried for the sake of more wavefronts at work, lost to their 4,900 atomics).
    // The copy of a block is shared out among all wavefronts of the workgroup, a node each in turn: a tree of
    // 80,000 nodes of 1,300 tokens is only 1,220 blocks, and one wavefront copies two KB at a time.
    for (int64_t id0 = 1 + (int64_t)blockIdx.x * kCompactBlock; id0 < n_slots; id0 += (int64_t)gridDim.x * kCompactBlock) {
        if (wv == 0) {
            const int64_t id = id0 + lane;
            const bool in = lane < kCompactBlock && id < n_slots;
            int32_t len = in ? tv.edge_len[id] : 0;
            len = len > 0 ? len : 0;
            const int64_t src = in ? tv.edge_off[id] : 0;
            const int32_t slot = in ? tv.slot_of[id] : -1;
            const int64_t incl = wave_inclusive_scan<int64_t>((int64_t)len, lane);
            const int64_t block_len = __shfl(incl, kWave - 1);
            int64_t base_dst = 0;
            if (lane == 0 && block_len > 0)
                base_dst = (int64_t)atomicAdd((unsigned long long *)&st->compact_cursor, (unsigned long long)block_len);
            base_dst = uni64(__shfl(base_dst, 0));
            bool ok = true;
            if (base_dst + block_len > dst_end) {  // cannot happen while total_tokens <= pool_half
                if (lane == 0) flag_error(st, 2u);
                ok = false;
            }
            const int64_t dst = base_dst + incl - len;
            s_from[lane] = src;
            s_to[lane] = dst;
            s_len[lane] = ok ? len : 0;
            if (ok && len > 0) {
                tv.edge_off[id] = dst;
                if (slot >= 0 && (uint32_t)slot <= tv.slot_mask && tv.slots[slot].child == (int32_t)id) tv.slots[slot].edge_off = dst;
                else flag_error(st, kDevInternal);
            }
        }
        __syncthreads();
        // every node's tokens by a whole wavefront, sixteen independent rows per trip
        for (int b = wv; b < kCompactBlock; b += n_wv) {
            const int32_t n = s_len[b];
            if (n <= 0) continue;
            const int64_t from = s_from[b], to = s_to[b];
            for (int32_t base = 0; base < n; base += 16 * kWave) {
                int32_t v[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int32_t i = base + r * kWave + lane;
                    v[r] = tv.pool[from + (i < n ? i : n - 1)];
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int32_t i = base + r * kWave + lane;
                    if (i < n) tv.pool[to + i] = v[r];
                }
            }
        }
        __syncthreads();
    }
}
__device__ __forceinline__ void compact_switch(const TreeView &tv, DevState *st) {
    st->active_half = 1 - st->active_half;
    st->pool_top = st->compact_cursor;
}
__device__ __forceinline__ void clear_table(const TreeView &tv, int64_t first, int64_t stride) {
    const int64_t n = (int64_t)tv.slot_mask + 1;
    for (int64_t i = first; i < n; i += stride) tv.slots[i].key = kEmptyKey;
}

__device__ __forceinline__ void write_stats(DevState *st, kLPM_stats *__restrict__ out) {
    if (st->need_rebuild) st->tombstones = 0;  // the table has just been rebuilt
    st->need_rebuild = 0;
    const int32_t skip = st->skip;
    st->skip = 0;  // (the kernels of a commit only ever raise it, several workgroups at a time)
    if (!out) return;
    out->total_tokens = st->total_tokens;
    out->inserted_tokens = skip ? 0 : st->inserted_tokens;
    out->evicted_tokens = st->evicted_tokens;
    out->n_nodes = st->n_nodes;
    out->new_nodes = skip ? 0 : st->new_nodes;
    out->evicted_nodes = st->evicted_nodes;
    out->device_error = st->device_error;
    out->clock = st->clock;
}

// All `count` workgroups of the grid wait here for each other (used on the rare maintenance path
// only).  The grid is small enough to be resident at once, so the wait ends; it is bounded all the
// same: false = the others did not arrive in time, and the caller gives up.
__device__ __forceinline__ bool maintenance_barrier(DevState *st, int slot, int count) {
    __shared__ int s_ok;
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        atomicAdd(&st->done[slot], 1);
        int ok = 1;
        for (int spins = 0; __hip_atomic_load(&st->done[slot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < count; ++spins) {
            if (spins > (1 << 24)) { ok = 0; break; }
            __builtin_amdgcn_s_sleep(8);
        }
        __threadfence();
        s_ok = ok;
    }
    __syncthreads();
    return s_ok != 0;
}

// Re-inserts every live node into the emptied child table.
__device__ __forceinline__ void fill_table(const TreeView &tv, DevState *st, int64_t first, int64_t stride) {
    const int32_t n_slots = st->n_slots;
    for (int64_t id = 1 + first; id < n_slots; id += stride) {
        int32_t len = tv.edge_len[id];
        if (len <= 0) continue;
        int64_t off = tv.edge_off[id];
        uint64_t key = make_key(tv.parent[id], tv.pool[off]);
        uint32_t h = hash_key(key) & tv.slot_mask;
        for (uint32_t probe = 0; probe <= tv.slot_mask; ++probe) {
            unsigned long long prev = atomicCAS((unsigned long long *)&tv.slots[h].key,
                                                (unsigned long long)kEmptyKey, (unsigned long long)key);
            if (prev == (unsigned long long)kEmptyKey) {
                tv.slots[h].child = (int32_t)id;
                tv.slots[h].edge_len = len;
                tv.slots[h].edge_off = off;
                tv.slot_of[id] = (int32_t)h;
                break;
            }
            h = (h + 1) & tv.slot_mask;
        }
    }
}

// `count` workgroups call this; true in the last one to arrive.
__device__ __forceinline__ bool last_of(DevState *st, int slot, int count) {
    __shared__ int s_last;
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        s_last = (atomicAdd(&st->done[slot], 1) == count - 1) ? 1 : 0;
    }
    __syncthreads();
    if (s_last) __threadfence();
    return s_last != 0;
}

// The launch that ends a commit and usually finds nothing to do but hand the counters to the
// caller.  Either pool compaction - when the active half no longer has room for a worst-case batch
// and holds garbage, every live edge span moves into the other half, the span kept in the child
// table is patched, and the last workgroup to finish switches halves - or, when evictions have
// left many tombstones, the refill of the child table (emptied by the workgroup that decided so).
// Never both: a commit that compacts leaves the rebuild to a later one.  The grid is sized for
// the compaction (a wavefront per node); without one only the first kEndBlocks workgroups stay.
constexpr int kEndBlocks = 128;
__global__ __launch_bounds__(256) void k_end_commit(TreeView tv, kLPM_stats *__restrict__ stats_out) {
    DevState *st = tv.st;
    const int need_compact = st->need_compact, need_rebuild = st->need_rebuild;
    const int n_blocks = need_compact ? (int)gridDim.x : ((int)gridDim.x < kEndBlocks ? (int)gridDim.x : kEndBlocks);
    if ((int)blockIdx.x >= n_blocks) return;
    if (need_compact) {
        compact_nodes(tv, st);
        if (last_of(st, 0, n_blocks) && threadIdx.x == 0) compact_switch(tv, st);
    } else if (need_rebuild) {
        // empty the table, wait for every workgroup to have done its share, re-insert the live nodes
        clear_table(tv, (int64_t)blockIdx.x * blockDim.x + threadIdx.x, (int64_t)n_blocks * blockDim.x);
        if (!maintenance_barrier(st, 0, n_blocks)) {
            if (threadIdx.x == 0) flag_error(st, kDevInternal);
            return;
        }
        fill_table(tv, st, (int64_t)blockIdx.x * blockDim.x + threadIdx.x, (int64_t)n_blocks * blockDim.x);
    }
    if (last_of(st, 3, n_blocks) && threadIdx.x == 0) write_stats(st, stats_out);
}

// The same by one workgroup, for trees small enough that its speed at the (rare) work does not
// matter.
constexpr int kSmallMaintainThreads = 1024;
template <int THREADS>
__device__ __forceinline__ void end_commit_small_body(const TreeView &tv, kLPM_stats *__restrict__ stats_out) {
    DevState *st = tv.st;
    const int tid = threadIdx.x;
    const int need_compact = st->need_compact, need_rebuild = st->need_rebuild;
    if (need_compact) {
        compact_nodes(tv, st);
        __syncthreads();
        if (tid == 0) compact_switch(tv, st);
    } else if (need_rebuild) {
        clear_table(tv, tid, THREADS);
        __syncthreads();
        fill_table(tv, st, tid, THREADS);
    }
    __syncthreads();
    if (tid == 0) write_stats(st, stats_out);
}
__global__ __launch_bounds__(kSmallMaintainThreads) void k_end_commit_small(TreeView tv,
                                                                             kLPM_stats *__restrict__ stats_out) {
    end_commit_small_body<kSmallMaintainThreads>(tv, stats_out);
}

// ------------------------------------------------------------------ tails
// (verify: the matches were handed in by the caller; a prompt whose match does not stand up to the
// local checks abandons the commit before anything is published)
__global__ __launch_bounds__(256) void k_copy_tails(TreeView tv, QView q, const int32_t *__restrict__ batch_idx,
                                                    CommitWs ws, int verify) {
    DevState *st = tv.st;
    const int32_t j = blockIdx.x;  // below the capacity of batch_idx and of the per-prompt arrays
    // the state words and this prompt's plan come in one round trip; nothing is followed from the
    // plan before j is known to be an admitted prompt
    const int32_t skip = st->skip, nb = st->nb;
    const int64_t pool_top = st->pool_top;
    const int32_t qi = batch_idx[j];
    const int32_t m = ws.bm_len[j];
    const int32_t e = ws.bm_node[j];
    const int64_t to = ws.tail_off[j];
    if (skip || j >= nb) return;
    const int32_t L = q.len[qi];
    const int32_t *__restrict__ src = q.tokens + q.off[qi] + m;
    if (verify && threadIdx.x == 0 && !hinted_match_ok(tv, src - m, L, m, e)) {
        st->skip = 1;
        atomicOr(&st->device_error, 4u /* KLPM_DEV_BAD_INPUT */);
    }
    int32_t *__restrict__ dst = tv.pool + pool_top + to;
    const int32_t len = L - m;
    // eight independent rows per trip (lanes past the end re-read the last token, stores are masked)
    for (int32_t base = 0; base < len; base += 8 * (int32_t)blockDim.x) {
        int32_t v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            int32_t i = base + r * (int32_t)blockDim.x + (int32_t)threadIdx.x;
            v[r] = src[i < len ? i : len - 1];
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            int32_t i = base + r * (int32_t)blockDim.x + (int32_t)threadIdx.x;
            if (i < len) dst[i] = v[r];
        }
    }
}

// ------------------------------------------------------------------ plan and tails in one launch
// For batches of up to kFusedPlanMax prompts the plan is not a kernel of its own: a workgroup takes
// kPlanGroup consecutive prompts of the batch, reads the whole batch's match lengths itself (a few KB,
// two round trips) and derives from them everything it needs - the admission, where its tails go (the
// sum of the tails before them), whether the commit goes ahead - exactly as every other workgroup
// does from the same inputs; workgroup 0 also writes the commit's scalars.  What only concerns one
// prompt (its span in the token array, its node, the local checks of a match handed in by the caller,
// its reserved ids and group key) is read and checked by one lane per prompt of the workgroup that
// owns it, while the other wavefronts already copy: the tails of a group lie side by side in the pool,
// so the copy runs over them as over one span.  Nothing here raises or lowers a flag that another
// workgroup of the same launch reads: the skip flag is only ever raised, and the end of the previous
// commit has lowered it.  (Measured on batches of 1,024 prompts with 1.7M tail tokens: one prompt per
// 256-thread workgroup, each workgroup reading everything about every prompt, 20 us; groups of 8, 4
// and 2 prompts per 1,024-thread workgroup 18, 14 and 19 us - fewer workgroups repeat less of the plan,
// more of them copy faster.)
constexpr int kFusedPlanMax = 2048;
constexpr int kFusedThreads = 256;
constexpr int kPlanGroup = 4;        // prompts per workgroup of a large batch
constexpr int kPlanSmallBatch = 512;  // batches up to this size: one prompt per 256-thread workgroup (fewer rounds in a row count for more than repeated reads)

// The key is absent from the child table (any lane on its own; the tree is not being modified).
__device__ __forceinline__ bool slot_absent_lane(const TreeView &tv, uint64_t key) {
    uint32_t h = hash_key(key) & tv.slot_mask;
    for (uint32_t probe = 0; probe <= tv.slot_mask; ++probe) {
        const uint64_t k = tv.slots[h].key;
        if (k == key) return false;
        if (k == kEmptyKey) return true;
        h = (h + 1) & tv.slot_mask;
    }
    return true;
}

template <int THREADS, int GROUP>
__device__ __forceinline__ void plan_copy_body(TreeView tv, QView q, const int32_t *__restrict__ batch_idx,
                                               const int32_t *__restrict__ n_selected, int32_t batch_cap, CommitWs ws,
                                               const int32_t *__restrict__ hint_len,
                                               const int32_t *__restrict__ hint_node) {
    constexpr int kPer = kFusedPlanMax / THREADS;
    __shared__ int64_t p_before[THREADS / kWave], p_total[THREADS / kWave];
    __shared__ int32_t p_bad[THREADS / kWave];
    __shared__ int32_t s_nb;
    __shared__ uint32_t s_err;
    __shared__ int32_t s_qi[GROUP], s_L[GROUP], s_m[GROUP];
    __shared__ int64_t s_src[GROUP];     // first tail token of each own prompt in q.tokens
    __shared__ int32_t s_start[GROUP + 1];  // tails of the own prompts, running sum
    __shared__ int64_t s_off1;                 // GROUP == 1: the own prompt's span and node
    __shared__ int32_t s_e1;
    DevState *st = tv.st;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int32_t j0 = (int32_t)blockIdx.x * GROUP;
    // one round trip: the persistent counters and every prompt's batch index; a second one: what
    // hangs on the indices (length and match length of every prompt)
    const int32_t f0 = st->free_cnt, ns0 = st->n_slots, active_half = st->active_half;
    const int64_t pool_top = st->pool_top;
    const uint64_t clock0 = st->clock;
    const int32_t n_live = live_count(q.n, q.n_live);
    int32_t qi[kPer], L[kPer], m[kPer];
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
        const int32_t i = t * THREADS + tid;
        qi[t] = i < batch_cap ? batch_idx[i] : -1;
    }
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
        const int32_t i = t * THREADS + tid;
        const bool in = i < batch_cap && qi[t] >= 0 && qi[t] < q.n;  // (q.n bounds the loads, n_live the admission)
        L[t] = in ? q.len[qi[t]] : 0;
        m[t] = !in ? -1 : hint_len ? hint_len[qi[t]] : ws.bm_len[i];
    }
    // (a workgroup with one prompt of its own asks for that prompt's span and node in the same round)
    int64_t off1 = -1;
    int32_t e1 = -1;
    if (GROUP == 1 && j0 < batch_cap && tid == (j0 & (THREADS - 1))) {
        const int t1 = j0 / THREADS;
        int32_t q1 = -1;
#pragma unroll
        for (int t = 0; t < kPer; ++t) q1 = t == t1 ? qi[t] : q1;
        if (q1 >= 0 && q1 < q.n) {
            off1 = q.off[q1];
            e1 = hint_len ? hint_node[q1] : ws.bm_node[j0];
        }
    }
    if (tid == 0) {
        uint32_t err = 0;
        s_nb = commit_gate(tv, n_selected, batch_cap, &err);
        s_err = err;
    }
    if (tid < GROUP) s_m[tid] = -1;
    __syncthreads();
    const int32_t nb = s_nb;
    const uint32_t err = s_err;
    int64_t before = 0, total = 0;
    int32_t bad = 0;
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
        const int32_t i = t * THREADS + tid;
        if (i >= nb) continue;
        // (without hints the match inside the commit has checked index and span of every admitted
        // prompt and left -1 for what it refused)
        if (qi[t] < 0 || qi[t] >= n_live || L[t] < 1 || L[t] > tv.max_prompt_len || m[t] < 0 || m[t] > L[t]) {
            bad = 1;
            continue;
        }
        const int64_t tl = (int64_t)(L[t] - m[t]);
        total += tl;
        if (i < j0) before += tl;
        if (i >= j0 && i < j0 + GROUP) {
            s_qi[i - j0] = qi[t];
            s_L[i - j0] = L[t];
            s_m[i - j0] = m[t];
            if (GROUP == 1) {
                s_off1 = off1;
                s_e1 = e1;
            }
        }
    }
    before = wave_sum(before);
    total = wave_sum(total);
    bad = wave_sum(bad);
    if (lane == 0) { p_before[wv] = before; p_total[wv] = total; p_bad[wv] = bad; }
    __syncthreads();
    before = 0; total = 0; bad = 0;
#pragma unroll
    for (int w2 = 0; w2 < THREADS / kWave; ++w2) { before += p_before[w2]; total += p_total[w2]; bad += p_bad[w2]; }
    // (the end of every commit leaves room for a worst-case batch if compaction can make it; tails
    // that still do not fit mean the pool is too small for what must stay cached)
    const int64_t half_end = ((int64_t)active_half + 1) * tv.pool_half;
    const bool pool_full = nb > 0 && !bad && pool_top + total > half_end;
    const bool skip = err != 0 || bad != 0 || pool_full;
    if (blockIdx.x == 0 && tid == 0) {
        uint32_t e = err;
        if (bad) e |= 4u;        // KLPM_DEV_BAD_INPUT
        if (pool_full) e |= 2u;  // KLPM_DEV_POOL_FULL
        if (e) atomicOr(&st->device_error, e);
        if (skip) st->skip = 1;
        st->nb = nb;
        st->need_compact = 0;
        st->need_rebuild = 0;
        st->do_evict = 0;
        st->tail_total = nb > 0 ? total : 0;
        st->inserted_tokens = 0;
        st->evicted_tokens = 0;
        st->new_nodes = 0;
        st->evicted_nodes = 0;
        st->free_cnt0 = f0;
        st->n_slots0 = ns0;
        st->clock0 = clock0;
        for (int i = 0; i < 12; ++i) st->done[i] = 0;
    }
    if (skip || j0 >= nb) return;
    const int32_t own = nb - j0 < GROUP ? nb - j0 : GROUP;
    // where the own prompts' tails start in the span they form in the pool
    if (tid < GROUP) {
        int32_t run = 0;
        for (int c = 0; c < tid; ++c) run += c < own ? s_L[c] - s_m[c] : 0;
        s_start[tid] = run;
        const bool mine = tid < own;
        int64_t off = !mine ? 0 : GROUP == 1 ? s_off1 : q.off[s_qi[tid]];
        if (off < 0 || off + (int64_t)(mine ? s_L[tid] : 0) > q.n_tokens) off = -1;  // (its owner lane refuses the commit)
        s_src[tid] = off < 0 ? -1 : off + (int64_t)(mine ? s_m[tid] : 0);
        if (tid == GROUP - 1) s_start[GROUP] = run + (mine ? s_L[tid] - s_m[tid] : 0);
    }
    __syncthreads();
    // the last wavefront: one lane per own prompt for what only concerns that prompt (the others already
    // copy meanwhile)
    if (wv == THREADS / kWave - 1 && lane < own) {
        const int32_t j = j0 + lane, Lj = s_L[lane], mj = s_m[lane], qj = s_qi[lane];
        int64_t mine = 0;  // tails of the own prompts before this one
        for (int c = 0; c < lane; ++c) mine += (int64_t)(s_L[c] - s_m[c]);
        // first round trip: the prompt's span and node, the reserved ids
        const int64_t off = GROUP == 1 ? s_off1 : q.off[qj];
        const int32_t e = GROUP == 1 ? s_e1 : hint_len ? hint_node[qj] : ws.bm_node[j];
        const int32_t id0 = reserved_id_at(tv, 2 * j, f0, ns0), id1 = reserved_id_at(tv, 2 * j + 1, f0, ns0);
        bool ok = off >= 0 && off + (int64_t)Lj <= q.n_tokens && e >= 0 && e < tv.max_nodes;
        const int32_t es = ok ? e : kRoot;
        const int64_t os = ok ? off : 0;
        // second: the node's edge and the prompt's tokens around the end of the match
        const int32_t el = tv.edge_len[es], de = tv.depth_end[es];
        const int64_t eo = tv.edge_off[es];
        const int32_t *__restrict__ x = q.tokens + os;
        const int32_t nxt = (ok && mj < Lj) ? x[mj] : -1;
        const int32_t last = (ok && mj > 0) ? x[mj - 1] : 0;
        const bool inside = mj < de;
        if (hint_len && ok) {
            // what can be checked locally about a match handed in by the caller: the node is alive, the
            // match ends inside that node's edge (or is empty at the root), the last matched token is
            // the edge's token there, and neither the edge nor a child continues the prompt
            if (mj == 0) {
                ok = es == kRoot;
            } else if (es == kRoot || el <= 0 || mj > de || mj <= de - el) {
                ok = false;
            } else {
                const int64_t at = eo + (int64_t)(mj - 1 - (de - el));
                const int32_t t0 = tv.pool[at];
                const int32_t t1 = (mj < Lj && mj < de) ? tv.pool[at + 1] : 0;
                ok = t0 == last;
                if (ok && mj < Lj) ok = mj < de ? t1 != nxt : slot_absent_lane(tv, make_key(es, nxt));
            }
        }
        if (!ok) {
            st->skip = 1;
            atomicOr(&st->device_error, 4u /* KLPM_DEV_BAD_INPUT */);
        }
        uint64_t g;
        if (!inside && mj == Lj) {
            g = kNoGroup;  // already present and ending on a node boundary: ticks only
        } else if (inside) {
            g = (uint64_t)(uint32_t)es << 33;
        } else {
            g = ((uint64_t)(uint32_t)es << 33) | (1ull << 32) | (uint64_t)(uint32_t)nxt;
        }
        ws.used[j] = 0;
        ws.leaf_tok[j] = 0;
        ws.lcp_lead[j] = kLcpPending;
        ws.resv_id[2 * j] = id0;
        ws.resv_id[2 * j + 1] = id1;
        if (hint_len) {
            ws.bm_len[j] = mj;
            ws.bm_node[j] = es;
        }
        ws.gkey[j] = g;
        ws.end_node[j] = es;
        ws.next_tok[j] = nxt;
        ws.tail_off[j] = before + mine;
        ws.p_off[j] = os;
        ws.p_len[j] = Lj;
        ws.p_de[j] = de;
    }
    // everybody: the own prompts' tails as one span of the pool (eight independent rows per trip)
    const int32_t len = s_start[GROUP];
    int32_t *__restrict__ dst = tv.pool + pool_top + before;
    for (int32_t base = 0; base < len; base += 8 * THREADS) {
        int32_t v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            int32_t i = base + r * THREADS + tid;
            i = i < len ? i : len - 1;
            int c = 0;
#pragma unroll
            for (int u = 1; u < GROUP; ++u) c += (i >= s_start[u]) ? 1 : 0;  // (empty tails share their start with the next)
            const int64_t sp = s_src[c];
            v[r] = q.tokens[sp >= 0 ? sp + (int64_t)(i - s_start[c]) : 0];  // (no branch around the load)
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int32_t i = base + r * THREADS + tid;
            if (i < len) dst[i] = v[r];
        }
    }
}
constexpr int kPlanCopyThreads = 1024;  // (what a workgroup of a large batch spends its time on is the copy: rows in flight)
__global__ __launch_bounds__(kPlanCopyThreads) void k_plan_copy(TreeView tv, QView q, const int32_t *__restrict__ batch_idx,
                                                                const int32_t *__restrict__ n_selected, int32_t batch_cap,
                                                                CommitWs ws, const int32_t *__restrict__ hint_len,
                                                                const int32_t *__restrict__ hint_node) {
    plan_copy_body<kPlanCopyThreads, kPlanGroup>(tv, q, batch_idx, n_selected, batch_cap, ws, hint_len, hint_node);
}
__global__ __launch_bounds__(kFusedThreads) void k_plan_copy_small(TreeView tv, QView q,
                                                                   const int32_t *__restrict__ batch_idx,
                                                                   const int32_t *__restrict__ n_selected, int32_t batch_cap,
                                                                   CommitWs ws, const int32_t *__restrict__ hint_len,
                                                                   const int32_t *__restrict__ hint_node) {
    plan_copy_body<kFusedThreads, 1>(tv, q, batch_idx, n_selected, batch_cap, ws, hint_len, hint_node);
}

// ------------------------------------------------------------------ structure pass
// Loads that must observe other compute units' table inserts bypass the per-CU cache.
__device__ __forceinline__ uint64_t ld_u64(const uint64_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int32_t ld_i32(const int32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int64_t ld_i64(const int64_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A node record read with loads that see other compute units' writes; the four loads are issued
// together (one round trip).
struct NodeRec {
    int32_t parent, edge_len, depth_end;
    int64_t edge_off;
};
__device__ __forceinline__ NodeRec load_node(const TreeView &tv, int32_t id) {
    int32_t pa = ld_i32(&tv.parent[id]);
    int32_t el = ld_i32(&tv.edge_len[id]);
    int32_t de = ld_i32(&tv.depth_end[id]);
    int64_t eo = ld_i64(&tv.edge_off[id]);
    NodeRec r;
    r.parent = uni(pa);
    r.edge_len = uni(el);
    r.depth_end = uni(de);
    r.edge_off = uni64(eo);
    return r;
}

__device__ __forceinline__ int32_t slot_find_live(const TreeView &tv, uint64_t key, int32_t &child, int32_t &edge_len,
                                                  int64_t &edge_off) {
    uint32_t h = hash_key(key) & tv.slot_mask;
    for (uint32_t probe = 0; probe <= tv.slot_mask; ++probe) {
        // all four fields in one round trip; the payload is only meaningful when the key matches,
        // and a key is only ever looked up by the wavefront that inserted it
        uint64_t k = ld_u64(&tv.slots[h].key);
        int32_t c = ld_i32(&tv.slots[h].child);
        int32_t l = ld_i32(&tv.slots[h].edge_len);
        int64_t o = ld_i64(&tv.slots[h].edge_off);
        k = (uint64_t)uni64((int64_t)k);
        c = uni(c);
        l = uni(l);
        o = uni64(o);
        if (k == key) {
            child = c;
            edge_len = l;
            edge_off = o;
            return (int32_t)h;
        }
        if (k == kEmptyKey) return -1;
        h = (h + 1) & tv.slot_mask;
    }
    return -1;
}

// lane 0 only. Takes the first free slot of the probe sequence, empty or left by an evicted node.
// The caller has just looked the key up and not found it.
__device__ __forceinline__ int32_t slot_insert_from(const TreeView &tv, uint32_t h, uint64_t key, int32_t child,
                                                    int32_t edge_len, int64_t edge_off) {
    for (uint32_t probe = 0; probe <= tv.slot_mask; ++probe) {
        unsigned long long *kp = (unsigned long long *)&tv.slots[h].key;
        unsigned long long prev = atomicCAS(kp, (unsigned long long)kEmptyKey, (unsigned long long)key);
        bool mine = (prev == (unsigned long long)kEmptyKey);
        if (!mine && prev == (unsigned long long)kTombKey) {
            // (the tombstone counter is not decremented: it counts evictions since the last rebuild,
            // an upper bound that needs no shared atomic here)
            mine = (atomicCAS(kp, (unsigned long long)kTombKey, (unsigned long long)key) == (unsigned long long)kTombKey);
        }
        if (mine) {
            tv.slots[h].child = child;
            tv.slots[h].edge_len = edge_len;
            tv.slots[h].edge_off = edge_off;
            tv.slot_of[child] = (int32_t)h;
            return (int32_t)h;
        }
        h = (h + 1) & tv.slot_mask;
    }
    flag_error(tv.st, kDevInternal);  // (the table has two slots per node: it cannot be full)
    return -1;
}
__device__ __forceinline__ int32_t slot_insert(const TreeView &tv, uint64_t key, int32_t child, int32_t edge_len,
                                               int64_t edge_off) {
    return slot_insert_from(tv, hash_key(key) & tv.slot_mask, key, child, edge_len, edge_off);
}
// Two inserts whose first attempts travel together (one round trip when both home slots are free,
// which is the rule in a table with two slots per node).
__device__ __forceinline__ void slot_insert_pair(const TreeView &tv, uint64_t key_a, int32_t child_a, int32_t len_a,
                                                 int64_t off_a, uint64_t key_b, int32_t child_b, int32_t len_b,
                                                 int64_t off_b, int32_t &slot_a, int32_t &slot_b) {
    const uint32_t ha = hash_key(key_a) & tv.slot_mask, hb = hash_key(key_b) & tv.slot_mask;
    if (ha == hb) {
        slot_a = slot_insert_from(tv, ha, key_a, child_a, len_a, off_a);
        slot_b = slot_insert_from(tv, hb, key_b, child_b, len_b, off_b);
        return;
    }
    const unsigned long long pa = atomicCAS((unsigned long long *)&tv.slots[ha].key, (unsigned long long)kEmptyKey,
                                            (unsigned long long)key_a);
    const unsigned long long pb = atomicCAS((unsigned long long *)&tv.slots[hb].key, (unsigned long long)kEmptyKey,
                                            (unsigned long long)key_b);
    if (pa == (unsigned long long)kEmptyKey) {
        tv.slots[ha].child = child_a;
        tv.slots[ha].edge_len = len_a;
        tv.slots[ha].edge_off = off_a;
        tv.slot_of[child_a] = (int32_t)ha;
        slot_a = (int32_t)ha;
    } else {  // (taken, or a tombstone: the ordinary probe sequence, from the home slot again)
        slot_a = slot_insert_from(tv, ha, key_a, child_a, len_a, off_a);
    }
    if (pb == (unsigned long long)kEmptyKey) {
        tv.slots[hb].child = child_b;
        tv.slots[hb].edge_len = len_b;
        tv.slots[hb].edge_off = off_b;
        tv.slot_of[child_b] = (int32_t)hb;
        slot_b = (int32_t)hb;
    } else {
        slot_b = slot_insert_from(tv, hb, key_b, child_b, len_b, off_b);
    }
}

// Split node c (reached through table slot s) after its first `at` edge tokens. The new node takes
// the upper part; c keeps the lower part, its id, its end boundary, its children and its tick.
// Returns the new upper node (wave-uniform) or -1.
// (leaf: the prompt goes on below the cut with token `tok`; its leaf - id, len tokens at pool index
// off, ending at depth `end` - is hung below the new node in the same go, both table inserts
// travelling together)
struct LeafBelow {
    bool want;
    int32_t id, tok, len, end;
    int64_t off;
};
__device__ __forceinline__ int32_t split_node(const TreeView &tv, const CommitWs &ws, int32_t j, int32_t c,
                                              const NodeRec &rec, int32_t s, int32_t at, uint64_t tick, int32_t new_id,
                                              int lane, int32_t &low_first_out, int32_t &low_slot_out,
                                              const LeafBelow &leaf, int32_t &leaf_slot_out,
                                              bool have_low = false, int32_t low_known = 0) {
    int32_t up = -1, low_first = 0, low_slot = -1, leaf_slot = -1;
    if (lane == 0) {
        // first token of the lower part (tokens never move)
        low_first = have_low ? low_known : tv.pool[rec.edge_off + at];
        up = new_id;
        if (up < 0) flag_error(tv.st, 1u);
        if (up > 0) {
            int64_t eo = rec.edge_off;
            int32_t el = rec.edge_len;
            int32_t de = rec.depth_end;
            tv.parent[up] = rec.parent;
            tv.edge_off[up] = eo;
            tv.edge_len[up] = at;
            tv.depth_end[up] = de - el + at;
            tv.tick[up] = tick;
            tv.slots[s].child = up;
            tv.slots[s].edge_len = at;
            tv.slot_of[up] = s;
            tv.edge_off[c] = eo + at;
            tv.edge_len[c] = el - at;
            tv.parent[c] = up;
            if (leaf.want) {
                tv.parent[leaf.id] = up;
                tv.edge_off[leaf.id] = leaf.off;
                tv.edge_len[leaf.id] = leaf.len;
                tv.depth_end[leaf.id] = leaf.end;
                tv.tick[leaf.id] = tick;
                slot_insert_pair(tv, make_key(up, low_first), c, el - at, eo + at, make_key(up, leaf.tok), leaf.id,
                                 leaf.len, leaf.off, low_slot, leaf_slot);
                atomicOr(&ws.used[j], 3);
                ws.leaf_tok[j] = leaf.len;
            } else {
                low_slot = slot_insert(tv, make_key(up, low_first), c, el - at, eo + at);
                atomicOr(&ws.used[j], 1);  // (zero since the plan)
            }
        }
    }
    up = uni(__shfl(up, 0));
    low_first_out = uni(__shfl(low_first, 0));
    low_slot_out = uni(__shfl(low_slot, 0));
    leaf_slot_out = uni(__shfl(leaf_slot, 0));
    wave_sync();
    return up;
}

// wave_common_prefix(a, b, lim) that also hands back, from the same round trip, the tokens the
// insertion needs next: at a mismatch j < lim the two differing tokens a[j], b[j]; when all lim
// positions agree, a[lim] (if a has a_len > lim tokens) and b[lim] (if b has b_len > lim).
// Values that do not exist come back as -1.
__device__ __forceinline__ int32_t common_prefix_and_next(const int32_t *__restrict__ a, int32_t a_len,
                                                          const int32_t *__restrict__ b, int32_t b_len, int32_t lim,
                                                          int lane, int32_t &a_tok, int32_t &b_tok) {
    // the two tokens behind the compared span, requested together with the first window
    const int32_t a_after = a[lim < a_len ? lim : a_len - 1];
    const int32_t b_after = b[lim < b_len ? lim : b_len - 1];
    const int32_t jj = wave_common_prefix(a, b, lim, lane);
    if (jj < lim) {  // (re-reads two tokens of a window that has just been fetched: served by the cache)
        a_tok = uni(a[jj]);
        b_tok = uni(b[jj]);
    } else {
        a_tok = lim < a_len ? uni(a_after) : -1;
        b_tok = lim < b_len ? uni(b_after) : -1;
    }
    return jj;
}

// What an insertion reads about its prompt before it touches the tree.  A lane loads these for a
// prompt of its own (two round trips, whatever the number of lanes doing so); the wavefront then
// takes one lane's values.
struct MemberIn {
    int32_t qi, m, e, split_id, leaf_id, tok_m, L, de_e;
    int64_t to, qoff;
};
__device__ __forceinline__ void member_load_own(MemberIn &v, const int32_t *__restrict__ batch_idx, const CommitWs &ws,
                                                int32_t j) {  // indexed by the prompt's place in the batch
    v.qi = batch_idx[j];
    v.m = ws.bm_len[j];
    v.e = ws.bm_node[j];
    v.to = ws.tail_off[j];
    v.split_id = ws.resv_id[2 * j];
    v.leaf_id = ws.resv_id[2 * j + 1];
    v.tok_m = ws.next_tok[j];
}
__device__ __forceinline__ void member_load_refs(MemberIn &v, const TreeView &tv, const QView &q) {  // behind qi and e
    v.qoff = q.off[v.qi];
    v.L = q.len[v.qi];
    v.de_e = ld_i32(&tv.depth_end[v.e]);
}
__device__ __forceinline__ MemberIn member_load(const TreeView &tv, const QView &q,
                                                const int32_t *__restrict__ batch_idx, const CommitWs &ws, int32_t j) {
    MemberIn v;
    member_load_own(v, batch_idx, ws, j);
    member_load_refs(v, tv, q);
    return v;
}
// Everything about prompt j in one round trip, for batches whose plan also left the prompt's span and the
// end depth of its stop node (an old node: it keeps its end whatever is cut above it) beside the rest.
__device__ __forceinline__ MemberIn member_load_planned(const int32_t *__restrict__ batch_idx, const CommitWs &ws,
                                                        int32_t j) {
    MemberIn v;
    member_load_own(v, batch_idx, ws, j);
    v.qoff = ws.p_off[j];
    v.L = ws.p_len[j];
    v.de_e = ws.p_de[j];
    return v;
}
__device__ __forceinline__ MemberIn member_from_lane(const MemberIn &v, int b) {
    MemberIn r;
    r.qi = uni(__shfl(v.qi, b));
    r.m = uni(__shfl(v.m, b));
    r.e = uni(__shfl(v.e, b));
    r.split_id = uni(__shfl(v.split_id, b));
    r.leaf_id = uni(__shfl(v.leaf_id, b));
    r.tok_m = uni(__shfl(v.tok_m, b));
    r.L = uni(__shfl(v.L, b));
    r.de_e = uni(__shfl(v.de_e, b));
    r.to = uni64(__shfl(v.to, b));
    r.qoff = uni64(__shfl(v.qoff, b));
    return r;
}

// State a wavefront keeps across the prompts of one group: the piece of the group's old edge that
// the previous prompt ended its search in (the upper part it has just cut off, or the piece that
// ends exactly at its match), with that piece's record and table slot.  Picks of one group come
// mostly in falling match length, so the next prompt's piece is this one or the one above it.
struct GroupCtx {
    uint64_t clock0;
    int64_t pool_top;
    // The table entries this wavefront has made in this commit, one per lane.  Everything a member
    // of the group can meet below its stop was made by this wavefront (nothing continued the
    // prompt there before, and other groups stop elsewhere), so a lookup is a compare across the
    // lanes; the table in memory is written all the same and takes over if 64 entries are not enough.
    int32_t c_parent, c_tok, c_child, c_el, c_slot;
    int64_t c_eo;
    int32_t n_ent;
    bool cache_ok;
    int32_t piece;  // -1: none yet
    int32_t piece_slot;  // slot of `piece` in its parent's table, -1 if not known
    NodeRec piece_rec;
};

__device__ __forceinline__ void made_add(GroupCtx &g, int lane, int32_t parent, int32_t tok, int32_t child, int32_t el,
                                         int64_t eo, int32_t slot) {
    if (g.n_ent >= kWave || slot < 0) {
        g.cache_ok = false;
        return;
    }
    if (lane == g.n_ent) {
        g.c_parent = parent;
        g.c_tok = tok;
        g.c_child = child;
        g.c_el = el;
        g.c_eo = eo;
        g.c_slot = slot;
    }
    ++g.n_ent;
}
// the entry in table slot `slot` now leads to `child` over `el` tokens (its edge was cut)
__device__ __forceinline__ void made_cut(GroupCtx &g, int lane, int32_t slot, int32_t child, int32_t el) {
    if (lane < g.n_ent && g.c_slot == slot) {
        g.c_child = child;
        g.c_el = el;
    }
}

// lead_h >= 0: the prompt's tail agrees with the tail of the group's first prompt in exactly lead_h
// tokens (both stopped at the same depth m), and that tail starts at pool index lead_base.  An edge
// met at depth d whose span starts at lead_base + (d - m) is a stretch of that first prompt's tail,
// so how far the prompt follows it is known without reading it.
// below >= 0: the prompt's stop lay inside an old edge that another part of this launch cuts at depth
// m; `below` is the node that ends at that cut, and the insertion starts there.
__device__ void insert_prompt(const TreeView &tv, const QView &q, const CommitWs &ws, int32_t j, const MemberIn &in,
                              GroupCtx &g, int lane, int32_t lead_h = kLcpNone, int64_t lead_base = 0, int32_t below = -1,
                              int32_t below_depth = -1, int32_t below_tok = -1) {
    DevState *st = tv.st;
    const int32_t m = in.m, e = in.e, split_id = in.split_id, leaf_id = in.leaf_id, tok_m = in.tok_m;
    const int32_t L = in.L, de_e = in.de_e;
    const uint64_t tick = g.clock0 + (uint64_t)j;
    const int64_t tail_base = g.pool_top + in.to;  // pool index holding x[m]
    const int32_t *__restrict__ x = q.tokens + in.qoff;

    int32_t cur = below >= 0 ? below : e;
    int32_t d = below >= 0 && below_depth >= 0 ? below_depth : m;  // (a start below a node may lie deeper than the match)
    bool fresh = false;  // cur has just been created by this wavefront: nothing hangs below it yet
    bool leaf_done = false;  // the prompt's leaf went in together with a split
    if (below < 0 && e != kRoot && m < de_e) {
        // The match stopped inside the edge that node e had before this commit. Earlier prompts of
        // this group may have cut that edge into a chain of pieces ending in e; find the piece
        // whose span (start, end] contains depth m.
        NodeRec rec;
        int32_t s = -1;
        if (g.piece >= 0 && m <= g.piece_rec.depth_end) {
            cur = g.piece;
            rec = g.piece_rec;
            s = g.piece_slot;
        } else {
            rec = load_node(tv, cur);
        }
        for (int guard = 0; guard <= tv.max_batch + 1; ++guard) {
            if (rec.depth_end - rec.edge_len < m) break;
            cur = rec.parent;
            rec = load_node(tv, cur);
            s = -1;
        }
        g.piece = cur;
        g.piece_rec = rec;
        g.piece_slot = s;
        if (m < rec.depth_end) {
            int32_t ds = rec.depth_end - rec.edge_len;
            if (s < 0) {
                int32_t c2, el2;
                int64_t eo2;
                int32_t first = uni(tv.pool[rec.edge_off]);
                s = slot_find_live(tv, make_key(rec.parent, first), c2, el2, eo2);
                if (s >= 0 && c2 != cur) s = -1;
            }
            if (s < 0 || m - ds <= 0) {
                if (lane == 0) flag_error(st, kDevInternal);
                return;
            }
            int32_t low_first, low_slot, leaf_slot;
            LeafBelow lf;
            lf.want = m < L && leaf_id > 0;
            lf.id = leaf_id;
            lf.tok = tok_m;
            lf.len = L - m;
            lf.end = L;
            lf.off = tail_base;
            int32_t up = split_node(tv, ws, j, cur, rec, s, m - ds, tick, split_id, lane, low_first, low_slot, lf,
                                    leaf_slot);
            if (up < 0) return;
            made_cut(g, lane, s, up, m - ds);
            made_add(g, lane, up, low_first, cur, rec.edge_len - (m - ds), rec.edge_off + (int64_t)(m - ds), low_slot);
            if (lf.want) made_add(g, lane, up, lf.tok, lf.id, lf.len, lf.off, leaf_slot);
            leaf_done = lf.want;
            // the upper part takes over the slot and the start of the edge
            g.piece = up;
            g.piece_slot = s;
            g.piece_rec.parent = rec.parent;
            g.piece_rec.edge_len = m - ds;
            g.piece_rec.depth_end = m;
            g.piece_rec.edge_off = rec.edge_off;
            cur = leaf_done ? lf.id : up;
            if (leaf_done) d = L;
            fresh = true;
        }
    }
    // From here on every child met is a node created by this commit; compare for real.  Each
    // compare brings along the token that decides the next step, a node that this wavefront has
    // just made has no children to look up, and a node reached through its table slot is described
    // by that slot: a member of a large group costs a lookup, a compare and its stores.
    int32_t tok = below >= 0 && below_depth >= 0 ? below_tok : tok_m;  // x[d] (the first unmatched token came with the plan)
    while (d < L) {
        int32_t c = -1, el = 0, s = -1;
        int64_t eo = 0;
        if (g.cache_ok) {
            const uint64_t hit = __ballot(lane < g.n_ent && g.c_parent == cur && g.c_tok == tok);
            if (hit) {
                const int b = (int)__builtin_ctzll(hit);
                c = uni(__shfl(g.c_child, b));
                el = uni(__shfl(g.c_el, b));
                eo = uni64(__shfl(g.c_eo, b));
                s = uni(__shfl(g.c_slot, b));
            }
        } else if (!fresh) {
            s = slot_find_live(tv, make_key(cur, tok), c, el, eo);
        }
        if (s < 0) {
            int32_t leaf = -1, leaf_slot = -1;
            if (lane == 0) {
                leaf = leaf_id;
                if (leaf < 0) flag_error(st, 1u);
                if (leaf > 0) {
                    int64_t off = tail_base + (int64_t)(d - m);
                    tv.parent[leaf] = cur;
                    tv.edge_off[leaf] = off;
                    tv.edge_len[leaf] = L - d;
                    tv.depth_end[leaf] = L;
                    tv.tick[leaf] = tick;
                    leaf_slot = slot_insert(tv, make_key(cur, tok), leaf, L - d, off);
                    atomicOr(&ws.used[j], 2);
                    ws.leaf_tok[j] = L - d;
                }
            }
            leaf = uni(__shfl(leaf, 0));
            leaf_slot = uni(__shfl(leaf_slot, 0));
            wave_sync();
            if (leaf < 0) return;
            made_add(g, lane, cur, tok, leaf, L - d, tail_base + (int64_t)(d - m), leaf_slot);
            cur = leaf;
            d = L;
            break;
        }
        const int32_t lim = el < L - d ? el : L - d;
        int32_t a_tok, b_tok, jj;
        if (lead_h >= 0 && eo == lead_base + (int64_t)(d - m) && m + lead_h > d) {
            const int32_t agree = m + lead_h - d;
            jj = agree < lim ? agree : lim;
            // the two tokens behind the agreed span, one round trip
            const int32_t av = x[d + jj < L ? d + jj : L - 1];
            const int32_t bv = tv.pool[eo + (jj < el ? jj : el - 1)];
            a_tok = d + jj < L ? uni(av) : -1;
            b_tok = jj < el ? uni(bv) : -1;
        } else {
            jj = common_prefix_and_next(x + d, L - d, tv.pool + eo, el, lim, lane, a_tok, b_tok);
        }
        if (jj <= 0) {  // the first token matched by construction; anything else is corruption
            if (lane == 0) flag_error(st, kDevInternal);
            return;
        }
        tok = a_tok;  // x[d + jj], if the prompt goes on
        if (jj == el) {
            cur = c;
            d += el;
            continue;
        }
        // split c after jj tokens; it hangs below cur, which ends at depth d, and the slot mirrors its edge
        NodeRec rec;
        rec.parent = cur;
        rec.edge_len = el;
        rec.depth_end = d + el;
        rec.edge_off = eo;
        int32_t low_first, low_slot, leaf_slot;
        LeafBelow lf;
        lf.want = d + jj < L && leaf_id > 0;
        lf.id = leaf_id;
        lf.tok = a_tok;
        lf.len = L - (d + jj);
        lf.end = L;
        lf.off = tail_base + (int64_t)(d + jj - m);
        const int32_t up = split_node(tv, ws, j, c, rec, s, jj, tick, split_id, lane, low_first, low_slot, lf, leaf_slot,
                                      true, b_tok);
        if (up < 0) return;
        made_cut(g, lane, s, up, jj);
        made_add(g, lane, up, low_first, c, el - jj, eo + (int64_t)jj, low_slot);
        if (lf.want) {
            made_add(g, lane, up, lf.tok, lf.id, lf.len, lf.off, leaf_slot);
            cur = lf.id;
            d = L;
            break;
        }
        cur = up;
        d += jj;
        fresh = true;
    }
    if (lane == 0) ws.end_node[j] = cur;
}

// The core of cutting one node's edge at several depths at once, one cut request per lane (lanes
// below `cnt`, those with `cuts` set; requests are in pick order, several may name the same depth).
// Node `e` with record `rec` hangs in table slot `s`; every depth lies strictly inside its edge.  The
// lowest lane of every distinct depth creates the piece that ends there with its split id; the
// topmost piece takes over slot s, the node itself - keeping id, end and children - is re-hung below
// the last piece.  Returns, per lane, the id of the piece that ends at the lane's depth.
__device__ __forceinline__ int32_t cut_edge_lanes(const TreeView &tv, const CommitWs &ws, const GroupCtx &ctx, int32_t e,
                                                  const NodeRec &rec, int32_t s, int32_t cnt, bool cuts, int32_t j,
                                                  int32_t depth, int32_t split_id, int lane) {
    const int32_t ds = rec.depth_end - rec.edge_len;
    // where my depth stands among the requested depths
    const int32_t m = cuts ? depth : 0x7FFFFFFF;
    int32_t prev_m = ds, next_m = 0x7FFFFFFF, cutter = lane;
    for (int k = 0; k < cnt; ++k) {
        const int32_t mk = __shfl(m, k);
        if (mk < m && mk > prev_m) prev_m = mk;
        if (mk > m && mk < next_m) next_m = mk;
        if (mk == m && k < cutter) cutter = k;
    }
    int32_t prev_cut = -1;
    for (int k = cnt - 1; k >= 0; --k)
        if (__shfl(m, k) == prev_m) prev_cut = k;
    const bool is_cutter = cuts && cutter == lane;
    const bool is_last = is_cutter && next_m == 0x7FFFFFFF;
    const int32_t up_id = __shfl(split_id, cutter);
    const int32_t prev_up = __shfl(split_id, prev_cut < 0 ? 0 : prev_cut);
    // the first token of my piece and (largest depth) of what is left of the node, one round trip
    int32_t ftok = 0, low_first = 0;
    if (is_cutter && prev_cut >= 0) ftok = tv.pool[rec.edge_off + (int64_t)(prev_m - ds)];
    if (is_last) low_first = tv.pool[rec.edge_off + (int64_t)(depth - ds)];
    if (is_cutter) {
        const int64_t off = rec.edge_off + (int64_t)(prev_m - ds);
        tv.parent[up_id] = prev_cut < 0 ? rec.parent : prev_up;
        tv.edge_off[up_id] = off;
        tv.edge_len[up_id] = depth - prev_m;
        tv.depth_end[up_id] = depth;
        tv.tick[up_id] = ctx.clock0 + (uint64_t)j;
        atomicOr(&ws.used[j], 1);
        if (prev_cut < 0) {  // the topmost piece takes over the node's table slot and the start of the edge
            tv.slots[s].child = up_id;
            tv.slots[s].edge_len = depth - prev_m;
            tv.slot_of[up_id] = s;
        } else {
            slot_insert(tv, make_key(prev_up, ftok), up_id, depth - prev_m, off);
        }
        if (is_last) {
            const int64_t low_off = rec.edge_off + (int64_t)(depth - ds);
            tv.edge_off[e] = low_off;
            tv.edge_len[e] = rec.depth_end - depth;
            tv.parent[e] = up_id;
            slot_insert(tv, make_key(up_id, low_first), e, rec.depth_end - depth, low_off);
        }
    }
    return up_id;
}

// The same for more cut requests than lanes: request i sits in lane i % 64, row i / 64 (R rows, so up to
// 64 R requests; lanes hold the rows' values side by side).  Used for an old edge that more than 64 prompts
// of a batch stop inside.
template <int R>
__device__ __forceinline__ void cut_edge_rows(const TreeView &tv, const CommitWs &ws, const GroupCtx &ctx, int32_t e,
                                              const NodeRec &rec, int32_t s, int32_t cnt, const bool (&cuts)[R],
                                              const int32_t (&j)[R], const int32_t (&depth)[R],
                                              const int32_t (&split_id)[R], int lane) {
    const int32_t ds = rec.depth_end - rec.edge_len;
    int32_t m[R], prev_m[R], next_m[R], cutter[R], prev_cut[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        m[r] = cuts[r] ? depth[r] : 0x7FFFFFFF;
        prev_m[r] = ds;
        next_m[r] = 0x7FFFFFFF;
        cutter[r] = r * kWave + lane;
        prev_cut[r] = -1;
    }
    // where every request's depth stands among all requested depths
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int32_t row_n = cnt - rr * kWave < kWave ? cnt - rr * kWave : kWave;
        for (int k = 0; k < row_n; ++k) {
            const int32_t mk = __shfl(m[rr], k);
            const int32_t idx = rr * kWave + k;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (mk < m[r] && mk > prev_m[r]) prev_m[r] = mk;
                if (mk > m[r] && mk < next_m[r]) next_m[r] = mk;
                if (mk == m[r] && idx < cutter[r]) cutter[r] = idx;
            }
        }
    }
    // the first request, in pick order, that cuts at the next smaller depth
#pragma unroll
    for (int rr = R - 1; rr >= 0; --rr) {
        const int32_t row_n = cnt - rr * kWave < kWave ? cnt - rr * kWave : kWave;
        for (int k = row_n - 1; k >= 0; --k) {
            const int32_t mk = __shfl(m[rr], k);
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (mk == prev_m[r]) prev_cut[r] = rr * kWave + k;
        }
    }
    // split id of a request by its index (its row differs from lane to lane)
    auto id_of = [&](int32_t idx) -> int32_t {
        int32_t v = 0;
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            const int32_t t = __shfl(split_id[rr], idx & (kWave - 1));
            if ((idx >> 6) == rr) v = t;
        }
        return v;
    };
    int32_t up_id[R], prev_up[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        up_id[r] = id_of(cutter[r]);
        prev_up[r] = id_of(prev_cut[r] < 0 ? 0 : prev_cut[r]);
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const bool is_cutter = cuts[r] && cutter[r] == r * kWave + lane;
        const bool is_last = is_cutter && next_m[r] == 0x7FFFFFFF;
        // the first token of this piece and (largest depth) of what is left of the node, one round trip
        int32_t ftok = 0, low_first = 0;
        if (is_cutter && prev_cut[r] >= 0) ftok = tv.pool[rec.edge_off + (int64_t)(prev_m[r] - ds)];
        if (is_last) low_first = tv.pool[rec.edge_off + (int64_t)(depth[r] - ds)];
        if (is_cutter) {
            const int32_t up = up_id[r];
            const int64_t off = rec.edge_off + (int64_t)(prev_m[r] - ds);
            tv.parent[up] = prev_cut[r] < 0 ? rec.parent : prev_up[r];
            tv.edge_off[up] = off;
            tv.edge_len[up] = depth[r] - prev_m[r];
            tv.depth_end[up] = depth[r];
            tv.tick[up] = ctx.clock0 + (uint64_t)j[r];
            atomicOr(&ws.used[j[r]], 1);
            if (prev_cut[r] < 0) {  // the topmost piece takes over the node's table slot and the start of the edge
                tv.slots[s].child = up;
                tv.slots[s].edge_len = depth[r] - prev_m[r];
                tv.slot_of[up] = s;
            } else {
                slot_insert(tv, make_key(prev_up[r], ftok), up, depth[r] - prev_m[r], off);
            }
            if (is_last) {
                const int64_t low_off = rec.edge_off + (int64_t)(depth[r] - ds);
                tv.edge_off[e] = low_off;
                tv.edge_len[e] = rec.depth_end - depth[r];
                tv.parent[e] = up;
                slot_insert(tv, make_key(up, low_first), e, rec.depth_end - depth[r], low_off);
            }
        }
    }
}

// The prompts of a batch whose matches stopped inside one old edge cut it at their stop depths.
// Inserted one after the other every prompt costs a few dependent round trips, and a popular edge
// collects dozens of them; but the pieces follow from the sorted stop depths alone.  So the wavefront
// of the first such prompt takes one prompt per lane (at most 64, among the first 1,024 of the batch):
// the lowest lane of every distinct depth m creates the piece that ends at m (with its reserved id),
// hangs it below the piece of the next smaller depth - the topmost piece takes over the old table
// slot - and the lane of the largest depth re-hangs the old node, which keeps its id, its end and
// its children, below the last piece.  What the prompts add behind their cuts is inserted by other
// wavefronts of the same launch (one per depth and next token), which only need the id of the piece
// that ends at their depth: the split id reserved for the first prompt, in pick order, that stops
// there.  Ticks are the cutting prompts' own; the tick pass raises them as for any insert.
// Returns false with nothing touched if the tree and its table disagree.
__device__ bool cut_old_edge(const TreeView &tv, const QView &q, const CommitWs &ws, const int32_t *__restrict__ batch_idx,
                             const GroupCtx &ctx, int32_t g, int32_t e, uint32_t mine_e, int lane) {
    __shared__ int32_t s_mem[kCutRows * kWave];
    constexpr int kRows = 16;
    const uint64_t below = (1ull << lane) - 1ull;
    int32_t cnt = 1;
    if (lane == 0) s_mem[0] = g;
    for (int t = g / kWave; t < kRows; ++t) {
        const bool bit = (mine_e >> t) & 1u;
        const uint64_t mask = __ballot(bit);
        if (!mask) continue;
        const int32_t pos = cnt + (int32_t)__popcll(mask & below);
        if (bit && pos < kCutRows * kWave) s_mem[pos] = t * kWave + lane;
        cnt += (int32_t)__popcll(mask);
    }
    if (cnt > kCutRows * kWave) return false;  // (the caller has counted: cannot happen)
    wave_sync();
    if (cnt > kWave) {
        // more prompts than lanes: kCutRows requests per lane
        const int32_t pa_w = ld_i32(&tv.parent[e]), el_w = ld_i32(&tv.edge_len[e]), de_w = ld_i32(&tv.depth_end[e]);
        const int64_t eo_w = ld_i64(&tv.edge_off[e]);
        const int32_t s_w = ld_i32(&tv.slot_of[e]);
        bool act[kCutRows];
        int32_t jj[kCutRows], mv[kCutRows], sp[kCutRows];
#pragma unroll
        for (int r = 0; r < kCutRows; ++r) {
            act[r] = r * kWave + lane < cnt;
            jj[r] = act[r] ? s_mem[r * kWave + lane] : g;
            mv[r] = ws.bm_len[jj[r]];
            sp[r] = ws.resv_id[2 * jj[r]];
        }
        NodeRec wrec;
        wrec.parent = uni(pa_w);
        wrec.edge_len = uni(el_w);
        wrec.depth_end = uni(de_w);
        wrec.edge_off = uni64(eo_w);
        const int32_t sw = uni(s_w);
        const int32_t dsw = wrec.depth_end - wrec.edge_len;
        bool badw = sw < 0 || (uint32_t)sw > tv.slot_mask;
#pragma unroll
        for (int r = 0; r < kCutRows; ++r)
            if (act[r] && (mv[r] <= dsw || mv[r] >= wrec.depth_end || sp[r] <= 0)) badw = true;
        if (__ballot(badw) || uni(ld_i32(&tv.slots[sw < 0 ? 0 : sw].child)) != e) {
            if (lane == 0) flag_error(tv.st, kDevInternal);
            return false;
        }
        cut_edge_rows<kCutRows>(tv, ws, ctx, e, wrec, sw, cnt, act, jj, mv, sp, lane);
        wave_sync();
        return true;
    }
    const bool active = lane < cnt;
    const int32_t j = active ? s_mem[lane] : g;
    // (the old node's record and slot travel with the members' inputs)
    const int32_t pa_v = ld_i32(&tv.parent[e]), el_v = ld_i32(&tv.edge_len[e]), de_v = ld_i32(&tv.depth_end[e]);
    const int64_t eo_v = ld_i64(&tv.edge_off[e]);
    const int32_t s_v = ld_i32(&tv.slot_of[e]);
    const int32_t m_v = ws.bm_len[j], split_v = ws.resv_id[2 * j];
    NodeRec rec;
    rec.parent = uni(pa_v);
    rec.edge_len = uni(el_v);
    rec.depth_end = uni(de_v);
    rec.edge_off = uni64(eo_v);
    const int32_t s = uni(s_v);
    const int32_t ds = rec.depth_end - rec.edge_len;
    bool bad = active && (m_v <= ds || m_v >= rec.depth_end || split_v <= 0);
    if (s < 0 || (uint32_t)s > tv.slot_mask) bad = true;
    if (__ballot(bad) || uni(ld_i32(&tv.slots[s < 0 ? 0 : s].child)) != e) {
        if (lane == 0) flag_error(tv.st, kDevInternal);
        return false;
    }
    cut_edge_lanes(tv, ws, ctx, e, rec, s, cnt, active, j, m_v, split_v, lane);
    wave_sync();
    return true;
}

// Batches of up to 1,024 prompts (the group keys, match lengths and next tokens of all of them fit
// the registers of a wavefront: one request per lane and row).  Wavefront g looks at prompt g:
//   - prompts that stopped at the same node boundary with the same next token form a group; the
//     first of them, in pick order, inserts the group one after the other below that node;
//   - prompts that stopped inside the same old edge: the first of them cuts the edge for all (one
//     prompt per lane, cut_old_edge); behind the cuts the prompts group by stop depth and next token,
//     and the first prompt of every such group inserts it below the piece that ends at that depth;
//   - a prompt that is not the first of its group measures how far its unmatched tail agrees with
//     the tail of that first prompt, which the inserting wavefront picks up (bounded wait).
// Groups touch disjoint structure, so they proceed concurrently (compare-and-swap table inserts).
__device__ __forceinline__ void structure_body(TreeView tv, QView q, const int32_t *__restrict__ batch_idx,
                                                     CommitWs ws) {
    DevState *st = tv.st;
    const int lane = threadIdx.x;
    const int32_t g = blockIdx.x;  // below the capacity of batch_idx and of the per-prompt arrays
    constexpr int kRows = 16;
    // One round trip for everything that does not depend on anything else: the commit's state, every
    // prompt's key, match length and next token, and this prompt's own inputs (read before it is
    // known that g is an admitted prompt; nothing is followed from them until then).
    const int32_t skip_v = st->skip;
    const int32_t nb_v = st->nb;
    const uint64_t key_v = ws.gkey[g];
    uint64_t kk[kRows];
    int32_t mm[kRows], tt[kRows];
#pragma unroll
    for (int t = 0; t < kRows; ++t) {
        const int32_t i = t * kWave + lane;
        const int32_t ic = i < tv.max_batch ? i : tv.max_batch - 1;
        kk[t] = ws.gkey[ic];
        mm[t] = ws.bm_len[ic];
        tt[t] = ws.next_tok[ic];
    }
    GroupCtx ctx;
    ctx.clock0 = st->clock0;
    ctx.pool_top = st->pool_top;
    ctx.n_ent = 0;
    ctx.cache_ok = true;
    ctx.c_parent = ctx.c_tok = ctx.c_child = ctx.c_el = ctx.c_slot = -1;
    ctx.c_eo = 0;
    ctx.piece = -1;
    ctx.piece_slot = -1;
    ctx.piece_rec = NodeRec{};
    const MemberIn own = member_load_planned(batch_idx, ws, g);
    if (uni(skip_v)) return;
    const int32_t nb = uni(nb_v);
    if (g >= nb) return;
    const uint64_t key = uni64(key_v);
    if (key == kNoGroup) return;
    const bool inside = ((key >> 32) & 1ull) == 0;
    const int32_t m = uni(own.m), tok = uni(own.tok_m);
    // who shares the old edge with me (stops inside it), and who also shares depth and next token
    bool first_e = true, first_s = true;
    uint32_t mine_e = 0, mine_s = 0;
    int32_t count_e = 0, cutter = 0x7FFFFFFF, leader = 0x7FFFFFFF;
#pragma unroll
    for (int t = 0; t < kRows; ++t) {
        const int32_t i = t * kWave + lane;
        const bool eq_e = i < nb && kk[t] == key;
        const bool eq_d = eq_e && (!inside || mm[t] == m);
        const bool eq_s = eq_d && (!inside || tt[t] == tok);
        if (eq_e && i < g) first_e = false;
        if (eq_s && i < g) first_s = false;
        if (eq_e && i > g) mine_e |= 1u << t;
        if (eq_s && i > g) mine_s |= 1u << t;
        count_e += (int32_t)__popcll(__ballot(eq_e));
        const uint64_t md = __ballot(eq_d), ms = __ballot(eq_s);
        if (md && cutter == 0x7FFFFFFF) cutter = t * kWave + (int32_t)__builtin_ctzll(md);  // first prompt that stops at my depth
        if (ms && leader == 0x7FFFFFFF) leader = t * kWave + (int32_t)__builtin_ctzll(ms);  // first prompt of my group
    }
    first_e = !__ballot(!first_e);
    first_s = !__ballot(!first_s);
    // an edge that more prompts stop inside than the cutting wavefront takes (kCutRows per lane) is handled
    // the slow way: its prompts are one group, inserted one after the other by the first of them
    const bool cut_scheme = inside && count_e <= kCutRows * kWave;
    if (inside && !cut_scheme) {
        first_s = first_e;
        mine_s = mine_e;
        leader = 0x7FFFFFFF;
#pragma unroll
        for (int t = 0; t < kRows; ++t) {
            const uint64_t me = __ballot(t * kWave + lane < nb && kk[t] == key);
            if (me && leader == 0x7FFFFFFF) leader = t * kWave + (int32_t)__builtin_ctzll(me);
        }
    }
    // what hangs on indices: my prompt's span, and the piece my group hangs below (the split id
    // reserved for the first prompt that stops at my depth)
    int32_t below_v = -1;
    if (cut_scheme) below_v = ws.resv_id[2 * cutter];
    const MemberIn me = member_from_lane(own, 0);
    if (!first_s) {
        // Not the first of its group: that prompt's wavefront inserts this one.  Meanwhile this
        // wavefront measures how far the two unmatched tails agree, which lets the insertion walk
        // down the first prompt's new nodes without comparing tokens again.
        int32_t h = kLcpNone;
        const int32_t qf = batch_idx[leader], mf = ws.bm_len[leader];
        if (uni(mf) == me.m && me.m < me.L) {
            const int64_t off_f = uni64(q.off[uni(qf)]);
            const int32_t len_f = uni(q.len[uni(qf)]);
            const int32_t lim = (len_f < me.L ? len_f : me.L) - me.m;
            if (lim > 0) h = wave_common_prefix(q.tokens + me.qoff + me.m, q.tokens + off_f + me.m, lim, lane);
        }
        int32_t after = -1;  // my token behind the agreed span (what my own tail starts with below the cut)
        if (h >= 0 && me.m + h < me.L) after = uni(q.tokens[me.qoff + me.m + h]);
        if (lane == 0) {
            ws.lcp_tok[g] = after;
            __hip_atomic_store(&ws.lcp_lead[g], h, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        return;
    }
    int32_t below = -1;
    if (cut_scheme) {
        below = uni(below_v);
        if (first_e && !cut_old_edge(tv, q, ws, batch_idx, ctx, g, me.e, mine_e, lane)) return;
        if (below <= 0) {
            if (lane == 0) flag_error(st, 1u);
            return;
        }
    }
    const int64_t lead_base = ctx.pool_top + me.to;
    insert_prompt(tv, q, ws, g, me, ctx, lane, kLcpNone, 0, below);
    if (!__ballot(mine_s != 0)) return;
    // The later members of the group, one per lane.  Each has measured how far its tail agrees with
    // mine (its own wavefront did, concurrently), so it leaves the leaf that I have just hung at a
    // known depth: the members cut that leaf like an old edge (cut_edge_lanes) and hang what they
    // have behind their cuts below the pieces, all at once.  Only members that leave at the same
    // depth with the same token still meet each other; they are inserted one by one afterwards.
    if (me.m < me.L && ctx.n_ent == 1 && (!inside || cut_scheme)) {
        __shared__ int32_t s_mem[kWave];
        const uint64_t lower = (1ull << lane) - 1ull;
        int32_t cnt_all = 0;
        uint32_t by_lanes = 0;  // my members among the first 64 of the group: those go in all at once
        for (int t = g / kWave; t < kRows; ++t) {
            const bool bit = (mine_s >> t) & 1u;
            const uint64_t mask = __ballot(bit);
            if (!mask) continue;
            const int32_t pos = cnt_all + (int32_t)__popcll(mask & lower);
            if (bit && pos < kWave) {
                s_mem[pos] = t * kWave + lane;
                by_lanes |= 1u << t;
            }
            cnt_all += (int32_t)__popcll(mask);
        }
        const int32_t cnt = cnt_all < kWave ? cnt_all : kWave;
        {
            wave_sync();
            const bool active = lane < cnt;
            const int32_t j = active ? s_mem[lane] : g;
            const MemberIn mv = member_load_planned(batch_idx, ws, j);
            int32_t h = active ? kLcpPending : kLcpNone;
            for (int spin = 0; spin < 2048; ++spin) {
                if (h == kLcpPending) h = __hip_atomic_load(&ws.lcp_lead[j], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
                if (!__ballot(h == kLcpPending)) break;
                __builtin_amdgcn_s_sleep(8);
            }
            const int32_t after = active ? ld_i32(&ws.lcp_tok[j]) : -1;
            const int32_t span = (mv.L < me.L ? mv.L : me.L) - me.m;
            const bool ok = !active || (mv.m == me.m && h >= 1 && h <= span && mv.split_id > 0 && mv.leaf_id > 0);
            if (!__ballot(!ok)) {
                const int32_t leaf_id = uni(__shfl(ctx.c_child, 0)), leaf_slot = uni(__shfl(ctx.c_slot, 0));
                NodeRec lrec;
                lrec.parent = below >= 0 ? below : me.e;
                lrec.edge_len = me.L - me.m;
                lrec.depth_end = me.L;
                lrec.edge_off = lead_base;
                const int32_t d = me.m + h;            // where this member leaves my string
                const bool cuts = active && d < me.L;  // (d == my length: it goes on below the whole leaf)
                int32_t piece = cut_edge_lanes(tv, ws, ctx, leaf_id, lrec, leaf_slot, cnt, cuts, j, d, mv.split_id, lane);
                if (!cuts) piece = leaf_id;
                const bool has_tail = active && mv.L > d;
                bool conflict = false;
                for (int k = 0; k < cnt; ++k) {
                    const int32_t dk = __shfl(d, k), ak = __shfl(after, k);
                    const bool tk = __shfl((int)has_tail, k) != 0;
                    if (k < lane && has_tail && tk && dk == d && ak == after) conflict = true;
                }
                const int64_t off = ctx.pool_top + mv.to + (int64_t)h;
                int32_t made_slot = -1;
                const bool hangs = active && !conflict && has_tail;
                if (active && !conflict) {
                    int32_t end = piece, leaf_tokens = 0;
                    if (has_tail) {
                        tv.parent[mv.leaf_id] = piece;
                        tv.edge_off[mv.leaf_id] = off;
                        tv.edge_len[mv.leaf_id] = mv.L - d;
                        tv.depth_end[mv.leaf_id] = mv.L;
                        tv.tick[mv.leaf_id] = ctx.clock0 + (uint64_t)j;
                        made_slot = slot_insert(tv, make_key(piece, after), mv.leaf_id, mv.L - d, off);
                        atomicOr(&ws.used[j], 2);
                        end = mv.leaf_id;
                        leaf_tokens = mv.L - d;
                    }
                    ws.leaf_tok[j] = leaf_tokens;
                    ws.end_node[j] = end;
                }
                __threadfence();
                wave_sync();
                // Members that met each other (same depth, same token) agree with one another for longer than
                // with me: near-duplicates whose common part is longer than mine.  The first of such a class
                // has hung its leaf; the others now do with that leaf what everybody did with mine - every
                // lane measures by itself how far its member follows the class's first member, the class cuts
                // that leaf at those depths at once and hangs what is left - and so on while classes of
                // several members remain.  Small classes and what is left after kDeepRounds rounds are
                // inserted one after the other below.
                int32_t d_c = d, after_c = after, piece_c = piece, slot_c = made_slot;
                int64_t off_c = off;
                bool hangs_c = hangs, conflict_c = active && conflict;
                bool deeper = false;
                for (int round = 0; round < kDeepRounds; ++round) {
                    int32_t head = -1, csize = 0;
                    for (int k = 0; k < cnt; ++k) {
                        const int32_t pk = __shfl(piece_c, k), ak = __shfl(after_c, k);
                        const bool hk = __shfl((int)hangs_c, k) != 0, ck = __shfl((int)conflict_c, k) != 0;
                        if (conflict_c && pk == piece_c && ak == after_c) {
                            if (hk && head < 0) head = k;
                            if (ck) ++csize;
                        }
                    }
                    const int32_t hl = head < 0 ? 0 : head;
                    const int32_t slot_h = __shfl(slot_c, hl), L_h = __shfl(mv.L, hl);
                    const int64_t qoff_h = (int64_t)(((uint64_t)(uint32_t)__shfl((int32_t)((uint64_t)mv.qoff >> 32), hl) << 32) |
                                                     (uint64_t)(uint32_t)__shfl((int32_t)(uint32_t)mv.qoff, hl));
                    bool go = conflict_c && head >= 0 && csize >= kDeepMinClass && slot_h >= 0;
                    if (!__ballot(go)) break;
                    // how far my member follows the first member of its class (both continue with the same token)
                    int32_t h2 = 0;
                    if (go) {
                        const int32_t lim = (mv.L < L_h ? mv.L : L_h) - d_c;
                        const int32_t cap = lim < kDeepCompare ? lim : kDeepCompare;
                        const int32_t *__restrict__ xa = q.tokens + mv.qoff + d_c;
                        const int32_t *__restrict__ xb = q.tokens + qoff_h + d_c;
                        bool differ = false;
                        constexpr int kChunk = 32;  // tokens of both prompts requested per round trip
                        for (int32_t t = 0; t < cap && !differ; t += kChunk) {
                            int32_t av[kChunk], bv[kChunk];
#pragma unroll
                            for (int u = 0; u < kChunk; ++u) {
                                const int32_t i = t + u < cap ? t + u : cap - 1;
                                av[u] = xa[i];
                                bv[u] = xb[i];
                            }
#pragma unroll
                            for (int u = 0; u < kChunk; ++u) {
                                if (!differ && t + u < cap) {
                                    if (av[u] != bv[u]) differ = true; else ++h2;
                                }
                            }
                        }
                        if ((!differ && cap < lim) || h2 < 1) go = false;  // longer than a lane compares by itself: left to the slow road
                    }
                    const int32_t d_n = d_c + h2;
                    int32_t after_n = -1;
                    if (go && d_n < mv.L) after_n = q.tokens[mv.qoff + d_n];
                    const bool tail_n = go && mv.L > d_n;
                    // every class cuts the leaf of its first member
                    uint64_t heads = 0;
                    for (int k = 0; k < cnt; ++k)
                        if (__shfl((int)go, k)) heads |= 1ull << __shfl(hl, k);
                    if (!heads) break;
                    deeper = true;
                    int32_t piece_n = -1;
                    while (heads) {
                        const int b = (int)__builtin_ctzll(heads);
                        heads &= heads - 1ull;
                        const int32_t leaf_b = uni(__shfl(mv.leaf_id, b)), slot_b = uni(__shfl(slot_c, b));
                        const int32_t L_b = uni(__shfl(mv.L, b)), d_b = uni(__shfl(d_c, b));
                        NodeRec hrec;
                        hrec.parent = uni(__shfl(piece_c, b));
                        hrec.edge_len = L_b - d_b;
                        hrec.depth_end = L_b;
                        hrec.edge_off = uni64(__shfl(off_c, b));
                        const bool in_cls = go && head == b;
                        const bool cuts_b = in_cls && d_n < L_b;
                        const int32_t pc = cut_edge_lanes(tv, ws, ctx, leaf_b, hrec, slot_b, cnt, cuts_b, j, d_n, mv.split_id, lane);
                        if (in_cls) piece_n = cuts_b ? pc : leaf_b;
                    }
                    // who still meets whom behind the new cuts
                    bool conflict_n = false;
                    for (int k = 0; k < cnt; ++k) {
                        const int32_t pk = __shfl(piece_n, k), ak = __shfl(after_n, k);
                        const bool gk = __shfl((int)go, k) != 0, tk = __shfl((int)tail_n, k) != 0;
                        if (k < lane && go && tail_n && gk && tk && pk == piece_n && ak == after_n) conflict_n = true;
                    }
                    if (go) {
                        d_c = d_n;
                        after_c = after_n;
                        piece_c = piece_n;
                        off_c = ctx.pool_top + mv.to + (int64_t)(d_n - me.m);
                        conflict_c = conflict_n;
                        hangs_c = false;
                        slot_c = -1;
                        if (!conflict_n) {
                            int32_t end = piece_n, leaf_tokens = 0;
                            if (tail_n) {
                                tv.parent[mv.leaf_id] = piece_n;
                                tv.edge_off[mv.leaf_id] = off_c;
                                tv.edge_len[mv.leaf_id] = mv.L - d_n;
                                tv.depth_end[mv.leaf_id] = mv.L;
                                tv.tick[mv.leaf_id] = ctx.clock0 + (uint64_t)j;
                                slot_c = slot_insert(tv, make_key(piece_n, after_n), mv.leaf_id, mv.L - d_n, off_c);
                                atomicOr(&ws.used[j], 2);
                                end = mv.leaf_id;
                                leaf_tokens = mv.L - d_n;
                                hangs_c = true;
                            }
                            ws.leaf_tok[j] = leaf_tokens;
                            ws.end_node[j] = end;
                        }
                    }
                    __threadfence();
                    wave_sync();
                }
                // The members that still meet each other follow, one after the other.  Whatever they can find below
                // their pieces is a leaf that a lane has just hung there (the rest of my own leaf goes on with
                // my token, not theirs), so the record of this wavefront's table entries is set up from the
                // lanes: lane k describes the leaf of member k, if it hung one.  (After further rounds leaves have
                // been cut that the lanes do not describe any more: the table in memory answers then.)
                ctx.c_parent = hangs_c ? piece_c : -2;  // (no node has this id)
                ctx.c_tok = after_c;
                ctx.c_child = mv.leaf_id;
                ctx.c_el = mv.L - d_c;
                ctx.c_eo = off_c;
                ctx.c_slot = slot_c;
                ctx.n_ent = deeper ? kWave : cnt;
                ctx.cache_ok = !deeper && !__ballot(hangs_c && slot_c < 0);
                ctx.piece = -1;
                uint64_t todo = __ballot(conflict_c);
                while (todo) {
                    const int b = (int)__builtin_ctzll(todo);
                    todo &= todo - 1ull;
                    insert_prompt(tv, q, ws, uni(__shfl(j, b)), member_from_lane(mv, b), ctx, lane, kLcpNone, 0,
                                  uni(__shfl(piece_c, b)), uni(__shfl(d_c, b)), uni(__shfl(after_c, b)));
                }
                if (cnt_all <= kWave) return;
                // a group of more than 64 later members: the rest follow one after the other below, finding
                // what the lanes have made through the table in memory (the record kept in the lanes describes
                // the members' leaves only, not the pieces of my leaf)
                mine_s &= ~by_lanes;
                ctx.cache_ok = false;
                ctx.n_ent = kWave;
            }
        }
    }
    // A later member's overlap with this prompt's tail: worked out by that member's own wavefront,
    // which started together with this one.  The wait is bounded; without an answer the insertion
    // compares tokens as it would have anyway.
    auto overlap_of = [&](int32_t j2) -> int32_t {
        int32_t h = kLcpPending;
        for (int spin = 0; spin < 2048; ++spin) {
            h = uni(__hip_atomic_load(&ws.lcp_lead[j2], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT));
            if (h != kLcpPending) break;
            __builtin_amdgcn_s_sleep(8);
        }
        return h;
    };
    // later members of the group; every lane that owns a member of a row fetches that member's inputs
    for (int t = g / kWave; t < kRows; ++t) {
        const bool is_mine = (mine_s >> t) & 1u;
        uint64_t mask = __ballot(is_mine);
        if (!mask) continue;
        const MemberIn mv = member_load_planned(batch_idx, ws, is_mine ? t * kWave + lane : g);
        while (mask) {
            const int32_t b = (int32_t)__builtin_ctzll(mask);
            mask &= mask - 1ull;
            const MemberIn mi = member_from_lane(mv, b);
            const int32_t h = mi.m == me.m ? overlap_of(t * kWave + b) : kLcpNone;
            insert_prompt(tv, q, ws, t * kWave + b, mi, ctx, lane, h, lead_base, mi.m == me.m ? below : -1);
        }
    }
}
__global__ __launch_bounds__(kWave) void k_structure(TreeView tv, QView q, const int32_t *__restrict__ batch_idx,
                                                     CommitWs ws) {
    structure_body(tv, q, batch_idx, ws);
}

// Batches of more than 1,024 prompts: one wavefront per group of prompts that stopped at the same
// place of the old tree (inside the same edge, or at the same node with the same next token), the
// group's prompts inserted one after the other.
__global__ __launch_bounds__(kWave) void k_structure_wide(TreeView tv, QView q, const int32_t *__restrict__ batch_idx,
                                                     CommitWs ws) {
    DevState *st = tv.st;
    const int lane = threadIdx.x;
    const int32_t g = blockIdx.x;  // below the capacity of batch_idx and of the per-prompt arrays
    constexpr int kRows = 16;      // group keys of the first 1,024 prompts: one request per lane and row
    // One round trip for everything that does not depend on anything else: the commit's state, the
    // keys, and this prompt's own inputs (read before it is known that g is an admitted prompt;
    // nothing is followed from them until then).
    const int32_t skip_v = st->skip;
    const int32_t nb_v = st->nb;
    const uint64_t key_v = ws.gkey[g];
    uint64_t kk[kRows];
#pragma unroll
    for (int t = 0; t < kRows; ++t) {
        const int32_t i = t * kWave + lane;
        kk[t] = ws.gkey[i < tv.max_batch ? i : tv.max_batch - 1];
    }
    GroupCtx ctx;
    ctx.clock0 = st->clock0;
    ctx.pool_top = st->pool_top;
    ctx.n_ent = 0;
    ctx.cache_ok = true;
    ctx.c_parent = ctx.c_tok = ctx.c_child = ctx.c_el = ctx.c_slot = -1;
    ctx.c_eo = 0;
    ctx.piece = -1;
    ctx.piece_slot = -1;
    ctx.piece_rec = NodeRec{};
    MemberIn lead;
    member_load_own(lead, batch_idx, ws, g);
    if (uni(skip_v)) return;
    const int32_t nb = uni(nb_v);
    if (g >= nb) return;
    const uint64_t key = uni64(key_v);
    if (key == kNoGroup) return;
    member_load_refs(lead, tv, q);
    // the first prompt of a group (in pick order) owns the group; bit t of `mine` = prompt 64t+lane
    // is a later member
    bool dup = false;
    uint32_t mine0 = 0;
#pragma unroll
    for (int t = 0; t < kRows; ++t) {
        const int32_t i = t * kWave + lane;
        const bool eq = i < nb && kk[t] == key;
        dup |= eq && i < g;
        if (eq && i > g) mine0 |= 1u << t;
    }
    for (int32_t base = kRows * kWave; base < g; base += 16 * kWave) {
        uint64_t k2[16];
#pragma unroll
        for (int t = 0; t < 16; ++t) {  // sixteen rows requested together
            const int32_t i = base + t * kWave + lane;
            k2[t] = ws.gkey[i < g ? i : g];
        }
#pragma unroll
        for (int t = 0; t < 16; ++t) dup |= (base + t * kWave + lane < g) && (k2[t] == key);
    }
    if (__ballot(dup)) {
        // Not the first of its group: that prompt's wavefront inserts this one.  Meanwhile this
        // wavefront measures how far the two unmatched tails agree, which lets the insertion walk
        // down the first prompt's new nodes without comparing tokens again (prompts of one group
        // typically share a long new prefix, and each later one would compare it once more).
        int32_t f = -1;
#pragma unroll
        for (int t = 0; t < kRows; ++t) {
            const int32_t i = t * kWave + lane;
            const uint64_t mk = __ballot(i < nb && i < g && kk[t] == key);
            if (mk && f < 0) f = t * kWave + (int32_t)__builtin_ctzll(mk);
        }
        int32_t h = kLcpNone;
        if (f >= 0) {
            const int32_t qf = batch_idx[f], mf = ws.bm_len[f];
            const MemberIn me = member_from_lane(lead, 0);
            if (uni(mf) == me.m && me.m < me.L) {
                const int64_t off_f = uni64(q.off[uni(qf)]);
                const int32_t len_f = uni(q.len[uni(qf)]);
                const int32_t lim = (len_f < me.L ? len_f : me.L) - me.m;
                if (lim > 0) h = wave_common_prefix(q.tokens + me.qoff + me.m, q.tokens + off_f + me.m, lim, lane);
            }
        }
        if (lane == 0) __hip_atomic_store(&ws.lcp_lead[g], h, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    const MemberIn first_in = member_from_lane(lead, 0);
    const int64_t lead_base = ctx.pool_top + first_in.to;
    const int32_t lead_m = first_in.m;
    insert_prompt(tv, q, ws, g, first_in, ctx, lane);
    // A later member's overlap with this prompt's tail: worked out by that member's own wavefront,
    // which started together with this one.  The wait is bounded; without an answer the insertion
    // compares tokens as it would have anyway.
    auto overlap_of = [&](int32_t j2) -> int32_t {
        if (j2 >= kRows * kWave) return kLcpNone;  // (members beyond the first rows do not look for their leader)
        int32_t h = kLcpPending;
        for (int spin = 0; spin < 2048; ++spin) {
            h = uni(__hip_atomic_load(&ws.lcp_lead[j2], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT));
            if (h != kLcpPending) break;
            __builtin_amdgcn_s_sleep(8);
        }
        return h;
    };
    // later members of the group; every lane that owns a member of a row fetches that member's inputs
    auto row = [&](int32_t row_base, bool is_mine) {
        uint64_t mask = __ballot(is_mine);
        if (!mask) return;
        const MemberIn mv = member_load(tv, q, batch_idx, ws, is_mine ? row_base + lane : g);
        while (mask) {
            int32_t b = (int32_t)__builtin_ctzll(mask);
            mask &= mask - 1ull;
            const MemberIn mi = member_from_lane(mv, b);
            const int32_t h = mi.m == lead_m ? overlap_of(row_base + b) : kLcpNone;
            insert_prompt(tv, q, ws, row_base + b, mi, ctx, lane, h, lead_base);
        }
    };
    if (__ballot(mine0 != 0)) {
        for (int t = g / kWave; t < kRows; ++t) row(t * kWave, (mine0 >> t) & 1u);
    }
    // beyond the first 1,024: 4096 candidates at a time, bit t of `mine` = candidate base+64t+lane
    for (int32_t base = g + 1 > kRows * kWave ? g + 1 : kRows * kWave; base < nb; base += 64 * kWave) {
        uint64_t mine = 0;
        const int32_t rows = (nb - base + kWave - 1) / kWave < 64 ? (nb - base + kWave - 1) / kWave : 64;
#pragma unroll 8
        for (int32_t t = 0; t < rows; ++t) {
            int32_t i = base + t * kWave + lane;
            uint64_t k1 = ws.gkey[i < nb ? i : nb - 1];
            if (i < nb && k1 == key) mine |= (1ull << t);
        }
        if (!__ballot(mine != 0)) continue;
        for (int32_t t = 0; t < 64 && base + t * kWave < nb; ++t) row(base + t * kWave, (mine >> t) & 1ull);
    }
}

// ------------------------------------------------------------------ ticks, then publish the inserts
__device__ __forceinline__ void ticks_body(TreeView tv, CommitWs ws, int64_t budget, int64_t protect, int tick_bits, int n_pass,
                                               int evict_enqueued) {
    DevState *st = tv.st;
    const int tid = threadIdx.x;
    const int32_t j = blockIdx.x * blockDim.x + tid;
    // Everything the publishing below reads was written by the kernels before this one, so every
    // workgroup asks for it at once - the state words with the prompt's end node, then what hangs on
    // the batch size - and whichever workgroup turns out to be the last has it in registers.
    const int32_t v0 = j < tv.max_batch ? ws.end_node[j] : kRoot;
    const int32_t skip = st->skip, nb = st->nb, f0 = st->free_cnt0, ns0 = st->n_slots0, nodes0 = st->n_nodes;
    const int32_t active_half = st->active_half;
    const uint64_t clock0 = st->clock0;
    const int64_t tail_total = st->tail_total, pool_top0 = st->pool_top, total0 = st->total_tokens;
    const int32_t A = 2 * nb;  // reservations: two per admitted prompt
    // each thread owns a contiguous run of reservations; the first eight of the run (all of it for
    // batches up to 1,024) and the first eight rows of the per-prompt counters are read here
    const int32_t per = (A + 255) / 256;
    const int32_t lo = tid * per < A ? tid * per : A;
    const int32_t hi = lo + per < A ? lo + per : A;
    int32_t u[8], lt[8], head_u[8], head_id[8];
    if (!skip) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int32_t j2 = tid + t * 256;
            u[t] = j2 < nb ? ws.used[j2] : 0;
            lt[t] = j2 < nb ? ws.leaf_tok[j2] : 0;
            const int32_t a = lo + t;
            head_u[t] = a < hi ? ((ws.used[a >> 1] >> (a & 1)) & 1) : 1;
            head_id[t] = a < hi ? ws.resv_id[a] : 0;
        }
    }
    if (!skip && j < nb) {
        const uint64_t t = clock0 + (uint64_t)j;
        int32_t v = v0;
        for (int32_t guard = 0; guard <= tv.max_prompt_len && v > kRoot && v < tv.max_nodes; ++guard) {
            const int32_t up = tv.parent[v];  // requested together with the atomic: one round trip per level
            unsigned long long old = atomicMax((unsigned long long *)&tv.tick[v], (unsigned long long)t);
            // a strictly later prompt already stamped this node and stamps its ancestors too; an equal
            // value is this prompt's own stamp on a node it created, so keep climbing
            if (old > (unsigned long long)t) break;
            v = up;
        }
    }
    // the last workgroup publishes the inserts and decides whether anything must be evicted
    __shared__ int evict;
    __shared__ int32_t sbuf[256 / kWave];
    __shared__ int32_t s_carry;
    __shared__ unsigned long long s_tok;
    __shared__ int32_t s_new;
    if (!last_block_done(st, 1)) return;
    if (tid == 0) { s_carry = 0; s_tok = 0; s_new = 0; evict = 0; }
    __syncthreads();
    if (!skip) {
        // give back the reserved node ids that were not used, count what was added
        const int32_t from_free = A < f0 ? A : f0;
        const int32_t base = f0 - from_free;
        unsigned long long my_tok = 0;
        int32_t my_new = 0;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            my_new += (u[t] & 1) + ((u[t] >> 1) & 1);
            my_tok += (unsigned long long)lt[t];
        }
        // (further rows in groups of eight, all requested before any is used: a loop that uses each
        // value at once pays a round trip per iteration)
        for (int32_t j0 = tid + 8 * 256; j0 < nb; j0 += 8 * 256) {
            int32_t u2[8], lt2[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int32_t j2 = j0 + t * 256;
                u2[t] = j2 < nb ? ws.used[j2] : 0;
                lt2[t] = j2 < nb ? ws.leaf_tok[j2] : 0;
            }
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                my_new += (u2[t] & 1) + ((u2[t] >> 1) & 1);
                my_tok += (unsigned long long)lt2[t];
            }
        }
        // (summed across the wavefront first: 256 atomics on one LDS word are served one by one)
        my_tok = wave_sum(my_tok);
        my_new = wave_sum(my_new);
        if ((tid & (kWave - 1)) == 0) {
            atomicAdd(&s_tok, my_tok);
            atomicAdd(&s_new, my_new);
        }
        // one scan places the unused reservations
        int32_t cnt = 0;
#pragma unroll
        for (int t = 0; t < 8; ++t) cnt += head_u[t] ? 0 : 1;
        for (int32_t a = lo + 8; a < hi; ++a) cnt += ((ws.used[a >> 1] >> (a & 1)) & 1) ? 0 : 1;
        int32_t unused_total;
        int32_t incl = block_inclusive_scan<int32_t, 256>(cnt, sbuf, tid, unused_total);
        int32_t dst = base + incl - cnt;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (!head_u[t]) {
                if (dst >= 0 && dst < tv.max_nodes) tv.free_stack[dst] = head_id[t];
                ++dst;
            }
        }
        for (int32_t a = lo + 8; a < hi; ++a) {
            if (((ws.used[a >> 1] >> (a & 1)) & 1) == 0) {
                if (dst >= 0 && dst < tv.max_nodes) tv.free_stack[dst] = ws.resv_id[a];
                ++dst;
            }
        }
        if (tid == 255) s_carry = unused_total;
        __syncthreads();
    }
    if (tid == 0 && !skip) {
        // (stores only: what they are computed from came with the first round trip)
        const uint64_t clock = clock0 + (uint64_t)nb;
        const int64_t inserted = (int64_t)s_tok;
        const int64_t pool_top = pool_top0 + tail_total;
        const int64_t total = total0 + inserted;
        st->clock = clock;
        st->free_cnt = f0 - (A < f0 ? A : f0) + s_carry;
        if (A > f0) st->n_slots = ns0 + (A - f0);
        st->inserted_tokens = inserted;
        st->new_nodes = s_new;
        st->pool_top = pool_top;
        st->total_tokens = total;
        st->n_nodes = nodes0 + s_new;
        // pool compaction at the end of this commit: wanted when the active half could not take a
        // worst-case batch any more, useful when part of what it holds is garbage (spans of
        // evicted nodes; an eviction further down only adds to it)
        {
            const int64_t half_base = (int64_t)active_half * tv.pool_half;
            const int64_t room = half_base + tv.pool_half - pool_top;
            const int64_t used = pool_top - half_base;
            const int64_t worst = (int64_t)tv.max_batch * (int64_t)tv.max_prompt_len;
            if (room < worst && (used > total || total > budget)) {
                st->need_compact = 1;
                st->compact_cursor = (int64_t)(1 - active_half) * tv.pool_half;
            }
        }
        // the paths of the `protect` most recently admitted prompts (this batch included) stay
        st->keep_from = protect <= 0 ? ~0ull : ((uint64_t)protect >= clock ? 0ull : clock - (uint64_t)protect);
        int64_t need = total - budget;
        if (tick_bits < 64 && (clock >> tick_bits) != 0) {
            // the eviction passes enqueued behind this kernel were sized for a smaller clock
            flag_error(st, 16u /* KLPM_DEV_CLOCK_RANGE */);
            need = 0;
        }
        if (need > 0 && !evict_enqueued) {
            // the host left the eviction kernels out because the budget is at least what the
            // pool can hold: being over it means the counters are wrong
            flag_error(st, kDevInternal);
            need = 0;
        }
        if (need > 0) {
            st->do_evict = 1;
            st->need_evict = need;
            st->evict_rem = need;
            st->evict_prefix = 0;
            st->evict_all = 0;
            st->cand_cnt = 0;
            evict = 1;
        }
    }
    __syncthreads();
    if (evict)
        for (int i = tid; i < n_pass * kEvictBins; i += blockDim.x) ws.evict_hist[i] = 0;
}
__global__ __launch_bounds__(256) void k_ticks(TreeView tv, CommitWs ws, int64_t budget, int64_t protect, int tick_bits, int n_pass,
                                               int evict_enqueued) {
    ticks_body(tv, ws, budget, protect, tick_bits, n_pass, evict_enqueued);
}

// ------------------------------------------------------------------ eviction
// Order of removal: tick ascending, then depth descending (the deepest node of the oldest path is
// the one leaf carrying the smallest tick).  key = tick * 2^depth_bits + (depth_mask - depth_end).
// The cut key is found from the top: weighted digit histograms over all nodes narrow the key down to
// a window of 64 ticks; the few nodes inside that window are then collected and sorted, and a prefix
// sum of their lengths gives the exact cut.
constexpr int kEvictTailTicks = 6;  // log2 of the tick window that the sorting pass takes over

__device__ __forceinline__ uint64_t evict_key(const TreeView &tv, int64_t id, int depth_bits) {
    uint64_t dm = (1ull << depth_bits) - 1ull;
    return (tv.tick[id] << depth_bits) | (dm - (uint64_t)(uint32_t)tv.depth_end[id]);
}

// The sweeps over all nodes visit four nodes per thread and trip, every field requested before any
// is looked at (one round trip per trip; a loop that tests edge_len, then tick, then builds the key
// pays three per node).  f(id, edge_len, key) is called for every live node that may be evicted.
template <bool WITH_SLOT, bool WITH_DEPTH, int kUnroll, class F>
__device__ __forceinline__ void for_each_evictable_impl(const TreeView &tv, int32_t n_slots, uint64_t keep_from, int depth_bits,
                                                        int64_t first, int64_t stride, F f) {
    const uint64_t dm = (1ull << depth_bits) - 1ull;
    for (int64_t id0 = first; id0 < n_slots; id0 += kUnroll * stride) {
        int32_t len[kUnroll], de[kUnroll], sl[kUnroll];
        uint64_t tk[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t id = id0 + u * stride;
            const int64_t idc = id < n_slots ? id : 0;  // (the root has no edge: skipped below)
            len[u] = tv.edge_len[idc];
            tk[u] = tv.tick[idc];
            de[u] = WITH_DEPTH ? tv.depth_end[idc] : 0;
            sl[u] = WITH_SLOT ? tv.slot_of[idc] : -1;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t id = id0 + u * stride;
            if (id >= n_slots || len[u] <= 0 || tk[u] >= keep_from) continue;
            f(id, len[u], (tk[u] << depth_bits) | (dm - (uint64_t)(uint32_t)de[u]), sl[u]);
        }
    }
}
// f(id, edge_len, key)
template <class F>
__device__ __forceinline__ void for_each_evictable(const TreeView &tv, int32_t n_slots, uint64_t keep_from, int depth_bits,
                                                   int64_t first, int64_t stride, F f) {
    for_each_evictable_impl<false, true, 4>(tv, n_slots, keep_from, depth_bits, first, stride,
                                         [&](int64_t id, int32_t len, uint64_t key, int32_t) { f(id, len, key); });
}
// f(id, edge_len, key, slot): also brings the node's child-table slot along (for sweeps that remove nodes)
template <class F>
__device__ __forceinline__ void for_each_evictable_slot(const TreeView &tv, int32_t n_slots, uint64_t keep_from,
                                                        int depth_bits, int64_t first, int64_t stride, F f) {
    for_each_evictable_impl<true, true, 4>(tv, n_slots, keep_from, depth_bits, first, stride, f);
}

// f(id, edge_len, key, slot) for the nodes whose tick passes want(tick): only edge length and tick are read
// for every node, depth and table slot for those few (the sweep of a windowed eviction, whose window is a
// range of ticks)
template <class W, class F>
__device__ __forceinline__ void for_each_evictable_wanted(const TreeView &tv, int32_t n_slots, uint64_t keep_from,
                                                          int depth_bits, int64_t first, int64_t stride, W want, F f) {
    constexpr int kUnroll = 8;
    const uint64_t dm = (1ull << depth_bits) - 1ull;
    for (int64_t id0 = first; id0 < n_slots; id0 += kUnroll * stride) {
        int32_t len[kUnroll];
        uint64_t tk[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t id = id0 + u * stride;
            const int64_t idc = id < n_slots ? id : 0;  // (the root has no edge: skipped below)
            len[u] = tv.edge_len[idc];
            tk[u] = tv.tick[idc];
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t id = id0 + u * stride;
            if (id >= n_slots || len[u] <= 0 || tk[u] >= keep_from || !want(tk[u])) continue;
            const int32_t de = tv.depth_end[id], sl = tv.slot_of[id];
            f(id, len[u], (tk[u] << depth_bits) | (dm - (uint64_t)(uint32_t)de), sl);
        }
    }
}

// f(id, edge_len, key) with the depth part of the key left at its largest value: for sweeps that only look at
// key bits above the depth (the digit histograms), which then need not read the depths
template <class F>
__device__ __forceinline__ void for_each_evictable_tick(const TreeView &tv, int32_t n_slots, uint64_t keep_from,
                                                        int depth_bits, int64_t first, int64_t stride, F f) {
    for_each_evictable_impl<false, false, 8>(tv, n_slots, keep_from, depth_bits, first, stride,
                                          [&](int64_t id, int32_t len, uint64_t key, int32_t) { f(id, len, key); });
}

// One step of the search for the cut key, run by one workgroup of 256 threads once the weighted
// histogram of the current digit (`width` bits) is complete: pick the smallest digit whose inclusive
// weight reaches what is still to be freed, append it to the prefix and reduce the remainder.  When
// the nodes that may go (protected ones are left out of the histograms) do not free enough, all of
// them go.
__device__ void evict_descend_step(DevState *st, const int64_t *hist, int width, bool first) {
    __shared__ int64_t part[256 / kWave];
    __shared__ int pick;
    __shared__ int64_t s_below;
    const int tid = threadIdx.x;
    constexpr int per = kEvictBins / 256;  // contiguous bins per thread
    const int64_t rem = st->evict_rem;
    __syncthreads();
    if (tid == 0) { pick = (1 << width) - 1; s_below = 0; }
    int64_t w[per];
    int64_t mine = 0;
#pragma unroll
    for (int q = 0; q < per; ++q) {
        w[q] = hist[tid * per + q];
        mine += w[q];
    }
    int64_t all;
    int64_t run = block_inclusive_scan<int64_t, 256>(mine, part, tid, all) - mine;  // weight of the lower bins
#pragma unroll
    for (int q = 0; q < per; ++q) {
        if (run < rem && run + w[q] >= rem) { pick = tid * per + q; s_below = run; }
        run += w[q];
    }
    __syncthreads();
    if (tid == 0) {
        if (first && all < rem) st->evict_all = 1;
        st->evict_rem = rem - s_below;
        st->evict_prefix = (st->evict_prefix << width) | (uint64_t)pick;
    }
    __syncthreads();
}

// Histogram pass over every node: digit = bits [shift, shift + width) of the key, among the nodes
// whose higher key bits equal the prefix found so far.
__global__ __launch_bounds__(256) void k_evict_hist(TreeView tv, CommitWs ws, int pass, int shift, int width,
                                                    int depth_bits) {
    DevState *st = tv.st;
    const int do_evict = st->do_evict;  // (the state words are requested together)
    const uint64_t prefix = st->evict_prefix;  // digits fixed by the earlier passes
    const int32_t n_slots = st->n_slots;
    const uint64_t keep_from = st->keep_from;
    if (!do_evict) return;
    __shared__ unsigned long long h[kEvictBins];
    const int tid = threadIdx.x;
    for (int i = tid; i < kEvictBins; i += 256) h[i] = 0;
    __syncthreads();
    const int upper = shift + width;
    // (shift >= depth_bits: the digits of the histograms lie in the tick)
    for_each_evictable_tick(tv, n_slots, keep_from, depth_bits, 1 + (int64_t)blockIdx.x * blockDim.x + tid,
                            (int64_t)gridDim.x * blockDim.x, [&](int64_t, int32_t len, uint64_t key) {
        bool in_prefix = (pass == 0) || (upper >= 64 ? prefix == 0 : (key >> upper) == prefix);
        if (in_prefix) atomicAdd(&h[(key >> shift) & (uint64_t)((1 << width) - 1)], (unsigned long long)len);
    });
    __syncthreads();
    for (int i = tid; i < (1 << width); i += 256)
        if (h[i]) atomicAdd((unsigned long long *)&ws.evict_hist[pass * kEvictBins + i], h[i]);
    if (last_block_done(st, 4 + pass)) evict_descend_step(st, ws.evict_hist + pass * kEvictBins, width, pass == 0);
}

// Removes one live node: a tombstone in the table slot that leads to it (probe chains stay intact),
// its id back on the free stack; its tokens and the node are added to the two workgroup counters.
__device__ __forceinline__ void evict_remove_node(const TreeView &tv, DevState *st, int64_t id, int32_t len, int32_t slot,
                                                  unsigned long long *s_tok, int *s_cnt) {
    const int32_t pos = atomicAdd(&st->free_cnt, 1);
    tv.edge_len[id] = 0;
    if (slot >= 0 && (uint32_t)slot <= tv.slot_mask)
        __hip_atomic_store(&tv.slots[slot].key, kTombKey, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
        flag_error(st, kDevInternal);
    if (pos >= 0 && pos < tv.max_nodes) tv.free_stack[pos] = (int32_t)id;
    atomicAdd(s_tok, (unsigned long long)len);
    atomicAdd(s_cnt, 1);
}
// Removals of one workgroup, listed in LDS first: the workgroup then takes its places on the free
// stack with one atomic for all of them (an atomic per node on the one counter is served one by one,
// and a commit removes a thousand nodes and more).
constexpr int kRemovalList = 1024;
struct RemovalList {
    int32_t *ids, *slots;  // [kRemovalList] in LDS
    int32_t *n;            // LDS counter, zeroed by the caller
};
__device__ __forceinline__ void removal_push(const TreeView &tv, DevState *st, const RemovalList &rl, int64_t id, int32_t len,
                                             int32_t slot, unsigned long long *s_tok, int *s_cnt) {
    const int32_t at = atomicAdd(rl.n, 1);
    if (at < kRemovalList) {
        rl.ids[at] = (int32_t)id;
        rl.slots[at] = slot;
        atomicAdd(s_tok, (unsigned long long)len);
        atomicAdd(s_cnt, 1);
    } else {
        evict_remove_node(tv, st, id, len, slot, s_tok, s_cnt);  // (the list is full: one by one)
    }
}
// Every thread of the workgroup calls it (barriers inside); the list is empty afterwards.
__device__ __forceinline__ void removal_flush(const TreeView &tv, DevState *st, const RemovalList &rl, int tid, int n_threads) {
    __shared__ int32_t s_base;
    __syncthreads();
    const int32_t n = *rl.n < kRemovalList ? *rl.n : kRemovalList;
    if (tid == 0) s_base = n > 0 ? atomicAdd(&st->free_cnt, n) : 0;
    __syncthreads();
    const int32_t base = s_base;
    for (int32_t i = tid; i < n; i += n_threads) {
        const int32_t id = rl.ids[i], slot = rl.slots[i];
        tv.edge_len[id] = 0;
        if (slot >= 0 && (uint32_t)slot <= tv.slot_mask)
            __hip_atomic_store(&tv.slots[slot].key, kTombKey, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else
            flag_error(st, kDevInternal);
        const int32_t pos = base + i;
        if (pos >= 0 && pos < tv.max_nodes) tv.free_stack[pos] = id;
    }
    __syncthreads();
    if (tid == 0) *rl.n = 0;
    __syncthreads();
}
// Removes every live, unprotected node with key <= cut among the nodes first, first + stride, ...
__device__ __forceinline__ void evict_apply_sweep(const TreeView &tv, DevState *st, uint64_t cut, uint64_t keep_from,
                                                  int32_t n_slots, int depth_bits, int64_t first, int64_t stride,
                                                  unsigned long long *s_tok, int *s_cnt) {
    for_each_evictable_slot(tv, n_slots, keep_from, depth_bits, first, stride,
                            [&](int64_t id, int32_t len, uint64_t node_key, int32_t slot) {
        if (node_key <= cut) evict_remove_node(tv, st, id, len, slot, s_tok, s_cnt);
    });
}
// Books the removal (one thread, after every workgroup has added its counts): the child table is
// rebuilt at the end of this commit once tombstones start to lengthen the probe sequences.
__device__ __forceinline__ void evict_apply_publish(const TreeView &tv, DevState *st, int64_t ev_tok, int32_t ev_cnt) {
    st->total_tokens -= ev_tok;
    st->n_nodes -= ev_cnt;
    st->tombstones += ev_cnt;
    if ((int64_t)st->tombstones * 4 > (int64_t)tv.slot_mask + 1 && !st->need_compact) st->need_rebuild = 1;
}

// Last stretch of the search and the removal itself, in one sweep over the nodes.  The digit passes
// have narrowed the cut key down to the keys that agree with `prefix` above bit `shift`: a node
// whose key lies below that window goes for certain and is removed on the spot; the nodes inside the
// window (few: a window is 64 ticks wide) are collected, and the last workgroup to finish sorts them
// by key, cuts where their lengths add up to what is left to free, and removes those up to the cut.
// More nodes in the window than the sort holds (very deep paths stamped by few prompts) are handled
// by that workgroup with digit passes of its own over all nodes.
__device__ __forceinline__ void evict_gather_body(TreeView tv, CommitWs ws, int n_hist_pass, int shift, int depth_bits) {
    DevState *st = tv.st;
    const int do_evict = st->do_evict;
    const uint64_t prefix = st->evict_prefix;
    const int32_t n_slots = st->n_slots;
    const uint64_t keep_from = st->keep_from;
    const bool evict_all = st->evict_all != 0;
    if (!do_evict) return;
    __shared__ uint64_t s_key[kEvictCand];
    __shared__ int32_t s_len[kEvictCand];
    __shared__ int64_t part[256 / kWave];
    __shared__ unsigned long long s_cut;
    __shared__ unsigned long long s_tok;
    __shared__ int s_cnt;
    __shared__ int32_t l_ids[kRemovalList], l_slots[kRemovalList];
    __shared__ int32_t c_id[kEvictCand], c_slot[kEvictCand];
    __shared__ int32_t s_nrem, s_ncand, s_cbase;
    const RemovalList rl{l_ids, l_slots, &s_nrem};
    const int tid = threadIdx.x;
    if (tid == 0) { s_tok = 0; s_cnt = 0; s_nrem = 0; s_ncand = 0; }
    __syncthreads();
    const bool windowed = n_hist_pass > 0 && shift < 64;  // (otherwise every node that may go is a candidate)
    // (removals and candidates are listed in LDS: one atomic per workgroup on each of the shared counters)
    auto take = [&](int64_t id, int32_t len, uint64_t key, int32_t slot) {
        const uint64_t top = windowed ? (key >> shift) : 0ull;
        if (evict_all || (windowed && top < prefix)) {
            removal_push(tv, st, rl, id, len, slot, &s_tok, &s_cnt);
        } else if (!windowed || top == prefix) {
            const int32_t at = atomicAdd(&s_ncand, 1);
            if (at < kEvictCand) {  // (more than that in one workgroup: the search takes its other road, which only needs the count)
                s_key[at] = key;
                s_len[at] = len;
                c_id[at] = (int32_t)id;
                c_slot[at] = slot;
            }
        }
    };
    const int64_t first = 1 + (int64_t)blockIdx.x * blockDim.x + tid, stride = (int64_t)gridDim.x * blockDim.x;
    if (windowed && !evict_all && shift >= depth_bits) {
        // the window is a range of ticks: nodes above it (nearly all) are passed over on their tick alone
        const int tshift = shift - depth_bits;
        for_each_evictable_wanted(tv, n_slots, keep_from, depth_bits, first, stride,
                                  [&](uint64_t tick) { return (tick >> tshift) <= prefix; }, take);
    } else {
        for_each_evictable_slot(tv, n_slots, keep_from, depth_bits, first, stride, take);
    }
    removal_flush(tv, st, rl, tid, 256);
    if (tid == 0) s_cbase = s_ncand > 0 ? atomicAdd(&st->cand_cnt, s_ncand) : 0;
    __syncthreads();
    {
        const int32_t nc = s_ncand < kEvictCand ? s_ncand : kEvictCand, cbase = s_cbase;
        for (int32_t i = tid; i < nc; i += 256) {
            const int32_t at = cbase + i;
            if (at < kEvictCand) {
                ws.cand_key[at] = s_key[i];
                ws.cand_len[at] = s_len[i];
                ws.cand_id[at] = c_id[i];
                ws.cand_slot[at] = c_slot[i];
            }
        }
    }
    __syncthreads();
    if (tid == 0 && s_cnt) {
        atomicAdd((unsigned long long *)&st->evicted_tokens, s_tok);
        atomicAdd(&st->evicted_nodes, s_cnt);
    }
    if (!last_block_done(st, 10)) return;
    if (tid == 0) { s_tok = 0; s_cnt = 0; s_cut = ~0ull; }
    __syncthreads();
    const int32_t n = __hip_atomic_load(&st->cand_cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (evict_all) {
        // (everything that may go has gone in the sweeps)
    } else if (n > kEvictCand) {
        // digit passes over all nodes by this workgroup alone (rare): the remaining `shift` bits of the key
        unsigned long long *h = reinterpret_cast<unsigned long long *>(s_key);  // kEvictBins words fit
        int low = shift;
        while (low > 0) {
            const int width = low % kEvictDigitBits ? low % kEvictDigitBits : kEvictDigitBits;
            low -= width;
            const uint64_t pre = st->evict_prefix;
            for (int i = tid; i < kEvictBins; i += 256) h[i] = 0;
            __syncthreads();
            for (int64_t id = 1 + tid; id < n_slots; id += 256) {
                int32_t len = tv.edge_len[id];
                if (len <= 0 || tv.tick[id] >= keep_from) continue;
                uint64_t key = evict_key(tv, id, depth_bits);
                const int upper = low + width;
                bool in_prefix = (n_hist_pass == 0 && upper == shift) || upper >= 64 || (key >> upper) == pre;
                if (in_prefix) atomicAdd(&h[(key >> low) & (uint64_t)((1 << width) - 1)], (unsigned long long)len);
            }
            __syncthreads();
            evict_descend_step(st, reinterpret_cast<const int64_t *>(h), width, false);
        }
        // the key is complete: what lies below the window is gone already, the rest up to the cut goes now
        evict_apply_sweep(tv, st, st->evict_prefix, keep_from, n_slots, depth_bits, 1 + tid, 256, &s_tok, &s_cnt);
    } else {
        const int64_t rem = st->evict_rem;
        if (n <= 256) {
            // few collected nodes (the rule): no sort - every thread adds up the weights of the nodes whose
            // key is not above its own node's; the node at which that sum reaches the remainder is the last
            // one to go (all of them, should the weights fall short)
            if (tid < n) {
                s_key[tid] = __hip_atomic_load(&ws.cand_key[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_len[tid] = __hip_atomic_load(&ws.cand_len[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __syncthreads();
            if (tid < n) {
                const uint64_t mine = s_key[tid];
                int64_t upto = 0;
                for (int32_t i0 = 0; i0 < n; i0 += 16) {  // (sixteen LDS reads in flight; entries past n hold what an earlier commit left: masked)
                    uint64_t kk[16];
                    int32_t ll[16];
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        const int32_t i = (i0 + u) & (kEvictCand - 1);
                        kk[u] = s_key[i];
                        ll[u] = s_len[i];
                    }
#pragma unroll
                    for (int u = 0; u < 16; ++u) upto += (i0 + u < n && kk[u] <= mine) ? (int64_t)ll[u] : 0;
                }
                if (upto - (int64_t)s_len[tid] < rem && upto >= rem) s_cut = mine;
            }
            __syncthreads();
        } else {
            // sort the collected nodes by key in LDS, then the cut
            int32_t np2 = 1;
            while (np2 < n) np2 <<= 1;
            for (int32_t i = tid; i < np2; i += 256) {
                s_key[i] = i < n ? __hip_atomic_load(&ws.cand_key[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : ~0ull;
                s_len[i] = i < n ? __hip_atomic_load(&ws.cand_len[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
            }
            __syncthreads();
            sort_lds<256, kEvictCand / 256, true>(s_key, reinterpret_cast<uint32_t *>(s_len), np2, tid);
            // every thread owns a contiguous run of the sorted nodes; the node at which the running weight
            // reaches the remainder is the last one to go (all of them, should the weights fall short)
            const int32_t per = (n + 255) / 256;
            const int32_t lo = tid * per < n ? tid * per : n, hi = lo + per < n ? lo + per : n;
            int64_t mine = 0;
            for (int32_t i = lo; i < hi; ++i) mine += s_len[i];
            int64_t all;
            int64_t run = block_inclusive_scan<int64_t, 256>(mine, part, tid, all) - mine;
            for (int32_t i = lo; i < hi; ++i) {
                if (run < rem && run + s_len[i] >= rem) s_cut = s_key[i];
                run += s_len[i];
            }
            __syncthreads();
        }
        const uint64_t cut = s_cut;
        if (tid == 0) st->evict_prefix = cut;
        // keys are unique among live nodes (nodes that share a tick lie on one root path, at
        // different depths), so the collected nodes up to the cut are removed as they were stored
        for (int32_t i = tid; i < n; i += 256) {
            const uint64_t key = __hip_atomic_load(&ws.cand_key[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int32_t id = __hip_atomic_load(&ws.cand_id[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int32_t len = __hip_atomic_load(&ws.cand_len[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int32_t slot = __hip_atomic_load(&ws.cand_slot[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (key <= cut) removal_push(tv, st, rl, id, len, slot, &s_tok, &s_cnt);
        }
        removal_flush(tv, st, rl, tid, 256);
    }
    __syncthreads();
    if (tid == 0) {
        const int64_t ev_tok = (int64_t)__hip_atomic_load((unsigned long long *)&st->evicted_tokens, __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT) + (int64_t)s_tok;
        const int32_t ev_cnt = __hip_atomic_load(&st->evicted_nodes, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + s_cnt;
        st->evicted_tokens = ev_tok;
        st->evicted_nodes = ev_cnt;
        evict_apply_publish(tv, st, ev_tok, ev_cnt);
    }
}
__global__ __launch_bounds__(256) void k_evict_gather(TreeView tv, CommitWs ws, int n_hist_pass, int shift, int depth_bits) {
    evict_gather_body(tv, ws, n_hist_pass, shift, depth_bits);
}

// The whole commit of at most one prompt into a small tree (no more nodes than the eviction's sorting
// pass holds) in one launch of one workgroup: plan and tail copy, the insertion (first wavefront),
// the tick walk and the publishing, the eviction, the end-of-commit maintenance and the counters, one
// after the other with a workgroup barrier between them.  This is the shape of a scheduler that
// serves one query per step (Def. 2 as it stands): five dependent launches of a few microseconds
// each become one.
__global__ __launch_bounds__(kFusedThreads) void k_commit_one(TreeView tv, QView q, const int32_t *__restrict__ batch_idx,
                                                              const int32_t *__restrict__ n_selected, int32_t batch_cap,
                                                              CommitWs ws, const int32_t *__restrict__ hint_len,
                                                              const int32_t *__restrict__ hint_node, int64_t budget,
                                                              int64_t protect, int tick_bits, int final_shift,
                                                              int depth_bits, int may_evict,
                                                              kLPM_stats *__restrict__ stats_out) {
    // The steps below are chains of dependent reads of a few words each, and what they read was last
    // written by other kernels, possibly through another XCD's L2: every read would come from memory.  One
    // read per 64-byte line of everything they may touch (the node arrays and the child table of a small
    // tree, the commit's state and per-prompt records: some tens of KB), asked for at once up front, brings
    // it close before it is needed (measured on a Def. 3 queue: 27.4 -> 22.5 us for the whole kernel).
    {
        int32_t acc = 0;
        const int t = threadIdx.x;
        const int32_t mn = tv.max_nodes;
        for (int32_t i = t * 16; i < mn; i += kFusedThreads * 16)
            acc += tv.parent[i] + tv.edge_len[i] + tv.depth_end[i] + tv.slot_of[i] + tv.free_stack[i];
        for (int32_t i = t * 8; i < mn; i += kFusedThreads * 8) acc += (int32_t)tv.tick[i] + (int32_t)tv.edge_off[i];
        for (uint32_t i = t * 2u; i <= tv.slot_mask; i += kFusedThreads * 2u) acc += (int32_t)tv.slots[i].key;
        if (t * 16 < (int)(sizeof(DevState) / 4)) acc += reinterpret_cast<const int32_t *>(tv.st)[t * 16];
        if (t == 0) {
            acc += ws.bm_len[0] + ws.bm_node[0] + (int32_t)ws.tail_off[0] + (int32_t)ws.gkey[0] + ws.end_node[0] + ws.used[0] +
                   ws.leaf_tok[0] + ws.next_tok[0] + ws.lcp_lead[0] + ws.resv_id[0] + (int32_t)ws.p_off[0] + ws.p_len[0] +
                   ws.p_de[0] + ws.cand_id[0] + (int32_t)ws.cand_key[0] + ws.cand_len[0] + ws.cand_slot[0];
        }
        asm volatile("" ::"v"(acc));  // (the values are not used; the reads are)
    }
    // (one workgroup: the barrier between two steps orders what the first wrote before what the second reads)
    plan_copy_body<kFusedThreads, 1>(tv, q, batch_idx, n_selected, batch_cap, ws, hint_len, hint_node);
    __syncthreads();
    if (batch_cap > 0 && threadIdx.x < kWave) structure_body(tv, q, batch_idx, ws);
    __syncthreads();
    ticks_body(tv, ws, budget, protect, tick_bits, 0, may_evict);
    __syncthreads();
    if (may_evict) evict_gather_body(tv, ws, 0, final_shift, depth_bits);
    __syncthreads();
    end_commit_small_body<kFusedThreads>(tv, stats_out);
}

int commit_pipeline(kLPM_tree *t, const QView &q, const int32_t *batch_idx, const int32_t *n_selected,
                    int32_t batch_cap, int64_t budget, int64_t protect, kLPM_stats *stats_out, hipStream_t stream,
                    const int32_t *hint_len, const int32_t *hint_node) {
    const TreeView &tv = t->tv;
    const CommitWs &ws = t->ws;
    if (batch_cap > t->cfg.max_batch) batch_cap = t->cfg.max_batch;
    // eviction key = (tick, inverted depth); its width follows from host-known upper bounds
    const uint64_t clock_ub = t->clock_ub + (uint64_t)(batch_cap > 0 ? batch_cap : 0);
    const uint64_t clock_bound = clock_ub + t->clock_reserve;
    int tick_bits = 1;
    while (tick_bits < 64 && (clock_bound >> tick_bits)) ++tick_bits;
    const int key_bits = tick_bits + t->depth_bits;
    if (key_bits > 64) return KLPM_EINVAL;
    // digit passes narrow the tick down to a window of 2^tail ticks, the sorting pass does the rest
    const int tail = tick_bits < kEvictTailTicks ? tick_bits : kEvictTailTicks;
    const int hist_bits = tick_bits - tail;
    // (a tree of no more nodes than the sorting pass takes needs no digit passes at all)
    const bool tiny = tv.max_nodes <= kEvictCand;
    const int n_pass = tiny ? 0 : (hist_bits + kEvictDigitBits - 1) / kEvictDigitBits;  // <= 6: the arena holds six histograms
    const int final_shift = tiny ? key_bits : t->depth_bits + tail;  // key bits left to the sorting pass
    t->clock_ub = clock_ub;
    if (batch_cap > 0 && !hint_len) {
        int rc = launch_match(tv, q, batch_idx, n_selected, batch_cap, 1, ws.bm_len, ws.bm_node, stream);
        if (rc) return rc;
    }
    // Every live edge sits in the active half of the token pool, so a budget of at least that half
    // can never be exceeded: the eviction kernels (no-ops that still cost a launch each) are left out.
    const bool may_evict = budget < tv.pool_half;
    if (tiny && batch_cap <= 1) {
        hipLaunchKernelGGL(k_commit_one, dim3(1), dim3(kFusedThreads), 0, stream, tv, q, batch_idx, n_selected, batch_cap, ws,
                           hint_len, hint_node, budget, protect, tick_bits, final_shift, t->depth_bits, may_evict ? 1 : 0,
                           stats_out);
        return check_launch();
    }
    if (batch_cap <= kPlanSmallBatch) {
        hipLaunchKernelGGL(k_plan_copy_small, dim3(batch_cap > 0 ? batch_cap : 1), dim3(kFusedThreads), 0, stream, tv, q,
                           batch_idx, n_selected, batch_cap, ws, hint_len, hint_node);
    } else if (batch_cap <= kFusedPlanMax) {
        hipLaunchKernelGGL(k_plan_copy, dim3((batch_cap + kPlanGroup - 1) / kPlanGroup), dim3(kPlanCopyThreads), 0, stream,
                           tv, q, batch_idx, n_selected, batch_cap, ws, hint_len, hint_node);
    } else {
        hipLaunchKernelGGL(k_commit_plan, dim3(1), dim3(kPlanThreads), 0, stream, tv, q, batch_idx, n_selected, batch_cap,
                           ws, hint_len, hint_node);
        hipLaunchKernelGGL(k_copy_tails, dim3(batch_cap), dim3(256), 0, stream, tv, q, batch_idx, ws, hint_len ? 1 : 0);
    }
    if (batch_cap > 16 * kWave)
        hipLaunchKernelGGL(k_structure_wide, dim3(batch_cap), dim3(kWave), 0, stream, tv, q, batch_idx, ws);
    else if (batch_cap > 0)
        hipLaunchKernelGGL(k_structure, dim3(batch_cap), dim3(kWave), 0, stream, tv, q, batch_idx, ws);
    hipLaunchKernelGGL(k_ticks, dim3(batch_cap > 0 ? (batch_cap + 255) / 256 : 1), dim3(256), 0, stream, tv, ws,
                       budget, protect, tick_bits, n_pass, may_evict ? 1 : 0);
    if (may_evict) {
        // (few, fat workgroups: each ends with atomics on shared words - its histogram bins, the
        // counter that tells the last workgroup - which are served one by one)
        unsigned ge = (unsigned)(((int64_t)tv.max_nodes + 4095) / 4096);
        if (ge > 128u) ge = 128u;
        for (int p = 0; p < n_pass; ++p) {
            // the first digit takes what the others leave over, so that the last one ends at final_shift
            const int shift = final_shift + kEvictDigitBits * (n_pass - 1 - p);
            const int width = p == 0 ? hist_bits - kEvictDigitBits * (n_pass - 1) : kEvictDigitBits;
            hipLaunchKernelGGL(k_evict_hist, dim3(ge), dim3(256), 0, stream, tv, ws, p, shift, width, t->depth_bits);
        }
        hipLaunchKernelGGL(k_evict_gather, dim3(ge), dim3(256), 0, stream, tv, ws, n_pass, final_shift, t->depth_bits);
    }
    // the end of the commit: grid sized for pool compaction, one wavefront per node
    if (tiny) {
        hipLaunchKernelGGL(k_end_commit_small, dim3(1), dim3(kSmallMaintainThreads), 0, stream, tv, stats_out);
    } else {
        unsigned gn = (unsigned)(((int64_t)tv.max_nodes + 3) / 4);
        if (gn > 1024u) gn = 1024u;
        hipLaunchKernelGGL(k_end_commit, dim3(gn), dim3(256), 0, stream, tv, stats_out);
    }
    return check_launch();
}

}  // namespace klpm
