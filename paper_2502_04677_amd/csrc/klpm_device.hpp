// Device-side layout of the flattened radix tree and helpers shared by the HIP kernels.
//
// The prefix cache of RadixAttention (Sec. 1 of the paper) is kept entirely in HBM as
//   - structure-of-arrays node records (one node = one edge from its parent),
//   - an edge-token pool holding every edge label as a contiguous span,
//   - an open-addressing child table keyed by (parent id, first edge token) whose slots also carry
//     the child's edge span, so that one 32-byte slot read is enough to start comparing tokens.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace klpm {

constexpr int kWave = 64;
constexpr int32_t kRoot = 0;
constexpr int kEvictCand = 2048;  // nodes the last stretch of the eviction cut search sorts in LDS
constexpr uint64_t kEmptyKey = ~0ull;
// A slot whose node was evicted: probes walk past it, inserts may take it over. (No real key has
// parent id -1.)
constexpr uint64_t kTombKey = ~0ull - 1ull;

// Child-table slot. key = (parent id << 32) | first edge token.
struct __attribute__((aligned(32))) Slot {
    uint64_t key;
    int32_t child;
    int32_t edge_len;
    int64_t edge_off;
    int64_t pad;
};
static_assert(sizeof(Slot) == 32, "slot must be 32 bytes");

// Counters and per-call scalars, at the start of the arena.
struct DevState {
    int64_t total_tokens;  // tokens held by live nodes
    uint64_t clock;        // logical LRU clock: prompts admitted so far
    int64_t pool_top;      // absolute pool index of the next free token in the active half
    int32_t n_nodes;       // live non-root nodes
    int32_t n_slots;       // node ids in [0, n_slots) have been handed out at some time
    int32_t free_cnt;      // entries on the free-id stack
    int32_t active_half;   // which half of the pool holds the live spans
    uint32_t device_error; // sticky KLPM_DEV_* bits
    // ---- scalars of the commit in flight ----
    int32_t nb;            // admitted prompts in this commit
    int32_t skip;          // 1 = this commit is abandoned (error), later kernels do nothing
    int32_t pad2;
    int32_t free_cnt0;     // free_cnt / n_slots / pool_top / clock at the start of the structure pass
    int32_t n_slots0;
    int32_t need_compact;
    int32_t need_rebuild;
    int32_t do_evict;
    int32_t pad0;
    int64_t pool_top0;
    uint64_t clock0;
    int64_t tail_total;    // tokens of all unmatched tails of the batch
    int64_t compact_cursor;
    int64_t need_evict;    // tokens that must go
    int64_t inserted_tokens;
    int64_t evicted_tokens;
    int32_t new_nodes;
    int32_t evicted_nodes;
    int32_t done[12];      // workgroups finished, per fused kernel of the commit (4.. = eviction passes)
    int32_t tombstones;    // nodes evicted since the last child-table rebuild (upper bound of the tombstones)
    int32_t pad1;
    uint64_t evict_prefix; // digits of the eviction cut key fixed so far
    int64_t evict_rem;     // tokens still to free among the keys that share that prefix
    uint64_t keep_from;    // nodes with tick >= this belong to prompts in flight and are not evicted
    int32_t evict_all;     // the nodes that may go do not free enough: all of them go
    int32_t cand_cnt;      // nodes collected for the last stretch of the cut search
};

// Everything a kernel needs to walk or edit the tree; passed by value.
struct TreeView {
    DevState *st;
    int32_t *parent;
    int64_t *edge_off;   // absolute index into pool
    int32_t *edge_len;   // 0 = dead slot (root is id 0 with length 0)
    int32_t *depth_end;  // tokens from the root to the end of this node's edge
    uint64_t *tick;      // last-use tick
    int32_t *slot_of;    // index of the child-table slot that leads to this node
    int32_t *free_stack;
    Slot *slots;
    uint32_t slot_mask;  // number of slots - 1 (power of two)
    int32_t max_nodes;
    int32_t *pool;       // 2 * pool_half tokens
    int64_t pool_half;
    int32_t max_prompt_len;
    int32_t max_batch;
};

// Per-commit device workspace (inside the arena).
struct CommitWs {
    int32_t *bm_len;    // [max_batch] match length of admitted prompt j against the pre-commit tree
    int32_t *bm_node;   // [max_batch] node where that match stopped
    int64_t *tail_off;  // [max_batch] offset of prompt j's unmatched tail inside this commit's pool block
    uint64_t *gkey;     // [max_batch] key of the group of prompts that may touch the same new structure
    int32_t *end_node;  // [max_batch] node at which prompt j ends after insertion
    int32_t *used;      // [max_batch] bit 0: prompt j used its reserved split id, bit 1: its reserved leaf id
    int32_t *leaf_tok;  // [max_batch] tokens of the leaf prompt j added (0 if none)
    int32_t *next_tok;  // [max_batch] first unmatched token of prompt j (-1: matched in full)
    int32_t *lcp_lead;  // [max_batch] tokens that prompt j's unmatched tail shares with the tail of its group's first prompt
    int32_t *lcp_tok;   // [max_batch] prompt j's token behind that shared span (-1: the prompt ends there)
    int64_t *p_off;     // [max_batch] plan: where prompt j starts in the queue's token array
    int32_t *p_len;     // [max_batch] plan: prompt j's length
    int32_t *p_de;      // [max_batch] plan: depth at which prompt j's stop node ends
    int32_t *resv_id;   // [2*max_batch] scratch: the node ids reserved for this commit
    int64_t *evict_hist; // [6][2048] weighted digit histograms of the eviction cut search
    uint64_t *cand_key;  // [kEvictCand] eviction keys of the nodes collected for the last stretch of the search
    int32_t *cand_len;   // [kEvictCand] their edge lengths
    int32_t *cand_id;    // [kEvictCand] their node ids
    int32_t *cand_slot;  // [kEvictCand] their child-table slots
    int32_t *iota_idx;  // [max_batch] scratch batch indices for build_tree
    int32_t *iota_n;    // [1]
};

struct QView {
    const int32_t *tokens;
    const int64_t *off;
    const int32_t *len;
    int64_t n_tokens;
    int32_t n;
    const int32_t *n_live;  // device-side count (may be null): only the first min(n, *n_live) queries exist
};

__device__ __forceinline__ uint64_t make_key(int32_t parent, int32_t tok) {
    return ((uint64_t)(uint32_t)parent << 32) | (uint64_t)(uint32_t)tok;
}

__device__ __forceinline__ uint32_t hash_key(uint64_t k) {
    // 64-bit finaliser of the public-domain MurmurHash3
    k ^= k >> 33;
    k *= 0xff51afd7ed558ccdULL;
    k ^= k >> 33;
    k *= 0xc4ceb9fe1a85ec53ULL;
    k ^= k >> 33;
    return (uint32_t)k;
}

// Wave-uniform value: tells the compiler the value is the same in every lane (keeps it in an SGPR).
__device__ __forceinline__ int32_t uni(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int64_t uni64(int64_t v) {
    uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(uint32_t)(uint64_t)v);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Number of entries that exist: the host-side count, cut down by the device-side count if one is given.
__device__ __forceinline__ int32_t live_count(int32_t n, const int32_t *__restrict__ n_live) {
    if (!n_live) return n;
    int32_t v = *n_live;
    v = v < 0 ? 0 : v;
    return v < n ? v : n;
}

// k of Algorithm 1: the host's value, or the one that device memory holds when the launch runs
// (a k that an earlier kernel of the stream chose).
struct KArg {
    uint32_t k;
    const uint32_t *dev;
    __device__ __forceinline__ uint32_t get() const { return dev ? *dev : k; }
};

// Read-only probe (tree not being modified by this kernel). Returns the slot index or -1 and, when
// found, the child's id and edge span. All arguments are wave-uniform; so are the results.
__device__ __forceinline__ int32_t slot_find(const Slot *__restrict__ slots, uint32_t mask, uint64_t key,
                                             int32_t &child, int32_t &edge_len, int64_t &edge_off) {
    uint32_t h = hash_key(key) & mask;
    for (uint32_t probe = 0; probe <= mask; ++probe) {
        const uint4 *p = reinterpret_cast<const uint4 *>(slots + h);
        uint4 lo = p[0];
        uint4 hi = p[1];
        uint32_t k0 = (uint32_t)uni((int32_t)lo.x), k1 = (uint32_t)uni((int32_t)lo.y);
        uint32_t c = (uint32_t)uni((int32_t)lo.z), l = (uint32_t)uni((int32_t)lo.w);
        uint32_t o0 = (uint32_t)uni((int32_t)hi.x), o1 = (uint32_t)uni((int32_t)hi.y);
        // Both halves of the slot are made live here so that they are fetched in one round trip
        // (otherwise the payload read is deferred until after the key compare).
        asm volatile("" : "+s"(k0), "+s"(k1), "+s"(c), "+s"(l), "+s"(o0), "+s"(o1));
        uint64_t k = ((uint64_t)k1 << 32) | (uint64_t)k0;
        if (k == key) {
            child = (int32_t)c;
            edge_len = (int32_t)l;
            edge_off = (int64_t)(((uint64_t)o1 << 32) | (uint64_t)o0);
            return (int32_t)h;
        }
        if (k == kEmptyKey) return -1;
        h = (h + 1) & mask;
    }
    return -1;
}

// First position in [base, base + ROWS*64) at which a[] and b[] differ, or -1. Each lane reads
// single dwords, so neither span needs any alignment. Lanes past `lim` re-read the last valid
// element (no branch around the loads), and no result is looked at before every load of the window
// has been issued: the whole window costs one memory round trip.
template <int ROWS>
__device__ __forceinline__ int32_t window_mismatch(const int32_t *__restrict__ a, const int32_t *__restrict__ b,
                                                   int32_t base, int32_t lim, int lane) {
    int32_t av[ROWS], bv[ROWS];
    const int32_t last = lim - 1;
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        int32_t i = base + r * kWave + lane;
        int32_t ic = i < last ? i : last;
        av[r] = a[ic];
        bv[r] = b[ic];
    }
    int32_t res = -1;
#pragma unroll
    for (int r = ROWS - 1; r >= 0; --r) {
        uint64_t m = __ballot(av[r] != bv[r]);
        if (m) res = base + r * kWave + (int32_t)__builtin_ctzll(m);
    }
    // A clamped lane can only report a difference that the lane owning the last element reports
    // too, from a lower position, so res < lim whenever res >= 0.
    return res;
}

// Number of leading positions (< lim, lim >= 1) where a[] and b[] agree; the whole wavefront
// cooperates. Windows grow from 128 tokens (a mismatch right after a node boundary is the common
// case) to 1024 tokens (16 rows of query and edge tokens = 8 KB per wave in flight) on long edges.
__device__ __forceinline__ int32_t wave_common_prefix(const int32_t *__restrict__ a, const int32_t *__restrict__ b,
                                                      int32_t lim, int lane) {
    int32_t r = window_mismatch<2>(a, b, 0, lim, lane);
    if (r >= 0) return r;
    int32_t base = 2 * kWave;
    while (base < lim) {
        if (lim - base > 4 * kWave) {
            r = window_mismatch<16>(a, b, base, lim, lane);
            if (r >= 0) return r;
            base += 16 * kWave;
        } else {
            r = window_mismatch<4>(a, b, base, lim, lane);
            if (r >= 0) return r;
            base += 4 * kWave;
        }
    }
    return lim;
}

// Inclusive scan across the 64 lanes of a wavefront (no barrier, no LDS).
template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v, int lane) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        T t = __shfl_up(v, d);
        if (lane >= d) v += t;
    }
    return v;
}

// Inclusive scan across a workgroup of THREADS threads with two barriers: lanes scan inside their
// wavefront, the wavefront totals go through `part` (THREADS/64 elements of shared memory).
// `total` receives the sum over the whole workgroup. Every thread must call it.
template <typename T, int THREADS>
__device__ __forceinline__ T block_inclusive_scan(T v, T *part, int tid, T &total) {
    const int lane = tid & (kWave - 1), wv = tid / kWave;
    T incl = wave_inclusive_scan(v, lane);
    __syncthreads();  // `part` may still be read from an earlier call
    if (lane == kWave - 1) part[wv] = incl;
    __syncthreads();
    T before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < THREADS / kWave; ++w) {
        T p = part[w];
        all += p;
        if (w < wv) before += p;
    }
    total = all;
    return incl + before;
}

// How many prompts a commit admits (0 if it must be abandoned, with the reason in *err).
__device__ __forceinline__ int32_t commit_gate(const TreeView &tv, const int32_t *n_selected, int32_t batch_cap,
                                               uint32_t *err) {
    int32_t nb = n_selected ? *n_selected : 0;
    if (nb < 0) nb = 0;
    uint32_t e = 0;
    if (nb > batch_cap || nb > tv.max_batch) e |= 8u;  // KLPM_DEV_BATCH_OVERFLOW
    int64_t free_nodes = (int64_t)(tv.max_nodes - tv.st->n_slots) + (int64_t)tv.st->free_cnt;
    if (!e && 2ll * nb > free_nodes) e |= 1u;          // KLPM_DEV_NODES_FULL: a prompt adds at most two nodes
    *err = e;
    return e ? 0 : nb;
}

}  // namespace klpm
