// Arena layout, tree construction, the match/commit entry points, the canonical snapshot and the
// waiting-queue bookkeeping of an online run.
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "klpm_internal.hpp"
#include "wave_ops.hpp"

namespace klpm {

struct Layout {
    size_t state, parent, edge_off, edge_len, depth_end, tick, slot_of, free_stack, slots, pool;
    size_t bm_len, bm_node, tail_off, gkey, end_node, used, leaf_tok, next_tok, lcp_lead, lcp_tok, p_off, p_len, p_de, resv_id, evict_hist, cand_key, cand_len, cand_id, cand_slot, iota_idx, iota_n;
    size_t total;
    uint32_t n_slots_table;
};

static bool config_ok(const kLPM_config *c) {
    return c && c->budget_tokens >= 0 && c->pool_tokens > 0 && c->max_nodes >= 2 && c->max_nodes <= (1 << 30) &&
           c->max_batch >= 1 && c->max_batch <= 65536 && c->max_prompt_len >= 1 && c->max_prompt_len <= (1 << 28) &&
           c->pool_tokens <= (int64_t)1 << 40;
}

static Layout make_layout(const kLPM_config &c) {
    Layout L;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes, 256); return at; };
    uint32_t ns = 64;
    while (ns < 2u * (uint32_t)c.max_nodes) ns <<= 1;
    L.n_slots_table = ns;
    size_t mn = (size_t)c.max_nodes, mb = (size_t)c.max_batch;
    L.state = take(sizeof(DevState));
    L.parent = take(mn * 4);
    L.edge_off = take(mn * 8);
    L.edge_len = take(mn * 4);
    L.depth_end = take(mn * 4);
    L.tick = take(mn * 8);
    L.slot_of = take(mn * 4);
    L.free_stack = take(mn * 4);
    L.slots = take((size_t)ns * sizeof(Slot));
    L.pool = take((size_t)c.pool_tokens * 2 * 4);
    L.bm_len = take(mb * 4);
    L.bm_node = take(mb * 4);
    L.tail_off = take(mb * 8);
    L.gkey = take(mb * 8);
    L.end_node = take(mb * 4);
    L.used = take(mb * 4);
    L.leaf_tok = take(mb * 4);
    L.next_tok = take(mb * 4);
    L.lcp_lead = take(mb * 4);
    L.lcp_tok = take(mb * 4);
    L.p_off = take(mb * 8);
    L.p_len = take(mb * 4);
    L.p_de = take(mb * 4);
    L.resv_id = take(mb * 8);
    L.evict_hist = take(6 * 2048 * 8);  // eviction cut search: 6 passes of 2048 weighted bins
    L.cand_key = take((size_t)kEvictCand * 8);
    L.cand_len = take((size_t)kEvictCand * 4);
    L.cand_id = take((size_t)kEvictCand * 4);
    L.cand_slot = take((size_t)kEvictCand * 4);
    L.iota_idx = take(mb * 4);
    L.iota_n = take(256);
    L.total = o;
    return L;
}

__global__ __launch_bounds__(256) void k_tree_init(TreeView tv) {
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t ns = (int64_t)tv.slot_mask + 1;
    for (int64_t i = gid; i < ns; i += stride) {
        tv.slots[i].key = kEmptyKey;
        tv.slots[i].child = -1;
        tv.slots[i].edge_len = 0;
        tv.slots[i].edge_off = 0;
        tv.slots[i].pad = 0;
    }
    for (int64_t i = gid; i < tv.max_nodes; i += stride) {
        tv.parent[i] = -1;
        tv.edge_off[i] = 0;
        tv.edge_len[i] = 0;
        tv.depth_end[i] = 0;
        tv.tick[i] = 0;
        tv.slot_of[i] = -1;
        tv.free_stack[i] = 0;
    }
    if (gid == 0) {
        DevState *st = tv.st;
        char *p = (char *)st;
        for (size_t b = 0; b < sizeof(DevState); ++b) p[b] = 0;
        st->n_slots = 1;  // id 0 is the root
    }
}

__global__ __launch_bounds__(256) void k_iota(int32_t *__restrict__ idx, int32_t *__restrict__ n_out, int32_t base,
                                              int32_t count) {
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) idx[i] = base + i;
    if (i == 0) *n_out = count;
}

// ---- waiting-queue bookkeeping of an online run ----
// One launch: every workgroup owns a stretch of queue positions.  It reads the whole batch (a few KB)
// to learn which of its own positions retire, how many retire before its stretch, and what the batch
// costs; with that each surviving entry knows where it moves (down by the retired positions before
// it), retired entries get their TTFT, and the arrivals are appended behind the survivors together
// with the CSR view of the new queue.  Everything is read from the current buffer set (entries,
// count, clock, arrival cursor) and written to the other one, so workgroups never wait for each other.
constexpr int kQaThreads = 512;

struct QueueView {
    int32_t *id;
    uint64_t *arrival;
    int64_t *off;
    int32_t *len;
    int32_t *n;
    uint64_t *clock;
    int32_t *n_joined;
    int32_t cap;
};

struct ArrivalsView {  // arrivals in time order; `time` is null for the per-step lists of kLPM_queue_advance
    const int32_t *id;
    const uint64_t *time;
    int32_t n;
    uint32_t c_num, c_den;
};

// TIMED: Def. 2's timeline (cost with the attention term, arrivals join when their time has come,
// an idle scheduler waits for the next arrival); otherwise the n_new arrivals of this step join at
// the new time and the clock moves by at least 1.
template <bool TIMED>
__global__ __launch_bounds__(kQaThreads) void k_queue_advance(QueueView cur, QueueView next, QView all,
                                                              const int32_t *__restrict__ match_len,
                                                              const int32_t *__restrict__ batch_idx,
                                                              const int32_t *__restrict__ n_selected,
                                                              int32_t batch_cap, ArrivalsView pend,
                                                              int64_t *__restrict__ ttft,
                                                              int64_t *__restrict__ matched_accum,
                                                              uint32_t *__restrict__ dev_error) {
    __shared__ uint32_t bm[kQaThreads / 32];  // retired positions of this workgroup's stretch
    __shared__ unsigned long long s_cost, s_sum;
    __shared__ int32_t s_below, s_valid;
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * kQaThreads;
    // What can be requested without knowing the counts goes out with them: this thread's queue entry
    // (the buffers hold cap entries) and its first two batch entries (batch_cap of them exist).
    constexpr int kAhead = 2;
    const int64_t i = base + tid;
    const bool i_in = i < cur.cap;
    const int32_t my_id = i_in ? cur.id[i] : -1;
    const uint64_t my_arr = i_in ? cur.arrival[i] : 0;
    const int64_t my_off = i_in ? cur.off[i] : 0;
    const int32_t my_len = i_in ? cur.len[i] : 0;
    int32_t w_ahead[kAhead];
#pragma unroll
    for (int t = 0; t < kAhead; ++t) {
        const int32_t j = tid + t * kQaThreads;
        w_ahead[t] = j < batch_cap ? batch_idx[j] : -1;
    }
    int32_t nw = *cur.n;
    nw = nw < 0 ? 0 : (nw > cur.cap ? cur.cap : nw);
    int32_t nb = *n_selected;
    nb = nb < 0 ? 0 : (nb > batch_cap ? batch_cap : nb);
    const uint64_t clock = *cur.clock;
    if (tid < kQaThreads / 32) bm[tid] = 0u;
    if (tid == 0) { s_cost = 0; s_sum = 0; s_below = 0; s_valid = 0; }
    __syncthreads();
    {
        unsigned long long my_cost = 0;
        int32_t below = 0, valid = 0;
        auto retire = [&](int32_t w, int32_t len, int32_t m) {
            ++valid;
            if (w < base) ++below;
            else if (w < base + kQaThreads) atomicOr(&bm[(w - base) >> 5], 1u << ((w - base) & 31));
            m = m < 0 ? 0 : m;
            // (1 + c_attn |x|)(|x| - overlap) token times, in units of 1/c_den (Def. 2); c_attn = 0 otherwise
            if (len > m)
                my_cost += (unsigned long long)(len - m) *
                           (TIMED ? (unsigned long long)pend.c_den + (unsigned long long)pend.c_num * (unsigned long long)len
                                  : 1ull);
        };
        // the entries read ahead: their lengths and matches in one round trip
        int32_t len_a[kAhead], m_a[kAhead];
        bool ok_a[kAhead];
#pragma unroll
        for (int t = 0; t < kAhead; ++t) {
            const int32_t w = w_ahead[t];
            ok_a[t] = tid + t * kQaThreads < nb && w >= 0 && w < nw;
            len_a[t] = ok_a[t] ? cur.len[w] : 0;  // (the queue carries the CSR view of its prompts)
            m_a[t] = ok_a[t] ? match_len[w] : 0;
        }
#pragma unroll
        for (int t = 0; t < kAhead; ++t)
            if (ok_a[t]) retire(w_ahead[t], len_a[t], m_a[t]);
        for (int32_t j = tid + kAhead * kQaThreads; j < nb; j += kQaThreads) {
            const int32_t w = batch_idx[j];
            if (w < 0 || w >= nw) continue;
            retire(w, cur.len[w], match_len[w]);
        }
        my_cost = wave_sum(my_cost);
        below = wave_sum(below);
        valid = wave_sum(valid);
        if ((tid & (kWave - 1)) == 0) {
            if (my_cost) atomicAdd(&s_cost, my_cost);
            if (below) atomicAdd(&s_below, below);
            if (valid) atomicAdd(&s_valid, valid);
        }
    }
    __syncthreads();
    // the whole batch finishes together (Sec. 2.1)
    const uint64_t now = clock + ((TIMED || s_cost > 0) ? (uint64_t)s_cost : 1ull);
    const int32_t kept_all = nw - s_valid;
    const int32_t kept = kept_all < next.cap ? kept_all : next.cap;
    int32_t room = next.cap - kept;
    room = room < 0 ? 0 : room;
    uint64_t now_out = now;
    int32_t first = 0, add = pend.n;
    if (TIMED) {
        // pending arrivals whose time has come: times are sorted, so their number is a prefix length
        first = *cur.n_joined;
        first = first < 0 ? 0 : (first > pend.n ? pend.n : first);
        add = 0;
        for (int pass = 0; pass < 2; ++pass) {
            for (int32_t b = first; b < pend.n; b += kQaThreads) {
                const int32_t i = b + tid;
                const int c = __syncthreads_count(i < pend.n && pend.time[i] <= now_out);
                add += c;
                if (c < kQaThreads) break;
            }
            if (pass == 1 || kept_all > 0 || add > 0 || first >= pend.n) break;
            now_out = pend.time[first];  // nobody waiting: idle until the next arrival (Def. 2: max(R, t))
        }
    }
    const bool overflow = !TIMED && (add > room || kept_all > next.cap);
    add = add < room ? add : room;  // (timed: the rest stay pending, in order)
    unsigned long long my = 0;
    if (i < nw) {
        const int32_t m = match_len[i];
        if (m > 0) my = (unsigned long long)m;
        const uint32_t word = bm[tid >> 5], bit = 1u << (tid & 31);
        int32_t before = s_below + (int32_t)__popc(word & (bit - 1u));
        for (int wd = 0; wd < (tid >> 5); ++wd) before += (int32_t)__popc(bm[wd]);
        const int32_t id = my_id;
        if (word & bit) {
            if (id >= 0 && id < all.n) ttft[id] = (int64_t)(now - my_arr);  // TTFT = finish time - arrival
        } else {
            const int64_t dst = i - before;
            if (dst >= 0 && dst < kept) {
                next.id[dst] = id;
                next.arrival[dst] = my_arr;
                next.off[dst] = my_off;
                next.len[dst] = my_len;
            }
        }
    } else if (i < (int64_t)nw + add) {
        const int32_t r = (int32_t)(i - nw);
        const int32_t id = pend.id[first + r];
        const int64_t dst = (int64_t)kept + r;
        next.id[dst] = id;
        // a timed arrival keeps its own time; otherwise it is enqueued when the previous batch finished
        next.arrival[dst] = TIMED ? pend.time[first + r] : now;
        const bool ok = id >= 0 && id < all.n;
        next.off[dst] = ok ? all.off[id] : -1;
        next.len[dst] = ok ? all.len[id] : 0;
    }
    if (blockIdx.x == 0 && tid == 0) {
        if (overflow && dev_error) atomicOr(dev_error, 8u);
        *next.n = kept + add;
        *next.clock = now_out;
        if (next.n_joined) *next.n_joined = first + add;
    }
    if (matched_accum) {
        my = wave_sum(my);
        if ((tid & (kWave - 1)) == 0 && my) atomicAdd(&s_sum, my);
        __syncthreads();
        if (tid == 0 && s_sum) atomicAdd((unsigned long long *)matched_accum, s_sum);
    }
}

__global__ __launch_bounds__(256) void k_queue_gather(QueueView q, QView all) {
    int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    int32_t nw = *q.n;
    if (nw > q.cap) nw = q.cap;
    if (i >= nw) return;
    int32_t id = q.id[i];
    bool ok = id >= 0 && id < all.n;
    q.off[i] = ok ? all.off[id] : -1;  // an invalid id fails the bounds check of the match kernel
    q.len[i] = ok ? all.len[id] : 0;
}

static QView make_qview(const kLPM_queries *q) {
    QView v;
    v.tokens = q->tokens;
    v.off = q->off;
    v.len = q->len;
    v.n_tokens = q->n_tokens;
    v.n = q->n;
    v.n_live = q->n_live;
    return v;
}

static bool queries_ok(const kLPM_queries *q) {
    if (!q || q->n < 0 || q->n_tokens < 0) return false;
    if (q->n > 0 && (!q->tokens || !q->off || !q->len)) return false;
    return true;
}

}  // namespace klpm

using namespace klpm;

extern "C" int kLPM_arena_bytes(const kLPM_config *cfg, size_t *out_bytes) {
    if (!config_ok(cfg) || !out_bytes) return KLPM_EINVAL;
    *out_bytes = make_layout(*cfg).total;
    return KLPM_OK;
}

extern "C" int kLPM_build_tree(kLPM_tree **out, const kLPM_config *cfg, void *arena, size_t arena_bytes,
                               const kLPM_queries *initial, kLPM_stream stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!out || !config_ok(cfg) || !arena) return KLPM_EINVAL;
    if (initial && !queries_ok(initial)) return KLPM_EINVAL;
    Layout L = make_layout(*cfg);
    if (arena_bytes < L.total || ((uintptr_t)arena & 255u)) return KLPM_EARENA;
    kLPM_tree *t = new (std::nothrow) kLPM_tree();
    if (!t) return KLPM_ENOMEM;
    char *base = (char *)arena;
    t->cfg = *cfg;
    t->arena = arena;
    t->arena_bytes = arena_bytes;
    t->budget = cfg->budget_tokens;
    t->protect = 0;
    t->clock_ub = 0;
    t->clock_reserve = 0;
    t->depth_bits = 1;
    while ((cfg->max_prompt_len >> t->depth_bits) != 0) ++t->depth_bits;
    TreeView &tv = t->tv;
    tv.st = (DevState *)(base + L.state);
    tv.parent = (int32_t *)(base + L.parent);
    tv.edge_off = (int64_t *)(base + L.edge_off);
    tv.edge_len = (int32_t *)(base + L.edge_len);
    tv.depth_end = (int32_t *)(base + L.depth_end);
    tv.tick = (uint64_t *)(base + L.tick);
    tv.slot_of = (int32_t *)(base + L.slot_of);
    tv.free_stack = (int32_t *)(base + L.free_stack);
    tv.slots = (Slot *)(base + L.slots);
    tv.slot_mask = L.n_slots_table - 1;
    tv.max_nodes = cfg->max_nodes;
    tv.pool = (int32_t *)(base + L.pool);
    tv.pool_half = cfg->pool_tokens;
    tv.max_prompt_len = cfg->max_prompt_len;
    tv.max_batch = cfg->max_batch;
    CommitWs &ws = t->ws;
    ws.bm_len = (int32_t *)(base + L.bm_len);
    ws.bm_node = (int32_t *)(base + L.bm_node);
    ws.tail_off = (int64_t *)(base + L.tail_off);
    ws.gkey = (uint64_t *)(base + L.gkey);
    ws.end_node = (int32_t *)(base + L.end_node);
    ws.used = (int32_t *)(base + L.used);
    ws.leaf_tok = (int32_t *)(base + L.leaf_tok);
    ws.next_tok = (int32_t *)(base + L.next_tok);
    ws.lcp_lead = (int32_t *)(base + L.lcp_lead);
    ws.lcp_tok = (int32_t *)(base + L.lcp_tok);
    ws.p_off = (int64_t *)(base + L.p_off);
    ws.p_len = (int32_t *)(base + L.p_len);
    ws.p_de = (int32_t *)(base + L.p_de);
    ws.resv_id = (int32_t *)(base + L.resv_id);
    ws.evict_hist = (int64_t *)(base + L.evict_hist);
    ws.cand_key = (uint64_t *)(base + L.cand_key);
    ws.cand_len = (int32_t *)(base + L.cand_len);
    ws.cand_id = (int32_t *)(base + L.cand_id);
    ws.cand_slot = (int32_t *)(base + L.cand_slot);
    ws.iota_idx = (int32_t *)(base + L.iota_idx);
    ws.iota_n = (int32_t *)(base + L.iota_n);

    hipLaunchKernelGGL(k_tree_init, dim3(2048), dim3(256), 0, stream, tv);
    int rc = check_launch();
    if (rc == KLPM_OK && initial && initial->n > 0) {
        QView q = make_qview(initial);
        for (int32_t base_i = 0; base_i < initial->n && rc == KLPM_OK; base_i += cfg->max_batch) {
            int32_t cnt = std::min(cfg->max_batch, initial->n - base_i);
            hipLaunchKernelGGL(k_iota, dim3((cnt + 255) / 256), dim3(256), 0, stream, ws.iota_idx, ws.iota_n, base_i,
                               cnt);
            rc = commit_pipeline(t, q, ws.iota_idx, ws.iota_n, cnt, INT64_MAX, 0, nullptr, stream);
        }
    }
    if (rc != KLPM_OK) {
        delete t;
        return rc;
    }
    *out = t;
    return KLPM_OK;
}

extern "C" int kLPM_match(kLPM_tree *tree, const kLPM_queries *q, int32_t *match_len, int32_t *last_node,
                          kLPM_stream stream_) {
    if (!tree || !queries_ok(q)) return KLPM_EINVAL;
    if (q->n == 0) return KLPM_OK;
    if (!match_len) return KLPM_EINVAL;
    return launch_match(tree->tv, make_qview(q), nullptr, nullptr, q->n, 0, match_len, last_node,
                        (hipStream_t)stream_);
}

extern "C" int kLPM_commit(kLPM_tree *tree, const kLPM_queries *q, const int32_t *batch_idx,
                           const int32_t *n_selected, int32_t batch_cap, kLPM_stats *stats, kLPM_stream stream_) {
    if (!tree || !queries_ok(q) || batch_cap < 0) return KLPM_EINVAL;
    if (batch_cap > 0 && (!batch_idx || !n_selected)) return KLPM_EINVAL;
    if (batch_cap > tree->cfg.max_batch) return KLPM_EINVAL;
    return commit_pipeline(tree, make_qview(q), batch_idx, n_selected, batch_cap, tree->budget, tree->protect, stats,
                           (hipStream_t)stream_);
}

extern "C" int kLPM_commit_matched(kLPM_tree *tree, const kLPM_queries *q, const int32_t *match_len,
                                   const int32_t *last_node, const int32_t *batch_idx, const int32_t *n_selected,
                                   int32_t batch_cap, kLPM_stats *stats, kLPM_stream stream_) {
    if (!tree || !queries_ok(q) || batch_cap < 0 || !match_len || !last_node) return KLPM_EINVAL;
    if (batch_cap > 0 && (!batch_idx || !n_selected)) return KLPM_EINVAL;
    if (batch_cap > tree->cfg.max_batch) return KLPM_EINVAL;
    return commit_pipeline(tree, make_qview(q), batch_idx, n_selected, batch_cap, tree->budget, tree->protect, stats,
                           (hipStream_t)stream_, match_len, last_node);
}

extern "C" int kLPM_reserve_clock(kLPM_tree *tree, uint64_t extra_prompts) {
    if (!tree) return KLPM_EINVAL;
    tree->clock_reserve = extra_prompts;
    return KLPM_OK;
}

extern "C" int kLPM_set_protect(kLPM_tree *tree, int64_t recent_prompts) {
    if (!tree || recent_prompts < 0) return KLPM_EINVAL;
    tree->protect = recent_prompts;
    return KLPM_OK;
}

extern "C" int kLPM_set_budget(kLPM_tree *tree, int64_t budget_tokens) {
    if (!tree || budget_tokens < 0) return KLPM_EINVAL;
    tree->budget = budget_tokens;
    return KLPM_OK;
}

static bool queue_ok(const kLPM_queue *q) {
    return q && q->cap >= 0 && q->n && q->clock && (q->cap == 0 || (q->id && q->arrival && q->off && q->len));
}

static QueueView make_queue_view(const kLPM_queue *q) {
    QueueView v;
    v.id = q->id; v.arrival = q->arrival; v.off = q->off; v.len = q->len; v.n = q->n; v.clock = q->clock;
    v.n_joined = q->n_joined; v.cap = q->cap;
    return v;
}

static int queue_advance_impl(bool timed, const kLPM_queue *cur, const kLPM_queue *next, const kLPM_queries *all,
                              const int32_t *match_len, const int32_t *batch_idx, const int32_t *n_selected,
                              int32_t batch_cap, const ArrivalsView &pend, int64_t *ttft, int64_t *matched_accum,
                              uint32_t *dev_error, hipStream_t stream) {
    if (!queue_ok(cur) || !queue_ok(next) || !queries_ok(all) || batch_cap < 0 || pend.n < 0 || !ttft || !n_selected)
        return KLPM_EINVAL;
    if (cur->id == next->id || cur->arrival == next->arrival || cur->n == next->n || cur->clock == next->clock)
        return KLPM_EINVAL;
    if (timed && (!cur->n_joined || !next->n_joined || cur->n_joined == next->n_joined)) return KLPM_EINVAL;
    if ((batch_cap > 0 && (!batch_idx || !match_len)) || (pend.n > 0 && !pend.id)) return KLPM_EINVAL;
    QueueView c = make_queue_view(cur), n = make_queue_view(next);
    QView a = make_qview(all);
    // survivors come from at most cur->cap positions; how many arrivals join is decided on the device
    // in the timed case (at most next->cap of them)
    const int64_t work = (int64_t)cur->cap + (timed ? (int64_t)(pend.n < next->cap ? pend.n : next->cap) : (int64_t)pend.n);
    const unsigned blocks = (unsigned)((work + kQaThreads - 1) / kQaThreads);
    if (timed)
        hipLaunchKernelGGL(k_queue_advance<true>, dim3(blocks ? blocks : 1), dim3(kQaThreads), 0, stream, c, n, a, match_len,
                           batch_idx, n_selected, batch_cap, pend, ttft, matched_accum, dev_error);
    else
        hipLaunchKernelGGL(k_queue_advance<false>, dim3(blocks ? blocks : 1), dim3(kQaThreads), 0, stream, c, n, a, match_len,
                           batch_idx, n_selected, batch_cap, pend, ttft, matched_accum, dev_error);
    return check_launch();
}

extern "C" int kLPM_queue_advance(const kLPM_queue *cur, const kLPM_queue *next, const kLPM_queries *all,
                                  const int32_t *match_len, const int32_t *batch_idx, const int32_t *n_selected,
                                  int32_t batch_cap, const int32_t *new_id, int32_t n_new, int64_t *ttft,
                                  int64_t *matched_accum, uint32_t *dev_error, kLPM_stream stream_) {
    ArrivalsView pend{new_id, nullptr, n_new, 0u, 1u};
    return queue_advance_impl(false, cur, next, all, match_len, batch_idx, n_selected, batch_cap, pend, ttft, matched_accum,
                              dev_error, (hipStream_t)stream_);
}

extern "C" int kLPM_queue_advance_timed(const kLPM_queue *cur, const kLPM_queue *next, const kLPM_queries *all,
                                        const int32_t *match_len, const int32_t *batch_idx,
                                        const int32_t *n_selected, int32_t batch_cap, const kLPM_arrivals *pending,
                                        int64_t *ttft, int64_t *matched_accum, uint32_t *dev_error,
                                        kLPM_stream stream_) {
    if (!pending || pending->n < 0 || pending->c_den < 1u) return KLPM_EINVAL;
    if (pending->n > 0 && (!pending->id || !pending->time)) return KLPM_EINVAL;
    ArrivalsView pend{pending->id, pending->time, pending->n, pending->c_num, pending->c_den};
    return queue_advance_impl(true, cur, next, all, match_len, batch_idx, n_selected, batch_cap, pend, ttft, matched_accum,
                              dev_error, (hipStream_t)stream_);
}

extern "C" int kLPM_queue_gather(const kLPM_queue *q, const kLPM_queries *all, kLPM_stream stream_) {
    if (!queue_ok(q) || !queries_ok(all)) return KLPM_EINVAL;
    if (q->cap == 0) return KLPM_OK;
    hipLaunchKernelGGL(k_queue_gather, dim3((q->cap + 255) / 256), dim3(256), 0, (hipStream_t)stream_,
                       make_queue_view(q), make_qview(all));
    return check_launch();
}

extern "C" int kLPM_read_stats(kLPM_tree *tree, kLPM_stats *host_out, kLPM_stream stream_) {
    if (!tree || !host_out) return KLPM_EINVAL;
    if (hipStreamSynchronize((hipStream_t)stream_) != hipSuccess) return KLPM_EHIP;
    DevState st;
    if (hipMemcpy(&st, tree->tv.st, sizeof(st), hipMemcpyDeviceToHost) != hipSuccess) return KLPM_EHIP;
    std::memset(host_out, 0, sizeof(*host_out));
    host_out->total_tokens = st.total_tokens;
    host_out->n_nodes = st.n_nodes;
    host_out->device_error = st.device_error;
    host_out->clock = st.clock;
    if (st.clock > tree->clock_ub) tree->clock_ub = st.clock;  // admissions enqueued by graph replays
    return KLPM_OK;
}

// ---- canonical snapshot (host side; plumbing, not part of the scheduling step) ----
namespace {
struct SnapRec {
    int32_t depth_start, edge_len;
    uint64_t tick;
    int32_t n_children, pad;
};

struct HostTree {
    DevState st;
    std::vector<int32_t> parent, edge_len, depth_end;
    std::vector<int64_t> edge_off;
    std::vector<uint64_t> tick;
};

int download(kLPM_tree *t, HostTree &h, hipStream_t stream) {
    if (hipStreamSynchronize(stream) != hipSuccess) return KLPM_EHIP;
    if (hipMemcpy(&h.st, t->tv.st, sizeof(DevState), hipMemcpyDeviceToHost) != hipSuccess) return KLPM_EHIP;
    size_t n = (size_t)h.st.n_slots;
    if (n > (size_t)t->cfg.max_nodes) return KLPM_EHIP;
    h.parent.resize(n); h.edge_len.resize(n); h.depth_end.resize(n); h.edge_off.resize(n); h.tick.resize(n);
    if (hipMemcpy(h.parent.data(), t->tv.parent, n * 4, hipMemcpyDeviceToHost) != hipSuccess) return KLPM_EHIP;
    if (hipMemcpy(h.edge_len.data(), t->tv.edge_len, n * 4, hipMemcpyDeviceToHost) != hipSuccess) return KLPM_EHIP;
    if (hipMemcpy(h.depth_end.data(), t->tv.depth_end, n * 4, hipMemcpyDeviceToHost) != hipSuccess) return KLPM_EHIP;
    if (hipMemcpy(h.edge_off.data(), t->tv.edge_off, n * 8, hipMemcpyDeviceToHost) != hipSuccess) return KLPM_EHIP;
    if (hipMemcpy(h.tick.data(), t->tv.tick, n * 8, hipMemcpyDeviceToHost) != hipSuccess) return KLPM_EHIP;
    return KLPM_OK;
}
}  // namespace

extern "C" int kLPM_snapshot_bytes(kLPM_tree *tree, size_t *out_bytes, kLPM_stream stream_) {
    if (!tree || !out_bytes) return KLPM_EINVAL;
    if (hipStreamSynchronize((hipStream_t)stream_) != hipSuccess) return KLPM_EHIP;
    DevState st;
    if (hipMemcpy(&st, tree->tv.st, sizeof(st), hipMemcpyDeviceToHost) != hipSuccess) return KLPM_EHIP;
    *out_bytes = 24 + (size_t)st.n_nodes * sizeof(SnapRec) + (size_t)st.total_tokens * 4;
    return KLPM_OK;
}

extern "C" int kLPM_snapshot(kLPM_tree *tree, void *host_buf, size_t cap, size_t *out_bytes, kLPM_stream stream_) {
    if (!tree || !host_buf || !out_bytes) return KLPM_EINVAL;
    HostTree h;
    int rc = download(tree, h, (hipStream_t)stream_);
    if (rc) return rc;
    const size_t n_ids = h.parent.size();
    // live nodes and the span of the pool they use
    int64_t lo = INT64_MAX, hi = 0;
    size_t n_live = 0;
    int64_t tokens = 0;
    for (size_t id = 1; id < n_ids; ++id) {
        if (h.edge_len[id] <= 0) continue;
        ++n_live;
        tokens += h.edge_len[id];
        lo = std::min(lo, h.edge_off[id]);
        hi = std::max(hi, h.edge_off[id] + h.edge_len[id]);
    }
    size_t need = 24 + n_live * sizeof(SnapRec) + (size_t)tokens * 4;
    *out_bytes = need;
    if (cap < need) return KLPM_EARENA;
    std::vector<int32_t> pool;
    if (n_live) {
        if (lo < 0 || hi > 2 * tree->tv.pool_half) return KLPM_EHIP;
        pool.resize((size_t)(hi - lo));
        if (hipMemcpy(pool.data(), tree->tv.pool + lo, (size_t)(hi - lo) * 4, hipMemcpyDeviceToHost) != hipSuccess)
            return KLPM_EHIP;
    }
    // children lists (CSR by parent), each sorted by first edge token
    std::vector<int32_t> deg(n_ids + 1, 0);
    for (size_t id = 1; id < n_ids; ++id)
        if (h.edge_len[id] > 0 && h.parent[id] >= 0 && (size_t)h.parent[id] < n_ids) deg[h.parent[id] + 1]++;
    for (size_t i = 0; i < n_ids; ++i) deg[i + 1] += deg[i];
    std::vector<int32_t> kids((size_t)deg[n_ids]);
    {
        std::vector<int32_t> fill(deg.begin(), deg.end() - 1);
        for (size_t id = 1; id < n_ids; ++id)
            if (h.edge_len[id] > 0 && h.parent[id] >= 0 && (size_t)h.parent[id] < n_ids)
                kids[(size_t)fill[h.parent[id]]++] = (int32_t)id;
    }
    auto first_tok = [&](int32_t id) { return pool[(size_t)(h.edge_off[id] - lo)]; };
    for (size_t p = 0; p < n_ids; ++p)
        std::sort(kids.begin() + deg[p], kids.begin() + deg[p + 1],
                  [&](int32_t a, int32_t b) { return first_tok(a) < first_tok(b); });
    char *out = (char *)host_buf;
    int64_t head[3] = {(int64_t)n_live, tokens, (int64_t)h.st.clock};
    std::memcpy(out, head, 24);
    SnapRec *rec = (SnapRec *)(out + 24);
    int32_t *tok = (int32_t *)(out + 24 + n_live * sizeof(SnapRec));
    // iterative pre-order
    std::vector<int32_t> stack;
    for (int32_t i = deg[1] - 1; i >= deg[0]; --i) stack.push_back(kids[(size_t)i]);
    size_t written = 0;
    while (!stack.empty()) {
        int32_t id = stack.back();
        stack.pop_back();
        if (written >= n_live) return KLPM_EHIP;  // a cycle or a node reachable twice
        SnapRec r;
        r.depth_start = h.depth_end[id] - h.edge_len[id];
        r.edge_len = h.edge_len[id];
        r.tick = h.tick[id];
        r.n_children = deg[(size_t)id + 1] - deg[(size_t)id];
        r.pad = 0;
        rec[written++] = r;
        std::memcpy(tok, pool.data() + (h.edge_off[id] - lo), (size_t)h.edge_len[id] * 4);
        tok += h.edge_len[id];
        for (int32_t i = deg[(size_t)id + 1] - 1; i >= deg[(size_t)id]; --i) stack.push_back(kids[(size_t)i]);
    }
    if (written != n_live) return KLPM_EHIP;  // live nodes not reachable from the root
    return KLPM_OK;
}

extern "C" int kLPM_destroy(kLPM_tree *tree) {
    delete tree;
    return KLPM_OK;
}

extern "C" const char *kLPM_strerror(int code) {
    switch (code) {
        case KLPM_OK: return "ok";
        case KLPM_EINVAL: return "invalid argument";
        case KLPM_EARENA: return "arena or workspace too small or misaligned";
        case KLPM_EHIP: return "HIP runtime error";
        case KLPM_ENOMEM: return "host allocation failed";
        case KLPM_ELIMIT: return "input larger than the fixed maximum of this entry point";
        default: return "unknown error";
    }
}
