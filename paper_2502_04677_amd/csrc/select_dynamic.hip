// k-LPM batch selection with in-batch rescoring (Algorithm 1 applied inside one bin of B queries,
// Sec. 2.1, with the overlap credit of Def. 2 taken against everything processed so far).
//
// After a pick p the score of every remaining query i becomes max(score_i, overlap(x_i, x_p)).  Only
// few queries can gain: overlap(x_i, x_p) exceeds i's match against the cache only if x_p leaves the
// cached tree at the very place x_i does and goes on with the same token, i.e. if both have the same
// (stop node, match length, next token).  Queries are grouped by that key up front (a hash table
// gives every key a slot, a scan and a scatter lay each group's members out next to each other); a
// pick then rescans its own group only, one lane per member, and a query whose group has no other
// member can neither gain nor give.  The picks themselves are made by one wavefront walking
// the oldest-first and longest-match orders: whole k-cycles at a time while no picked query has a
// group, one pick at a time (static head of the longest-match order against the best boosted
// query) otherwise.
#include "klpm_internal.hpp"

namespace klpm {

constexpr int32_t kDynMaxN = 262144;  // two state bits per query are kept in LDS (64 KB)
constexpr int kPairGroup = 8;         // groups of up to this many queries get their pairwise common prefixes before the walk

struct DynWs {
    uint64_t *gk;       // [n] (stop node << 32) | next token
    int32_t *slot_of;   // [n] table slot of the query's group, -1: no group (prompt cached in full, bad input)
    uint8_t *multi;     // [n] 1: the group has at least two members
    int32_t *rep;       // [table] first query that claimed the slot, -1: free
    int32_t *cnt;       // [table] members
    int32_t *start;     // [table] first entry of the group in `members`
    int32_t *fill;      // [table] scratch of the scatter
    int32_t *tile_sum;  // [table / 8192, at least 1] scratch of the scan
    int32_t *members;   // [n] query indices, the members of a group next to each other
    int32_t *gstart;    // [n] where the query's group starts in `members`
    int32_t *gcnt;      // [n] members of the query's group
    uint64_t *bkey;     // [n] boosted set: (inverted score, position in the oldest-first order)
    int32_t *bidx;      // [n] boosted set: query index
    int32_t *bpos;      // [n] where a boosted query sits in the set
    int32_t *bslot;     // [n] boosted set: the query's member record (-1: its group has none)
    int32_t *gslot;     // [n] where the query sits in `members` (-1: no group)
    int4 *mrec;         // [n] member records of the small groups, in `members` order: query, oldest-first rank, current score, place in the boosted set
    int32_t *pair;      // [n][kPairGroup] small groups: common prefix of the member in this place with every member of its group
    uint32_t table_mask;
};

struct LiveQ {
    int32_t n;
    const int32_t *live;
    __device__ __forceinline__ int32_t get() const { return live_count(n, live); }
};

__device__ __forceinline__ uint32_t group_hash(uint64_t gk, int32_t m) {
    return hash_key(gk ^ ((uint64_t)(uint32_t)m * 0x9E3779B97F4A7C15ull));
}

__global__ __launch_bounds__(256) void k_dyn_init(QView q, const int32_t *__restrict__ match_len,
                                                  const int32_t *__restrict__ last_node, DynWs ws,
                                                  int32_t *__restrict__ dyn) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i <= (int64_t)ws.table_mask) {
        ws.rep[i] = -1;
        ws.cnt[i] = 0;
        ws.fill[i] = 0;
    }
    const int32_t n = live_count(q.n, q.n_live);
    if (i >= n) return;
    int32_t m = match_len[i];
    const int64_t off = q.off[i];
    const int32_t len = q.len[i];
    const bool ok = m >= 0 && off >= 0 && len >= 1 && off + (int64_t)len <= q.n_tokens && m <= len;
    dyn[i] = ok ? m : 0;
    ws.multi[i] = 0;
    // a prompt that is cached in full adds nothing to the cache and cannot gain either
    const bool grouped = ok && m < len;
    ws.slot_of[i] = grouped ? 0 : -1;
    ws.gk[i] = grouped ? (((uint64_t)(uint32_t)last_node[i] << 32) | (uint64_t)(uint32_t)q.tokens[off + m]) : 0ull;
}

__global__ __launch_bounds__(256) void k_dyn_insert(LiveQ nn, const int32_t *__restrict__ match_len, DynWs ws) {
    const int32_t n = nn.get();
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n || ws.slot_of[i] < 0) return;
    const uint64_t gk = ws.gk[i];
    const int32_t m = match_len[i];
    uint32_t h = group_hash(gk, m) & ws.table_mask;
    for (uint32_t probe = 0; probe <= ws.table_mask; ++probe) {
        int32_t r = atomicCAS(&ws.rep[h], -1, i);
        if (r == -1 || (ws.gk[r] == gk && match_len[r] == m)) break;  // claimed, or the group's slot
        h = (h + 1u) & ws.table_mask;
    }
    ws.slot_of[i] = (int32_t)h;
    atomicAdd(&ws.cnt[h], 1);
}

// Exclusive scan of the group sizes: where each group's members start in `members`.  Two launches:
// every workgroup sums its stretch of the table (eight slots per thread), then adds up the stretches
// before its own and scans inside it.
constexpr int kDynScanThreads = 1024;
constexpr int kDynScanPer = 8;
constexpr int kDynScanTile = kDynScanThreads * kDynScanPer;

__global__ __launch_bounds__(kDynScanThreads) void k_dyn_tile_sums(DynWs ws) {
    __shared__ int32_t s_sum;
    const int tid = threadIdx.x;
    if (tid == 0) s_sum = 0;
    __syncthreads();
    const int64_t table = (int64_t)ws.table_mask + 1;
    const int64_t base = (int64_t)blockIdx.x * kDynScanTile + (int64_t)tid * kDynScanPer;
    int32_t mine = 0;
#pragma unroll
    for (int u = 0; u < kDynScanPer; ++u) mine += base + u < table ? ws.cnt[base + u] : 0;
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) mine += __shfl_xor(mine, d);
    if ((tid & (kWave - 1)) == 0 && mine) atomicAdd(&s_sum, mine);
    __syncthreads();
    if (tid == 0) ws.tile_sum[blockIdx.x] = s_sum;
}

__global__ __launch_bounds__(kDynScanThreads) void k_dyn_offsets(DynWs ws) {
    __shared__ int32_t part[kDynScanThreads / kWave];
    __shared__ int32_t s_before;
    const int tid = threadIdx.x;
    if (tid == 0) s_before = 0;
    __syncthreads();
    int32_t before = 0;  // members in the tiles before this one (a table has at most 64 tiles)
    for (int32_t b = tid; b < (int32_t)blockIdx.x; b += kDynScanThreads) before += ws.tile_sum[b];
    if (before) atomicAdd(&s_before, before);
    const int64_t table = (int64_t)ws.table_mask + 1;
    const int64_t base = (int64_t)blockIdx.x * kDynScanTile + (int64_t)tid * kDynScanPer;
    int32_t c[kDynScanPer];
    int32_t mine = 0;
#pragma unroll
    for (int u = 0; u < kDynScanPer; ++u) {
        c[u] = base + u < table ? ws.cnt[base + u] : 0;
        mine += c[u];
    }
    int32_t all;
    int32_t run = block_inclusive_scan<int32_t, kDynScanThreads>(mine, part, tid, all) - mine + s_before;
#pragma unroll
    for (int u = 0; u < kDynScanPer; ++u) {
        if (base + u < table) ws.start[base + u] = run;
        run += c[u];
    }
}

__global__ __launch_bounds__(256) void k_dyn_scatter(LiveQ nn, DynWs ws) {
    const int32_t n = nn.get();
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t s = ws.slot_of[i];
    const int32_t gn = s >= 0 ? ws.cnt[s] : 0, g0 = s >= 0 ? ws.start[s] : 0;
    ws.multi[i] = gn > 1 ? 1 : 0;
    ws.gstart[i] = g0;
    ws.gcnt[i] = gn;
    ws.gslot[i] = -1;
    if (s < 0) return;
    const int32_t at = g0 + atomicAdd(&ws.fill[s], 1);
    if (at >= 0 && at < n) {
        ws.members[at] = i;
        ws.gslot[i] = at;
    }
}

// Small groups (2 .. kPairGroup queries): every pair's common prefix, found by the whole GPU before the
// walk (one wavefront per query compares it with the members behind it in its group), and one record per
// member, so that the walk's rescoring of such a group is one read of records and one row of prefixes
// instead of a chain of reads and token compares per pick.
__global__ __launch_bounds__(256) void k_dyn_pairs(QView q, const int32_t *__restrict__ match_len,
                                                   const uint32_t *__restrict__ rank_a, DynWs ws) {
    const int32_t n = live_count(q.n, q.n_live);
    const int lane = threadIdx.x & (kWave - 1);
    const int32_t i = (int32_t)((blockIdx.x * blockDim.x + threadIdx.x) / kWave);
    if (i >= n) return;
    const int32_t s = uni(ws.gslot[i]), g0 = uni(ws.gstart[i]), gn = uni(ws.gcnt[i]);
    if (s < 0 || gn < 2 || gn > kPairGroup) return;
    const int32_t a = s - g0;
    int32_t m = uni(match_len[i]);
    m = m < 0 ? 0 : m;
    const int64_t off_i = uni64(q.off[i]);
    const int32_t len_i = uni(q.len[i]);
    if (lane == 0) ws.mrec[s] = make_int4(i, (int32_t)rank_a[i], m, -1);
    const int32_t s0 = m + 1;  // the group shares the cached part and the next token
    for (int32_t b = a + 1; b < gn; ++b) {
        const int32_t jq = uni(ws.members[g0 + b]);
        const int64_t off_j = uni64(q.off[jq]);
        const int32_t len_j = uni(q.len[jq]);
        const int32_t lim = (len_i < len_j ? len_i : len_j) - s0;
        int32_t lcp = s0;
        if (lim > 0) lcp += wave_common_prefix(q.tokens + off_i + s0, q.tokens + off_j + s0, lim, lane);
        if (lane == 0) {
            ws.pair[(size_t)(g0 + a) * kPairGroup + b] = lcp;
            ws.pair[(size_t)(g0 + b) * kPairGroup + a] = lcp;
        }
    }
}

// loads and stores of the arrays the walking wavefront both writes and reads (one wavefront: nobody else
// looks at them while the kernel runs, so workgroup scope orders all there is to order)
template <typename T>
__device__ __forceinline__ T coh_load(const T *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
template <typename T>
__device__ __forceinline__ void coh_store(T *p, T v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

__device__ __forceinline__ uint64_t pack_key(int32_t score, uint32_t rank_a) {
    return ((uint64_t)(0x7FFFFFFFu - (uint32_t)score) << 32) | (uint64_t)rank_a;
}

__global__ __launch_bounds__(kWave) void k_dyn_walk(QView q, const int32_t *__restrict__ match_len, SelectOrders ord,
                                                    DynWs ws, int32_t *__restrict__ dyn, KArg ka, int32_t batch,
                                                    uint32_t *__restrict__ phase_inout,
                                                    int32_t *__restrict__ batch_idx,
                                                    int32_t *__restrict__ n_selected) {
    const uint32_t k = ka.get();
    __shared__ uint32_t st[kDynMaxN / 16];  // per query: bit 0 = picked, bit 1 = in the boosted set
    const int lane = threadIdx.x;
    const int32_t n = live_count(q.n, q.n_live);
    const int32_t nb = batch < n ? batch : n;
    const bool lpm_only = (k == 0u || k == 0xFFFFFFFFu);
    const uint32_t phase = lpm_only ? 0u : (*phase_inout % k);
    if (ord.violated && *ord.violated) {  // the caller's promise about the queue does not hold: select nothing, say so
        if (lane == 0) *n_selected = -1;
        return;
    }
    for (int32_t w = lane; w < (n + 15) / 16; w += kWave) st[w] = 0u;
    __syncthreads();
    if (lane == 0) {
        *n_selected = nb;
        *phase_inout = lpm_only ? 0u : (uint32_t)(((uint64_t)phase + (uint64_t)nb) % k);
    }
    auto state = [&](uint32_t e) -> uint32_t { return (st[e >> 4] >> ((e & 15u) * 2u)) & 3u; };
    auto set_bits = [&](uint32_t e, uint32_t bits) { atomicOr(&st[e >> 4], bits << ((e & 15u) * 2u)); };
    const uint32_t km1 = k - 1u;
    int32_t ia = 0, il = 0, j = 0, n_boost = 0;
    uint32_t pos = phase;  // (phase + j) mod k
    // best entry of the boosted set (smallest key), kept up to date lazily
    uint64_t kb = ~0ull;
    int32_t pb = -1;
    bool kb_valid = true;
    // Each order is looked at through a window of 64 consecutive entries held in registers (lane = entry;
    // what is read there never changes during the walk: the query, its place in the other order, whether it
    // has a group, its match length); a window is read again once the cursor has moved kReload entries into
    // it.  What does change - picked, boosted - is two bits per query in LDS.  Entries that a cursor has
    // passed are picked (oldest-first order) or picked or boosted (longest-match order), so they drop out
    // as candidates by their bits alone, wherever the window starts.
    constexpr int32_t kReload = 16;
    int32_t wa = -kWave, wl = -kWave;
    bool a_in = false, l_in = false;
    uint32_t a_el = 0, a_other = 0, l_el = 0, l_other = 0;
    int32_t a_multi = 0, l_multi = 0;
    uint64_t l_key = ~0ull;
    bool after_single = false;  // the pick before was made alone: such picks come in runs, and an attempt at whole cycles costs as much as a pick
    while (j < nb) {
        const bool oldest = !lpm_only && pos == 0u;
        if (ia - wa >= kReload || ia < wa) {
            wa = ia;
            a_in = wa + lane < n;
            a_el = 0; a_other = 0; a_multi = 0;
            if (a_in) {
                a_el = ord.order_a[wa + lane];
                a_other = ord.rank_l[a_el];
                a_multi = ws.multi[a_el];
            }
        }
        if (il - wl >= kReload || il < wl) {
            wl = il;
            l_in = wl + lane < n;
            l_el = 0; l_other = 0; l_multi = 0; l_key = ~0ull;
            if (l_in) {
                l_el = ord.order_l[wl + lane];
                l_other = ord.rank_a[l_el];
                l_multi = ws.multi[l_el];
                const int32_t ml = match_len[l_el];
                l_key = pack_key(ml < 0 ? 0 : ml, l_other);
            }
        }
        if (!kb_valid) {
            kb = ~0ull;
            pb = -1;
            for (int32_t b = lane; b < n_boost; b += kWave) {
                const uint64_t v = coh_load(&ws.bkey[b]);
                if (v < kb) { kb = v; pb = b; }
            }
#pragma unroll
            for (int d = kWave / 2; d > 0; d >>= 1) {
                const uint64_t ok = __shfl_xor(kb, d);
                const int32_t op = __shfl_xor(pb, d);
                if (ok < kb) { kb = ok; pb = op; }
            }
            kb_valid = true;
        }
        // A pick made in bulk must be one that needs no bookkeeping: it has no group (nobody gains
        // from it), it is not in the boosted set, and for a longest-match pick no boosted query
        // ranks before it.
        const uint32_t sa = a_in ? state(a_el) : 1u, sl = l_in ? state(l_el) : 1u;
        // ---- whole k-cycles at once
        if (oldest && k > 1u && (uint32_t)(nb - j) >= k && km1 <= (uint32_t)kWave && !after_single) {
            const bool cand_a = a_in && (sa & 1u) == 0u, cand_l = l_in && sl == 0u;
            const bool hard_a = a_multi != 0 || (sa & 2u) != 0u;
            const bool hard_l = l_multi != 0 || l_key > kb;
            const uint64_t mask_a = __ballot(cand_a), mask_l = __ballot(cand_l);
            int32_t c = (int32_t)__popcll(mask_a);
            const int32_t by_l = (int32_t)((uint32_t)__popcll(mask_l) / km1), by_b = (int32_t)((uint32_t)(nb - j) / k);
            c = by_l < c ? by_l : c;
            c = by_b < c ? by_b : c;
            if (c > 0) {
                const int32_t my_a = (int32_t)__popcll(mask_a & ((1ull << lane) - 1ull));
                const int32_t my_l = (int32_t)__popcll(mask_l & ((1ull << lane) - 1ull));
                // cycles before the first pick that needs bookkeeping
                const uint64_t ha = __ballot(cand_a && hard_a), hl = __ballot(cand_l && hard_l);
                if (ha) { const int32_t lim = (int32_t)__popcll(mask_a & ((1ull << __builtin_ctzll(ha)) - 1ull)); c = lim < c ? lim : c; }
                if (hl) {
                    const int32_t lim = (int32_t)((uint32_t)__popcll(mask_l & ((1ull << __builtin_ctzll(hl)) - 1ull)) / km1);
                    c = lim < c ? lim : c;
                }
                if (c > 0) {
                    const int32_t take_l = c * (int32_t)km1;
                    const bool ch_a = cand_a && my_a < c, ch_l = cand_l && my_l < take_l;
                    const int32_t ia_end = wa + (int32_t)__builtin_ctzll(__ballot(cand_a && my_a == c - 1)) + 1;
                    const int32_t il_end = wl + (int32_t)__builtin_ctzll(__ballot(cand_l && my_l == take_l - 1)) + 1;
                    // the two streams must not meet inside the consumed stretches
                    const uint64_t clash = __ballot((ch_a && a_other < (uint32_t)il_end) || (ch_l && l_other < (uint32_t)ia_end));
                    if (clash == 0ull) {
                        if (ch_a) { batch_idx[j + my_a * (int32_t)k] = (int32_t)a_el; set_bits(a_el, 1u); }
                        if (ch_l) {
                            const uint32_t cyc = (uint32_t)my_l / km1, within = (uint32_t)my_l - cyc * km1;
                            batch_idx[j + (int32_t)(cyc * k + 1u + within)] = (int32_t)l_el;
                            set_bits(l_el, 1u);
                        }
                        __syncthreads();
                        ia = ia_end;
                        il = il_end;
                        j += c * (int32_t)k;
                        continue;
                    }
                }
            }
        }
        // ---- a run of picks of one kind, up to the first pick that needs bookkeeping
        bool single_from_set = false;
        // (what this window's lanes hold is kept for the single pick further down)
        const uint32_t w_el = oldest ? a_el : l_el;
        const int32_t w_multi = oldest ? a_multi : l_multi;
        const int32_t w_base = oldest ? wa : wl;
        uint64_t w_key = ~0ull, w_mask = 0ull;
        {
            const uint32_t run = oldest ? (k == 1u ? (uint32_t)(nb - j) : 1u) : (lpm_only ? (uint32_t)(nb - j) : k - pos);
            const int32_t want = (int32_t)(run < (uint32_t)(nb - j) ? run : (uint32_t)(nb - j));
            const bool cand = oldest ? (a_in && (sa & 1u) == 0u) : (l_in && sl == 0u);
            bool hard = w_multi != 0;
            if (oldest) {
                hard = hard || (sa & 2u) != 0u;
            } else if (cand) {
                w_key = l_key;
                hard = hard || (n_boost > 0 && w_key > kb);
            }
            const uint64_t mask = __ballot(cand), hmask = __ballot(cand && hard);
            w_mask = mask;
            const int32_t my = (int32_t)__popcll(mask & ((1ull << lane) - 1ull));
            int32_t take = (int32_t)__popcll(mask);
            take = take < want ? take : want;
            if (hmask) {
                const int32_t clean = (int32_t)__popcll(mask & ((1ull << __builtin_ctzll(hmask)) - 1ull));
                take = clean < take ? clean : take;
            }
            if (take > 0) {
                if (cand && my < take) { batch_idx[j + my] = (int32_t)w_el; set_bits(w_el, 1u); }
                __syncthreads();
                const int32_t next = w_base + (int32_t)__builtin_ctzll(__ballot(cand && my == take - 1)) + 1;
                if (oldest) ia = next; else il = next;
                j += take;
                pos = lpm_only ? 0u : (uint32_t)(((uint64_t)pos + (uint64_t)take) % k);
                after_single = false;
                continue;
            }
            if (mask == 0ull) {  // nothing pickable in this window
                if (w_base + kWave < n) {  // look further along the order
                    if (oldest) ia = w_base + kWave; else il = w_base + kWave;
                    continue;
                }
                if (oldest) break;          // unreachable while nb <= n
                if (n_boost == 0) break;    // unreachable while nb <= n
                il = n;
                single_from_set = true;     // only boosted queries are left
            }
            // otherwise the next pick needs bookkeeping: it is made on its own below
        }
        // ---- one pick; then the rescoring of the pick's group
        int32_t p = -1;
        int32_t p_multi = -1;  // whether the pick has a group, if a lane already knows
        int32_t p_at = -1;     // its place in the boosted set, if it was taken from there
        if (oldest) {
            const int f = (int)__builtin_ctzll(w_mask);  // not empty: see the run block above
            p = __shfl((int32_t)w_el, f);
            p_multi = __shfl(w_multi, f);
            ia = w_base + f + 1;
        } else {
            // head of the static longest-match order among the queries never boosted, against the
            // best boosted query
            int32_t c1 = -1;
            uint64_t key1 = ~0ull;
            int32_t c1_multi = -1;
            if (!single_from_set) {
                const int f = (int)__builtin_ctzll(w_mask);  // not empty: see the run block above
                c1 = __shfl((int32_t)w_el, f);
                c1_multi = __shfl(w_multi, f);
                il = w_base + f;  // stays on it until it is picked
                key1 = (uint64_t)(((uint64_t)(uint32_t)__shfl((int32_t)(w_key >> 32), f) << 32) |
                                  (uint64_t)(uint32_t)__shfl((int32_t)(uint32_t)w_key, f));
            }
            if (kb < key1) {
                p = coh_load(&ws.bidx[pb]);
                p_at = pb;
            } else {
                p = c1;
                p_multi = c1_multi;
                il += 1;
            }
        }
        if (p < 0) break;  // unreachable while nb <= n
        after_single = true;
        p = uni(p);
        const uint32_t sp = state((uint32_t)p);
        if (lane == 0) {
            batch_idx[j] = p;
            set_bits((uint32_t)p, 1u);
        }
        if (sp & 2u) {  // leaves the boosted set: the last entry takes its place
            const int32_t at = p_at >= 0 ? p_at : uni(coh_load(&ws.bpos[p]));
            const int32_t last = n_boost - 1;
            if (lane == 0 && at != last) {
                const int32_t moved = coh_load(&ws.bidx[last]);
                const int32_t mslot = coh_load(&ws.bslot[last]);
                coh_store(&ws.bkey[at], coh_load(&ws.bkey[last]));
                coh_store(&ws.bidx[at], moved);
                coh_store(&ws.bslot[at], mslot);
                coh_store(&ws.bpos[moved], at);
                if (mslot >= 0) coh_store(&ws.mrec[mslot].w, at);
            }
            n_boost = last;
            kb_valid = false;
        }
        j += 1;
        pos = lpm_only ? 0u : (pos + 1u == k ? 0u : pos + 1u);
        if (p_multi < 0) p_multi = uni((int32_t)ws.multi[p]);
        if (uni(p_multi)) {
            // everything processed stays cached for the rest of the bin: raise the scores of the
            // pick's group to their common prefix with it.  One lane per member: its fields in one
            // round trip, the first kProbe tokens behind the shared part in another; only members
            // that agree with the pick beyond those are compared by the whole wavefront.
            constexpr int kProbe = 8;
            const int64_t off_p = uni64(q.off[p]);
            const int32_t len_p = uni(q.len[p]);
            const int32_t s0 = uni(match_len[p]) + 1;  // the group shares the cached part and the next token
            const int32_t g0 = uni(ws.gstart[p]), gn = uni(ws.gcnt[p]);  // (requested with the three reads above)
            const int32_t gs = uni(ws.gslot[p]);
            const uint64_t below = (1ull << lane) - 1ull;
            if (gn <= kPairGroup && gs >= g0 && gs < g0 + gn) {
                // a small group: the members' records and the pick's row of common prefixes, one round trip
                const bool mine = lane < gn;
                int4 rec = make_int4(-1, 0, 0, -1);
                int32_t ov = 0;
                if (mine) {
                    rec.x = coh_load(&ws.mrec[g0 + lane].x);
                    rec.y = coh_load(&ws.mrec[g0 + lane].y);
                    rec.z = coh_load(&ws.mrec[g0 + lane].z);
                    rec.w = coh_load(&ws.mrec[g0 + lane].w);
                    ov = ws.pair[(size_t)gs * kPairGroup + lane];
                }
                const int32_t i = rec.x;
                uint32_t si = 1u;
                if (mine && i >= 0) si = state((uint32_t)i);
                const bool act = mine && i >= 0 && i != p && (si & 1u) == 0u;
                const bool upd = act && ov > rec.z;
                const bool fresh = upd && (si & 2u) == 0u;
                const uint64_t fm = __ballot(fresh);
                const int32_t at = fresh ? n_boost + (int32_t)__popcll(fm & below) : rec.w;
                uint64_t key = ~0ull;
                if (upd) {
                    key = pack_key(ov, (uint32_t)rec.y);
                    coh_store(&dyn[i], ov);
                    coh_store(&ws.mrec[g0 + lane].z, ov);
                    coh_store(&ws.bkey[at], key);
                    if (fresh) {
                        coh_store(&ws.bidx[at], i);
                        coh_store(&ws.bslot[at], g0 + lane);
                        coh_store(&ws.bpos[i], at);
                        coh_store(&ws.mrec[g0 + lane].w, at);
                        set_bits((uint32_t)i, 2u);
                    }
                }
                n_boost += (int32_t)__popcll(fm);
                uint64_t bk = key;
                int32_t bp = at;
#pragma unroll
                for (int d = kWave / 2; d > 0; d >>= 1) {
                    const uint64_t ok = __shfl_xor(bk, d);
                    const int32_t op = __shfl_xor(bp, d);
                    if (ok < bk) { bk = ok; bp = op; }
                }
                if (kb_valid && bk < kb) { kb = bk; pb = bp; }
            } else
            for (int32_t b = 0; b < gn; b += kWave) {
                const int32_t t = b + lane;
                const int32_t i = t < gn ? ws.members[g0 + t] : -1;
                uint32_t si = 1u;
                if (i >= 0) si = state((uint32_t)i);
                const bool act = i >= 0 && i != p && (si & 1u) == 0u;
                int64_t off_i = 0;
                int32_t len_i = 0, cur = 0, at_old = -1;
                uint32_t ra = 0;
                if (act) {
                    off_i = q.off[i];
                    len_i = q.len[i];
                    cur = coh_load(&dyn[i]);
                    ra = ord.rank_a[i];
                    if (si & 2u) at_old = coh_load(&ws.bpos[i]);
                }
                const int32_t lim = len_i < len_p ? len_i : len_p;
                const int32_t rem = act ? lim - s0 : 0;  // tokens that may still agree
                int32_t add = 0;
                bool more = false;
                if (rem > 0) {
                    int32_t av[kProbe], bv[kProbe];
#pragma unroll
                    for (int u = 0; u < kProbe; ++u) {
                        const int32_t c = u < rem ? u : rem - 1;
                        av[u] = q.tokens[off_i + s0 + c];
                        bv[u] = q.tokens[off_p + s0 + c];
                    }
                    add = rem < kProbe ? rem : kProbe;
#pragma unroll
                    for (int u = kProbe - 1; u >= 0; --u)
                        if (u < rem && av[u] != bv[u]) add = u;
                    more = add == kProbe && rem > kProbe;
                }
                uint64_t longm = __ballot(more);
                while (longm) {
                    const int src = (int)__builtin_ctzll(longm);
                    longm &= longm - 1ull;
                    const int64_t oi = (int64_t)(((uint64_t)(uint32_t)__shfl((int32_t)((uint64_t)off_i >> 32), src) << 32) |
                                                 (uint64_t)(uint32_t)__shfl((int32_t)(uint32_t)off_i, src));
                    const int32_t ri = __shfl(rem, src);
                    const int32_t extra = wave_common_prefix(q.tokens + oi + s0 + kProbe, q.tokens + off_p + s0 + kProbe,
                                                             ri - kProbe, lane);
                    if (lane == src) add += extra;
                }
                const int32_t ov = s0 + add;
                const bool upd = act && ov > cur;
                const bool fresh = upd && (si & 2u) == 0u;
                const uint64_t fm = __ballot(fresh);
                const int32_t at = fresh ? n_boost + (int32_t)__popcll(fm & below) : at_old;
                uint64_t key = ~0ull;
                if (upd) {
                    key = pack_key(ov, ra);
                    coh_store(&dyn[i], ov);
                    coh_store(&ws.bkey[at], key);
                    if (fresh) {
                        coh_store(&ws.bidx[at], i);
                        coh_store(&ws.bslot[at], -1);
                        coh_store(&ws.bpos[i], at);
                        set_bits((uint32_t)i, 2u);
                    }
                }
                n_boost += (int32_t)__popcll(fm);
                // the best of the keys just written (keys only ever get smaller)
                uint64_t bk = key;
                int32_t bp = at;
#pragma unroll
                for (int d = kWave / 2; d > 0; d >>= 1) {
                    const uint64_t ok = __shfl_xor(bk, d);
                    const int32_t op = __shfl_xor(bp, d);
                    if (ok < bk) { bk = ok; bp = op; }
                }
                if (kb_valid && bk < kb) { kb = bk; pb = bp; }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");  // this pick's stores before the next reads of any lane
        __syncthreads();
    }
}

static size_t carve_dyn(DynWs &d, char *base, int32_t n, size_t start) {
    size_t o = start;
    auto take = [&](size_t bytes) { void *p = base ? base + o : nullptr; o += align_up(bytes, 256); return p; };
    size_t nn = (size_t)(n > 0 ? n : 1);
    uint32_t table = 64;
    while (table < 2 * nn) table <<= 1;
    d.table_mask = table - 1u;
    d.gk = (uint64_t *)take(nn * 8);
    d.slot_of = (int32_t *)take(nn * 4);
    d.multi = (uint8_t *)take(nn);
    d.rep = (int32_t *)take((size_t)table * 4);
    d.cnt = (int32_t *)take((size_t)table * 4);
    d.start = (int32_t *)take((size_t)table * 4);
    d.fill = (int32_t *)take((size_t)table * 4);
    d.tile_sum = (int32_t *)take((size_t)((table + 8191) / 8192) * 4);
    d.members = (int32_t *)take(nn * 4);
    d.gstart = (int32_t *)take(nn * 4);
    d.gcnt = (int32_t *)take(nn * 4);
    d.bkey = (uint64_t *)take(nn * 8);
    d.bidx = (int32_t *)take(nn * 4);
    d.bpos = (int32_t *)take(nn * 4);
    d.bslot = (int32_t *)take(nn * 4);
    d.gslot = (int32_t *)take(nn * 4);
    d.mrec = (int4 *)take(nn * 16);
    d.pair = (int32_t *)take(nn * 4 * kPairGroup);
    return o;
}

}  // namespace klpm

using namespace klpm;

extern "C" int kLPM_select_dynamic_workspace_bytes(int32_t n, size_t *out_bytes) {
    if (n < 0 || !out_bytes) return KLPM_EINVAL;
    DynWs d;
    *out_bytes = carve_dyn(d, nullptr, n, align_up(select_sort_workspace_bytes(n), 256));
    return KLPM_OK;
}

extern "C" int kLPM_select_dynamic(const kLPM_queries *q, const int32_t *match_len, const int32_t *last_node, uint32_t k,
                                   const uint32_t *k_dev, int32_t batch, uint32_t flags, int32_t max_match,
                                   uint32_t *phase_inout, int32_t *dyn_match, int32_t *batch_idx, int32_t *n_selected,
                                   void *workspace, size_t workspace_bytes, kLPM_stream stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!q || q->n < 0 || q->n > kDynMaxN || q->n_tokens < 0 || batch < 0 || !phase_inout || !n_selected) return KLPM_EINVAL;
    const int32_t n = q->n;
    if (n > 0 && (!q->tokens || !q->off || !q->len || !q->arrival || !match_len || !last_node || !dyn_match))
        return KLPM_EINVAL;
    if (n > 0 && batch > 0 && !batch_idx) return KLPM_EINVAL;
    size_t need = 0;
    kLPM_select_dynamic_workspace_bytes(n, &need);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u)) return KLPM_EARENA;
    const size_t sort_bytes = align_up(select_sort_workspace_bytes(n), 256);
    DynWs d;
    carve_dyn(d, (char *)workspace, n, sort_bytes);
    QView qv;
    qv.tokens = q->tokens; qv.off = q->off; qv.len = q->len; qv.n_tokens = q->n_tokens; qv.n = n; qv.n_live = q->n_live;
    SelectOrders ord;
    // the static orders are taken over the match lengths against the cache
    int rc = build_select_orders(q->arrival, match_len, nullptr, n, q->n_live, true, workspace, sort_bytes, stream, &ord,
                                 (flags & KLPM_SELECT_FIFO) != 0, max_match);
    if (rc) return rc;
    if (n > 0) {
        const int64_t work = (int64_t)d.table_mask + 1 > n ? (int64_t)d.table_mask + 1 : n;
        const unsigned g = (unsigned)((n + 255) / 256);
        hipLaunchKernelGGL(k_dyn_init, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, stream, qv, match_len, last_node, d,
                           dyn_match);
        hipLaunchKernelGGL(k_dyn_insert, dim3(g), dim3(256), 0, stream, LiveQ{n, q->n_live}, match_len, d);
        const unsigned tiles = (unsigned)(((int64_t)d.table_mask + kDynScanTile) / kDynScanTile);
        hipLaunchKernelGGL(k_dyn_tile_sums, dim3(tiles), dim3(kDynScanThreads), 0, stream, d);
        hipLaunchKernelGGL(k_dyn_offsets, dim3(tiles), dim3(kDynScanThreads), 0, stream, d);
        hipLaunchKernelGGL(k_dyn_scatter, dim3(g), dim3(256), 0, stream, LiveQ{n, q->n_live}, d);
        hipLaunchKernelGGL(k_dyn_pairs, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, stream, qv, match_len, ord.rank_a, d);
    }
    hipLaunchKernelGGL(k_dyn_walk, dim3(1), dim3(kWave), 0, stream, qv, match_len, ord, d, dyn_match, KArg{k, k_dev}, batch, phase_inout,
                       batch_idx, n_selected);
    return check_launch();
}
