/*
 * CPU ORACLE for the k-LPM scheduling step over a RadixAttention-style prefix
 * cache.  TEST INFRASTRUCTURE ONLY: a plain, slow, pointer-based reference
 * written from the paper, used by the tests and as the reported CPU baseline.
 * It shares no code with the GPU library and must never be called from the
 * product path.
 *
 * What each function follows:
 *   orc_match   - overlap(x, y) = length of the maximal common prefix (Sec. 1.2,
 *                 Notation), maximised over all strings held in the radix tree
 *                 that the prefix cache maintains (Sec. 1, RadixAttention).
 *   orc_select  - Algorithm 1 (k-LPM): process the oldest query, then k-1 times
 *                 the query with the largest prefix-cache hit; the resulting
 *                 order is cut into bins of B (Sec. 2.1).  k = 1 is FCFS and
 *                 k = infinity is LPM (Sec. 4).
 *   orc_commit  - the cache keeps what every processed query left behind in a
 *                 radix tree and evicts least-recently-used entries under a
 *                 fixed memory size (Sec. 1; fixed pool, Sec. 2.1).
 *   orc_def2    - completion times R(j_k) of the LLM-instance computation model
 *                 (Def. 2), fp64.
 *
 * Readings taken where the paper is silent (listed in the design notes): the
 * score is the absolute match length; ties go to the earlier arrival, then to
 * the lower queue index; the LPM endpoint is a pure longest-match order; an
 * edge is split where an inserted prompt diverges from it or ends inside it;
 * every admitted prompt gets one new tick of a logical clock and stamps it on
 * all nodes of its path; eviction removes whole leaves, smallest tick first,
 * until the token total is within budget; only commit touches ticks.
 *
 * Variants: the score handed to orc_select may be the hit rate floor(m 2^b / |x|)
 * instead of m (the wording of Algorithm 1), and a per-query tie key (uniform
 * random numbers: the footnote of Sec. 4.2) may decide between equal scores.
 *
 * Parity pins (tests, CPU-only): brute-force pairwise common prefixes, a
 * literal list-based Algorithm 1, a dictionary-of-paths LRU model, the worked
 * four-query example of Sec. 4.2, and the closed forms in the proof of Thm. 2.
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct ONode {
    struct ONode *parent;
    struct ONode **child; /* sorted by first edge token, ascending */
    int32_t n_child, cap_child;
    int32_t *tok; /* this node's edge label (owned copy) */
    int32_t len;
    uint64_t tick;  /* last use (logical clock) */
    int64_t slot;   /* index in OTree.all */
} ONode;

typedef struct OTree {
    ONode *root;
    ONode **all; /* every non-root node, unordered */
    int64_t n_all, cap_all;
    int64_t total_tokens;
    uint64_t clock;
} OTree;

typedef struct {
    int64_t total_tokens, inserted_tokens, evicted_tokens;
    int32_t n_nodes, new_nodes, evicted_nodes, pad;
    uint64_t clock;
} OStats;

static ONode *node_new(const int32_t *tok, int32_t len, uint64_t tick) {
    ONode *v = (ONode *)calloc(1, sizeof(ONode));
    v->tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)(len > 0 ? len : 1));
    if (len > 0) memcpy(v->tok, tok, sizeof(int32_t) * (size_t)len);
    v->len = len;
    v->tick = tick;
    v->slot = -1;
    return v;
}

static void tree_register(OTree *t, ONode *v) {
    if (t->n_all == t->cap_all) {
        t->cap_all = t->cap_all ? 2 * t->cap_all : 1024;
        t->all = (ONode **)realloc(t->all, sizeof(ONode *) * (size_t)t->cap_all);
    }
    v->slot = t->n_all;
    t->all[t->n_all++] = v;
}

static void tree_unregister(OTree *t, ONode *v) {
    ONode *last = t->all[t->n_all - 1];
    t->all[v->slot] = last;
    last->slot = v->slot;
    t->n_all--;
}

/* position of the child whose edge starts with `first`, or the insertion point */
static int32_t child_pos(const ONode *v, int32_t first, int *found) {
    int32_t lo = 0, hi = v->n_child;
    while (lo < hi) {
        int32_t mid = lo + (hi - lo) / 2;
        if (v->child[mid]->tok[0] < first) lo = mid + 1; else hi = mid;
    }
    *found = (lo < v->n_child && v->child[lo]->tok[0] == first);
    return lo;
}

static ONode *child_find(const ONode *v, int32_t first) {
    int found;
    int32_t p = child_pos(v, first, &found);
    return found ? v->child[p] : NULL;
}

static void child_add(ONode *v, ONode *c) {
    int found;
    int32_t p = child_pos(v, c->tok[0], &found);
    if (v->n_child == v->cap_child) {
        v->cap_child = v->cap_child ? 2 * v->cap_child : 2;
        v->child = (ONode **)realloc(v->child, sizeof(ONode *) * (size_t)v->cap_child);
    }
    memmove(v->child + p + 1, v->child + p, sizeof(ONode *) * (size_t)(v->n_child - p));
    v->child[p] = c;
    v->n_child++;
    c->parent = v;
}

static void child_remove(ONode *v, ONode *c) {
    int found;
    int32_t p = child_pos(v, c->tok[0], &found);
    memmove(v->child + p, v->child + p + 1, sizeof(ONode *) * (size_t)(v->n_child - p - 1));
    v->n_child--;
}

OTree *orc_tree_new(void) {
    OTree *t = (OTree *)calloc(1, sizeof(OTree));
    t->root = node_new(NULL, 0, 0);
    return t;
}

static void free_rec(ONode *v) {
    for (int32_t i = 0; i < v->n_child; i++) free_rec(v->child[i]);
    free(v->child);
    free(v->tok);
    free(v);
}

void orc_tree_free(OTree *t) {
    if (!t) return;
    free_rec(t->root);
    free(t->all);
    free(t);
}

int64_t orc_total_tokens(const OTree *t) { return t->total_tokens; }
int64_t orc_n_nodes(const OTree *t) { return t->n_all; }
uint64_t orc_clock(const OTree *t) { return t->clock; }

/* ---- match: longest prefix of x held in the tree (max over cached strings of overlap) ---- */
static int32_t match_one(const OTree *t, const int32_t *x, int32_t len) {
    const ONode *cur = t->root;
    int32_t d = 0;
    while (d < len) {
        const ONode *c = child_find(cur, x[d]);
        if (!c) break;
        int32_t lim = c->len < len - d ? c->len : len - d;
        int32_t j = 0;
        while (j < lim && c->tok[j] == x[d + j]) j++;
        d += j;
        if (j < c->len) break; /* diverged, or the prompt ended, inside this edge */
        cur = c;
    }
    return d;
}

void orc_match(const OTree *t, const int32_t *tokens, const int64_t *off, const int32_t *len, int32_t n,
               int32_t *match_len) {
    for (int32_t i = 0; i < n; i++) match_len[i] = match_one(t, tokens + off[i], len[i]);
}

typedef struct {
    const OTree *t;
    const int32_t *tokens;
    const int64_t *off;
    const int32_t *len;
    int32_t *out;
    int32_t begin, end;
} MatchJob;

static void *match_worker(void *p) {
    MatchJob *j = (MatchJob *)p;
    for (int32_t i = j->begin; i < j->end; i++) j->out[i] = match_one(j->t, j->tokens + j->off[i], j->len[i]);
    return NULL;
}

/* the same walk with the queue split statically over host threads (the tree is read-only here) */
void orc_match_mt(const OTree *t, const int32_t *tokens, const int64_t *off, const int32_t *len, int32_t n,
                  int32_t *match_len, int32_t n_threads) {
    if (n_threads < 1) n_threads = 1;
    if (n_threads > 256) n_threads = 256;
    pthread_t th[256];
    MatchJob job[256];
    for (int32_t w = 0; w < n_threads; w++) {
        job[w].t = t; job[w].tokens = tokens; job[w].off = off; job[w].len = len; job[w].out = match_len;
        job[w].begin = (int32_t)((int64_t)n * w / n_threads);
        job[w].end = (int32_t)((int64_t)n * (w + 1) / n_threads);
        pthread_create(&th[w], NULL, match_worker, &job[w]);
    }
    for (int32_t w = 0; w < n_threads; w++) pthread_join(th[w], NULL);
}

/* ---- select: Algorithm 1 over a static score vector, cut after B picks ---- */
/* k == 0 or k == UINT32_MAX encodes k = infinity (pure LPM order, no oldest pick). */
/* tie (may be NULL): a per-query key that decides between equal scores before the arrival time does;
 * filled with independent uniform numbers it gives the uniformly random tie-break that the
 * theory of Sec. 4.2 assumes (footnote there). */
int32_t orc_select(const uint64_t *arrival, const int32_t *match_len, const uint32_t *tie, int32_t n, uint32_t k,
                   int32_t batch, uint32_t *phase_inout, int32_t *batch_idx) {
    int lpm_only = (k == 0u || k == 0xFFFFFFFFu);
    uint32_t phase = lpm_only ? 0u : (*phase_inout % k);
    char *taken = (char *)calloc((size_t)(n > 0 ? n : 1), 1);
    int32_t n_out = batch < n ? batch : n;
    if (n_out < 0) n_out = 0;
    for (int32_t j = 0; j < n_out; j++) {
        int oldest_slot = !lpm_only && ((phase + (uint32_t)j) % k == 0u);
        int32_t best = -1;
        for (int32_t i = 0; i < n; i++) {
            if (taken[i]) continue;
            if (best < 0) { best = i; continue; }
            if (oldest_slot) {
                /* oldest waiting query; equal times -> lower index (i ascending keeps the first) */
                if (arrival[i] < arrival[best]) best = i;
            } else {
                /* largest prefix-cache hit; ties -> smaller tie key (if any), earlier arrival, lower index */
                if (match_len[i] != match_len[best]) {
                    if (match_len[i] > match_len[best]) best = i;
                } else if (tie && tie[i] != tie[best]) {
                    if (tie[i] < tie[best]) best = i;
                } else if (arrival[i] < arrival[best]) {
                    best = i;
                }
            }
        }
        taken[best] = 1;
        batch_idx[j] = best;
    }
    free(taken);
    *phase_inout = lpm_only ? 0u : (uint32_t)(((uint64_t)phase + (uint64_t)n_out) % k);
    return n_out;
}

static int32_t overlap(const int32_t *a, int32_t la, const int32_t *b, int32_t lb) {
    int32_t lim = la < lb ? la : lb, j = 0;
    while (j < lim && a[j] == b[j]) j++;
    return j;
}

/* ---- select with in-batch rescoring (the dynamic rule of Def. 2 inside one bin) ----
 * Def. 2 credits a query with its overlap with the prompt processed just before it; with a cache
 * that keeps what it has processed, a query picked later in the same bin overlaps with the cached
 * strings *and* with every prompt picked before it in the bin.  So after each pick p the score of
 * every remaining query i becomes max(score_i, overlap(x_i, x_p)); Algorithm 1's rule is applied to
 * the current scores.  score[] holds the match lengths against the cache on entry and, on return,
 * for a picked query its score when it was picked, for the others their final score. */
int32_t orc_select_dynamic(const int32_t *tokens, const int64_t *off, const int32_t *len, const uint64_t *arrival,
                           int32_t *score, int32_t n, uint32_t k, int32_t batch, uint32_t *phase_inout,
                           int32_t *batch_idx) {
    int lpm_only = (k == 0u || k == 0xFFFFFFFFu);
    uint32_t phase = lpm_only ? 0u : (*phase_inout % k);
    char *taken = (char *)calloc((size_t)(n > 0 ? n : 1), 1);
    int32_t n_out = batch < n ? batch : n;
    if (n_out < 0) n_out = 0;
    for (int32_t j = 0; j < n_out; j++) {
        int oldest_slot = !lpm_only && ((phase + (uint32_t)j) % k == 0u);
        int32_t best = -1;
        for (int32_t i = 0; i < n; i++) {
            if (taken[i]) continue;
            if (best < 0) { best = i; continue; }
            if (oldest_slot) {
                if (arrival[i] < arrival[best]) best = i;
            } else if (score[i] > score[best] || (score[i] == score[best] && arrival[i] < arrival[best])) {
                best = i;
            }
        }
        if (best < 0) break; /* cannot happen: n_out <= n */
        taken[best] = 1;
        batch_idx[j] = best;
        for (int32_t i = 0; i < n; i++) {
            if (taken[i]) continue;
            int32_t ov = overlap(tokens + off[i], len[i], tokens + off[best], len[best]);
            if (ov > score[i]) score[i] = ov;
        }
    }
    free(taken);
    *phase_inout = lpm_only ? 0u : (uint32_t)(((uint64_t)phase + (uint64_t)n_out) % k);
    return n_out;
}

/* ---- commit: insert admitted prompts in pick order, then LRU-evict to the budget ---- */
static void split_edge(OTree *t, ONode *v, int32_t j) {
    /* v keeps tok[0..j); a new lower node takes tok[j..len), v's children and v's old tick */
    ONode *low = node_new(v->tok + j, v->len - j, v->tick);
    low->child = v->child; low->n_child = v->n_child; low->cap_child = v->cap_child;
    for (int32_t i = 0; i < low->n_child; i++) low->child[i]->parent = low;
    v->child = NULL; v->n_child = 0; v->cap_child = 0;
    v->len = j;
    child_add(v, low);
    tree_register(t, low);
}

static void insert_one(OTree *t, const int32_t *x, int32_t len, uint64_t tick, OStats *st) {
    ONode *cur = t->root;
    int32_t d = 0;
    while (d < len) {
        ONode *c = child_find(cur, x[d]);
        if (!c) {
            ONode *leaf = node_new(x + d, len - d, tick);
            child_add(cur, leaf);
            tree_register(t, leaf);
            t->total_tokens += len - d;
            st->inserted_tokens += len - d;
            st->new_nodes++;
            return;
        }
        int32_t lim = c->len < len - d ? c->len : len - d;
        int32_t j = 0;
        while (j < lim && c->tok[j] == x[d + j]) j++;
        if (j < c->len) { split_edge(t, c, j); st->new_nodes++; }
        c->tick = tick;
        cur = c;
        d += j;
    }
}

/* protect: the paths of the `protect` most recently admitted prompts (ticks >= clock - protect) are in
 * flight and must stay; eviction stops when the least recently used leaf is one of them, even if
 * the total is still above the budget. */
static void evict_to_budget(OTree *t, int64_t budget, int64_t protect, OStats *st) {
    uint64_t keep_from = (protect <= 0) ? UINT64_MAX : ((uint64_t)protect >= t->clock ? 0 : t->clock - (uint64_t)protect);
    while (t->total_tokens > budget && t->n_all > 0) {
        ONode *victim = NULL;
        for (int64_t i = 0; i < t->n_all; i++) {
            ONode *v = t->all[i];
            if (v->n_child != 0) continue;
            if (!victim || v->tick < victim->tick) victim = v;
        }
        if (victim->tick >= keep_from) break;
        child_remove(victim->parent, victim);
        tree_unregister(t, victim);
        t->total_tokens -= victim->len;
        st->evicted_tokens += victim->len;
        st->evicted_nodes++;
        free(victim->child);
        free(victim->tok);
        free(victim);
    }
}

void orc_commit(OTree *t, const int32_t *tokens, const int64_t *off, const int32_t *len, const int32_t *batch_idx,
                int32_t n_batch, int64_t budget, int64_t protect, OStats *st) {
    memset(st, 0, sizeof(*st));
    for (int32_t j = 0; j < n_batch; j++) {
        int32_t q = batch_idx[j];
        insert_one(t, tokens + off[q], len[q], t->clock, st);
        t->clock++;
    }
    evict_to_budget(t, budget, protect, st);
    st->total_tokens = t->total_tokens;
    st->n_nodes = (int32_t)t->n_all;
    st->clock = t->clock;
}

/* ---- canonical snapshot: header, node records in DFS pre-order (children by ascending first token), tokens ---- */
typedef struct { int32_t depth_start, edge_len; uint64_t tick; int32_t n_children, pad; } SnapRec;

static void snap_rec(const ONode *v, int32_t depth, SnapRec **rec, int32_t **tok) {
    for (int32_t i = 0; i < v->n_child; i++) {
        const ONode *c = v->child[i];
        (*rec)->depth_start = depth; (*rec)->edge_len = c->len; (*rec)->tick = c->tick;
        (*rec)->n_children = c->n_child; (*rec)->pad = 0;
        (*rec)++;
        memcpy(*tok, c->tok, sizeof(int32_t) * (size_t)c->len);
        *tok += c->len;
        snap_rec(c, depth + c->len, rec, tok);
    }
}

size_t orc_snapshot_bytes(const OTree *t) {
    return 24 + (size_t)t->n_all * sizeof(SnapRec) + (size_t)t->total_tokens * 4;
}

size_t orc_snapshot(const OTree *t, void *buf, size_t cap) {
    size_t need = orc_snapshot_bytes(t);
    if (cap < need) return 0;
    int64_t *h = (int64_t *)buf;
    h[0] = t->n_all; h[1] = t->total_tokens; h[2] = (int64_t)t->clock;
    SnapRec *rec = (SnapRec *)((char *)buf + 24);
    int32_t *tok = (int32_t *)((char *)buf + 24 + (size_t)t->n_all * sizeof(SnapRec));
    snap_rec(t->root, 0, &rec, &tok);
    return need;
}

/* ---- Def. 2: completion times for a given processing order (last-prompt cache model) ---- */

void orc_def2(const int32_t *tokens, const int64_t *off, const int32_t *len, const uint64_t *arrival,
              const int32_t *order, int32_t n, double c_attn, double t_start, double *completion) {
    double r_prev = t_start;
    for (int32_t p = 0; p < n; p++) {
        int32_t q = order[p];
        double x = (double)len[q];
        double ov = 0.0;
        if (p > 0) {
            int32_t qp = order[p - 1];
            ov = (double)overlap(tokens + off[q], len[q], tokens + off[qp], len[qp]);
        }
        double start = r_prev > (double)arrival[q] ? r_prev : (double)arrival[q];
        r_prev = start + (1.0 + c_attn * x) * (x - ov);
        completion[q] = r_prev;
    }
}
