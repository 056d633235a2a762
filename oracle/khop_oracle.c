/*
 * CPU oracle for batched k-hop knowledge-graph retrieval.  TEST INFRASTRUCTURE
 * ONLY: this file is the slow, plain reference that the GPU library is checked
 * against.  Nothing in the product path may include, link or call it, and it
 * shares no code with the HIP sources.
 *
 * What it computes (one query at a time, queries independent):
 *
 *   A knowledge graph is a set of triples t = (s_t, r_t, o_t), t = 0..T-1
 *   (paper Sec. 3.1).  The column index t of the SUB / OBJ / REL incidence
 *   matrices (Eq. 1-3) is the triple's position in the input arrays and is used
 *   as its edge id.  One hop maps an entity indicator vector q to
 *   q . SUB . OBJ (Eq. 4): a triple is active when its subject is set in q
 *   (Eq. 5-6), and an active triple sets its object.  A per-query relation
 *   whitelist M removes active triples whose relation is not in M before the
 *   OBJ product.  Iterating from the seed vector q^(0) gives q^(h).
 *
 *   hop(v)   = the least h in [0, k] with q^(h)[v] = 1   ("within k relational
 *              steps", Sec. 3.1); undefined when there is none.
 *   pred(v)  = for hop(v) = h >= 1 the smallest edge id t with o_t = v,
 *              r_t in M and hop(s_t) = h - 1; -1 for seeds.
 *   trav(h)  = number of triples whose subject has hop h - 1 (the triples the
 *              hop inspects, whatever their relation), h = 1..k.
 *
 * Two evaluation modes give the same numbers by construction of the
 * definition; both are kept so that each checks the other:
 *   mode 0: per-subject index of triple ids (stable counting sort, so ids
 *           ascend inside a subject), levels kept as lists;
 *   mode 1: no index at all - every hop rescans the whole triple list.
 *
 * Shortest-path listing (oracle_paths): for a target v with hop(v) = d the
 * paths are all edge sequences (t_1..t_d) with s_{t_1} a seed, o_{t_i} =
 * s_{t_{i+1}}, o_{t_d} = v, hop(s_{t_i}) = i - 1 and every r_{t_i} in M
 * (the chains of active triples of Eq. 5-7, restricted to shortest ones).
 * They are ordered lexicographically by (t_d, t_{d-1}, .., t_1) and the first
 * max_paths are returned, each written seed -> target.
 *
 * Walk-exact levels (oracle_walk_levels): the iteration of Eq. 4 taken
 * literally, without a visited set: level h holds the entities that end a walk
 * of exactly h allowed triples from a seed, q^(h) = q^(h-1) . SUB . OBJ with
 * the whitelist applied to the active triples.  An entity may appear in several
 * levels.  Pins: dense boolean matrix powers, brute-force walk enumeration,
 * closed forms on cycles / paths / self loops, and against oracle_khop itself
 * (union over h = reached set, first h = hop).
 *
 * Walk listing (oracle_walk_paths): the complete paths of Sec. 3.3 for the
 * iteration without a visited set.  For a pair (query, target, length d) the
 * walks are all edge sequences (t_1..t_d) with s_{t_1} a seed, o_{t_i} =
 * s_{t_{i+1}}, o_{t_d} = target and every r_{t_i} in M; an entity may repeat.
 * They are ordered lexicographically by (t_d, t_{d-1}, .., t_1) and the first
 * max_paths are returned, each written seed -> target.  Evaluated backward from
 * the target through the sets q^(d-1), .., q^(0), which are rebuilt here by
 * rescanning the triple list once per hop.  Pins
 * (tests/test_oracle_walk_paths_pins.py): forward enumeration of every walk,
 * walk counts from integer powers of the adjacency matrix, closed forms.
 *
 * Active-triple sets (oracle_active_triples): T_h of Eq. 5-6 for one query,
 * given the support of q^(h-1) as an entity list: every triple whose subject
 * is in that list and whose relation is in M, written out with the triple list
 * scanned once in index order and then ordered by (subject, triple index) -
 * the order of SUB's rows, with triple indices ascending inside a subject.
 * The caller takes (s_t, r_t, o_t) of Eq. 7 from the input arrays.  Pins
 * (tests/test_oracle_triples_pins.py): the dense product q . SUB of Eq. 5,
 * t^(h) . OBJ = q^(h) against oracle_walk_levels, |T_h| against trav(h),
 * closed forms and the hand-worked example.
 *
 * Parity pins (see tests/test_oracle_pins.py): boolean products of dense
 * SUB / REL / OBJ matrices, brute-force walk enumeration, closed forms on
 * paths / cycles / stars / trees, networkx and scipy shortest-path lengths,
 * mode 0 against mode 1, and the hop / pred invariants.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define UNREACHED 255

static int relation_allowed(const uint64_t *mask, int32_t r)
{
    if (!mask) return 1;
    return (int)((mask[r >> 6] >> (r & 63)) & 1u);
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Stable counting sort of triple ids by `key` (subject or object). */
static int build_index(const int32_t *key, int64_t T, int32_t E,
                       int64_t **first_out, int32_t **ids_out)
{
    int64_t *first = (int64_t *)calloc((size_t)E + 2, sizeof(int64_t));
    int32_t *ids = (int32_t *)malloc((size_t)(T > 0 ? T : 1) * sizeof(int32_t));
    if (!first || !ids) { free(first); free(ids); return -1; }
    for (int64_t t = 0; t < T; ++t) first[key[t] + 1]++;
    for (int32_t e = 0; e < E; ++e) first[e + 1] += first[e];
    int64_t *cursor = (int64_t *)malloc((size_t)(E + 1) * sizeof(int64_t));
    if (!cursor) { free(first); free(ids); return -1; }
    memcpy(cursor, first, (size_t)(E + 1) * sizeof(int64_t));
    for (int64_t t = 0; t < T; ++t) ids[cursor[key[t]]++] = (int32_t)t;
    free(cursor);
    *first_out = first;
    *ids_out = ids;
    return 0;
}

typedef struct {
    uint8_t *hop;      /* [E], UNREACHED when not reached */
    int32_t *pred;     /* [E] */
    int32_t *touched;  /* entities with hop set, in discovery order */
    int64_t n_touched;
} bfs_state;

static int state_init(bfs_state *st, int32_t E)
{
    st->hop = (uint8_t *)malloc((size_t)E);
    st->pred = (int32_t *)malloc((size_t)E * sizeof(int32_t));
    st->touched = (int32_t *)malloc((size_t)E * sizeof(int32_t));
    st->n_touched = 0;
    if (!st->hop || !st->pred || !st->touched) return -1;
    memset(st->hop, UNREACHED, (size_t)E);
    return 0;
}

static void state_reset(bfs_state *st)
{
    for (int64_t i = 0; i < st->n_touched; ++i) st->hop[st->touched[i]] = UNREACHED;
    st->n_touched = 0;
}

static void state_free(bfs_state *st)
{
    free(st->hop); free(st->pred); free(st->touched);
}

/* Relax one active triple t at hop h. */
static inline void relax(bfs_state *st, const int32_t *obj, int32_t t, int h)
{
    int32_t v = obj[t];
    if (st->hop[v] == UNREACHED) {
        st->hop[v] = (uint8_t)h;
        st->pred[v] = t;
        st->touched[st->n_touched++] = v;
    } else if (st->hop[v] == h && t < st->pred[v]) {
        st->pred[v] = t;
    }
}

/* One query.  The touched list is grouped by hop: level h occupies
 * touched[lvl_begin[h] .. lvl_begin[h+1]). */
static void bfs_one(bfs_state *st, int64_t T, const int32_t *subj,
                    const int32_t *rel, const int32_t *obj,
                    const int64_t *first, const int32_t *ids, int mode,
                    const int32_t *seeds, int64_t n_seeds, int k,
                    const uint64_t *mask, int64_t *trav /* [k] or NULL */)
{
    for (int64_t i = 0; i < n_seeds; ++i) {
        int32_t e = seeds[i];
        if (st->hop[e] == UNREACHED) {
            st->hop[e] = 0;
            st->pred[e] = -1;
            st->touched[st->n_touched++] = e;
        }
    }
    int64_t lvl_lo = 0, lvl_hi = st->n_touched;
    for (int h = 1; h <= k; ++h) {
        int64_t inspected = 0;
        if (lvl_hi == lvl_lo) break;
        if (mode == 0) {
            for (int64_t i = lvl_lo; i < lvl_hi; ++i) {
                int32_t s = st->touched[i];
                for (int64_t j = first[s]; j < first[s + 1]; ++j) {
                    int32_t t = ids[j];
                    ++inspected;
                    if (!relation_allowed(mask, rel[t])) continue;
                    relax(st, obj, t, h);
                }
            }
        } else {
            for (int64_t t = 0; t < T; ++t) {
                if (st->hop[subj[t]] != h - 1) continue;
                ++inspected;
                if (!relation_allowed(mask, rel[t])) continue;
                relax(st, obj, (int32_t)t, h);
            }
        }
        if (trav) trav[h - 1] = inspected;
        lvl_lo = lvl_hi;
        lvl_hi = st->n_touched;
    }
}

/*
 * Batched k-hop retrieval.  All pointers are host memory.
 *   rel_mask: NULL (every relation allowed) or uint64[Q][rel_words], bit r%64
 *             of word r/64 set when query q may follow relation r.
 *   reached_off[Q+1], traversed[Q*k] are caller-allocated; *entity, *hop,
 *   *pred are malloc'ed here (query-major, ascending entity id inside a
 *   query) and released with oracle_free.
 * Returns 0, or -1 on allocation failure / bad arguments.
 */
int oracle_khop(int64_t T, int32_t E, const int32_t *subj, const int32_t *rel,
                const int32_t *obj, int32_t Q, const int64_t *seed_off,
                const int32_t *seeds, int32_t k, const uint64_t *rel_mask,
                int32_t rel_words, int32_t mode, int32_t nthreads,
                int64_t *reached_off, int32_t **entity, uint8_t **hop,
                int32_t **pred, int64_t *traversed)
{
    if (k < 0 || k > 254 || E <= 0 || T < 0 || Q < 0) return -1;
    for (int64_t i = 0; i < seed_off[Q]; ++i)
        if (seeds[i] < 0 || seeds[i] >= E) return -1;
    int64_t *first = NULL;
    int32_t *ids = NULL;
    if (mode == 0 && build_index(subj, T, E, &first, &ids) != 0) return -1;

    int32_t **q_ent = (int32_t **)calloc((size_t)Q + 1, sizeof(*q_ent));
    int64_t *q_cnt = (int64_t *)calloc((size_t)Q + 1, sizeof(int64_t));
    uint8_t **q_hop = (uint8_t **)calloc((size_t)Q + 1, sizeof(*q_hop));
    int32_t **q_pred = (int32_t **)calloc((size_t)Q + 1, sizeof(*q_pred));
    int failed = 0;
    if (traversed && k > 0) memset(traversed, 0, (size_t)Q * (size_t)k * sizeof(int64_t));
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
#pragma omp parallel
    {
        bfs_state st;
        int ok = state_init(&st, E) == 0;
#pragma omp for schedule(dynamic, 1)
        for (int32_t q = 0; q < Q; ++q) {
            if (!ok) { failed = 1; continue; }
            const uint64_t *mask = rel_mask ? rel_mask + (size_t)q * rel_words : NULL;
            bfs_one(&st, T, subj, rel, obj, first, ids, mode,
                    seeds + seed_off[q], seed_off[q + 1] - seed_off[q], k, mask,
                    traversed ? traversed + (size_t)q * k : NULL);
            int64_t n = st.n_touched;
            qsort(st.touched, (size_t)n, sizeof(int32_t), cmp_i32);
            q_cnt[q] = n;
            q_ent[q] = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
            q_hop[q] = (uint8_t *)malloc((size_t)(n > 0 ? n : 1));
            q_pred[q] = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
            if (!q_ent[q] || !q_hop[q] || !q_pred[q]) { failed = 1; state_reset(&st); continue; }
            for (int64_t i = 0; i < n; ++i) {
                int32_t v = st.touched[i];
                q_ent[q][i] = v;
                q_hop[q][i] = st.hop[v];
                q_pred[q][i] = st.pred[v];
            }
            state_reset(&st);
        }
        state_free(&st);
    }
    reached_off[0] = 0;
    for (int32_t q = 0; q < Q; ++q) reached_off[q + 1] = reached_off[q] + q_cnt[q];
    int64_t N = reached_off[Q];
    *entity = (int32_t *)malloc((size_t)(N > 0 ? N : 1) * sizeof(int32_t));
    *hop = (uint8_t *)malloc((size_t)(N > 0 ? N : 1));
    *pred = (int32_t *)malloc((size_t)(N > 0 ? N : 1) * sizeof(int32_t));
    if (!*entity || !*hop || !*pred) failed = 1;
    for (int32_t q = 0; q < Q && !failed; ++q) {
        memcpy(*entity + reached_off[q], q_ent[q], (size_t)q_cnt[q] * sizeof(int32_t));
        memcpy(*hop + reached_off[q], q_hop[q], (size_t)q_cnt[q]);
        memcpy(*pred + reached_off[q], q_pred[q], (size_t)q_cnt[q] * sizeof(int32_t));
    }
    for (int32_t q = 0; q < Q; ++q) { free(q_ent[q]); free(q_hop[q]); free(q_pred[q]); }
    free(q_ent); free(q_cnt); free(q_hop); free(q_pred);
    free(first); free(ids);
    return failed ? -1 : 0;
}

void oracle_free(void *p) { free(p); }

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * First `max_paths` shortest paths for each (query, target) pair, in the order
 * stated at the top of this file.  count[i] receives the number written for
 * pair i (0 when the target is not reached within k hops; 1 empty path when it
 * is a seed); edges is int32[n_pairs][max_paths][k], -1 padded.
 *
 * Enumeration walks backward from the target over an object index whose triple
 * ids ascend, so candidates come out already in (t_d, t_{d-1}, ..) order; a
 * partial path is extended only through triples whose subject sits one hop
 * closer, and such a subject always has a valid triple of its own (that is
 * what its hop value means), so no branch dies and the walk can stop at
 * max_paths.
 */
typedef struct {
    const int32_t *subj, *rel;
    const int64_t *ofirst;
    const int32_t *oids;
    const uint8_t *hop;
    const uint64_t *mask;
    int32_t k, d, max_paths, found;
    int32_t *out;      /* [max_paths][k] */
    int32_t *stack;    /* [d] edges target-side first */
} path_ctx;

static void extend(path_ctx *c, int32_t v, int level)
{
    if (c->found >= c->max_paths) return;
    if (level == 0) {
        int32_t *row = c->out + (size_t)c->found * c->k;
        for (int i = 0; i < c->d; ++i) row[i] = c->stack[c->d - 1 - i];
        c->found++;
        return;
    }
    for (int64_t j = c->ofirst[v]; j < c->ofirst[v + 1]; ++j) {
        int32_t t = c->oids[j];
        if (c->hop[c->subj[t]] != level - 1) continue;
        if (!relation_allowed(c->mask, c->rel[t])) continue;
        c->stack[c->d - level] = t;
        extend(c, c->subj[t], level - 1);
        if (c->found >= c->max_paths) return;
    }
}

int oracle_paths(int64_t T, int32_t E, const int32_t *subj, const int32_t *rel,
                 const int32_t *obj, int32_t Q, const int64_t *seed_off,
                 const int32_t *seeds, int32_t k, const uint64_t *rel_mask,
                 int32_t rel_words, int64_t n_pairs, const int32_t *pair_query,
                 const int32_t *pair_target, int32_t max_paths,
                 int32_t *count, int32_t *edges)
{
    if (k < 0 || k > 254 || max_paths < 1) return -1;
    int64_t *sfirst = NULL, *ofirst = NULL;
    int32_t *sids = NULL, *oids = NULL;
    if (build_index(subj, T, E, &sfirst, &sids) != 0) return -1;
    if (build_index(obj, T, E, &ofirst, &oids) != 0) { free(sfirst); free(sids); return -1; }
    bfs_state st;
    if (state_init(&st, E) != 0) return -1;
    int32_t *stack = (int32_t *)malloc((size_t)(k > 0 ? k : 1) * sizeof(int32_t));
    for (int64_t i = 0; i < n_pairs * (int64_t)max_paths * k; ++i) edges[i] = -1;
    int32_t cur_q = -1;
    for (int64_t i = 0; i < n_pairs; ++i) {
        int32_t q = pair_query[i], v = pair_target[i];
        count[i] = 0;
        if (q < 0 || q >= Q || v < 0 || v >= E) continue;
        if (q != cur_q) {
            state_reset(&st);
            bfs_one(&st, T, subj, rel, obj, sfirst, sids, 0, seeds + seed_off[q],
                    seed_off[q + 1] - seed_off[q], k,
                    rel_mask ? rel_mask + (size_t)q * rel_words : NULL, NULL);
            cur_q = q;
        }
        if (st.hop[v] == UNREACHED) continue;
        path_ctx c;
        c.subj = subj; c.rel = rel; c.ofirst = ofirst; c.oids = oids;
        c.hop = st.hop;
        c.mask = rel_mask ? rel_mask + (size_t)q * rel_words : NULL;
        c.k = k; c.d = st.hop[v]; c.max_paths = max_paths; c.found = 0;
        c.out = edges + (size_t)i * max_paths * k;
        c.stack = stack;
        extend(&c, v, c.d);
        count[i] = c.found;
    }
    free(stack);
    state_free(&st);
    free(sfirst); free(sids); free(ofirst); free(oids);
    return 0;
}

/*
 * Walk-exact levels, Eq. 4 iterated without a visited set.
 *
 *   level_off : int64[(k+1) * Q + 1]; the list of level h of query q is
 *               entity[level_off[h * Q + q] .. level_off[h * Q + q + 1]),
 *               ascending entity id.  Level 0 = the distinct seeds.
 *   entity    : malloc'ed by the callee (oracle_free).
 */
int oracle_walk_levels(int64_t T, int32_t E, const int32_t *subj, const int32_t *rel,
                       const int32_t *obj, int32_t Q, const int64_t *seed_off,
                       const int32_t *seeds, int32_t k, const uint64_t *rel_mask,
                       int32_t rel_words, int32_t nthreads, int64_t *level_off,
                       int32_t **entity)
{
    if (k < 0 || k > 254 || E <= 0 || T < 0 || Q < 0) return -1;
    for (int64_t i = 0; i < seed_off[Q]; ++i)
        if (seeds[i] < 0 || seeds[i] >= E) return -1;
    int64_t *first = NULL;
    int32_t *ids = NULL;
    if (build_index(subj, T, E, &first, &ids) != 0) return -1;
    const int64_t cells = (int64_t)(k + 1) * Q;
    int32_t **lists = (int32_t **)calloc((size_t)cells + 1, sizeof(*lists));
    int64_t *counts = (int64_t *)calloc((size_t)cells + 1, sizeof(int64_t));
    int failed = !lists || !counts;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
#pragma omp parallel
    {
        /* stamp[v] == mark  <=>  v is in the level being built */
        int32_t *stamp = (int32_t *)calloc((size_t)E, sizeof(int32_t));
        int32_t *cur = (int32_t *)malloc((size_t)E * sizeof(int32_t));
        int32_t *nxt = (int32_t *)malloc((size_t)E * sizeof(int32_t));
        int32_t mark = 0;
        int ok = stamp && cur && nxt && !failed;
#pragma omp for schedule(dynamic, 1)
        for (int32_t q = 0; q < Q; ++q) {
            if (!ok) { failed = 1; continue; }
            const uint64_t *mask = rel_mask ? rel_mask + (size_t)q * rel_words : NULL;
            int64_t n_cur = 0;
            ++mark;
            for (int64_t i = seed_off[q]; i < seed_off[q + 1]; ++i)
                if (stamp[seeds[i]] != mark) { stamp[seeds[i]] = mark; cur[n_cur++] = seeds[i]; }
            for (int h = 0; h <= k; ++h) {
                qsort(cur, (size_t)n_cur, sizeof(int32_t), cmp_i32);
                int32_t *keep = (int32_t *)malloc((size_t)(n_cur > 0 ? n_cur : 1) * sizeof(int32_t));
                if (!keep) { failed = 1; break; }
                memcpy(keep, cur, (size_t)n_cur * sizeof(int32_t));
                lists[(int64_t)h * Q + q] = keep;
                counts[(int64_t)h * Q + q] = n_cur;
                if (h == k) break;
                /* next level: objects of the allowed triples whose subject is in this level */
                int64_t n_nxt = 0;
                ++mark;
                for (int64_t i = 0; i < n_cur; ++i) {
                    int32_t s = cur[i];
                    for (int64_t p = first[s]; p < first[s + 1]; ++p) {
                        int32_t t = ids[p];
                        if (!relation_allowed(mask, rel[t])) continue;
                        int32_t v = obj[t];
                        if (stamp[v] != mark) { stamp[v] = mark; nxt[n_nxt++] = v; }
                    }
                }
                int32_t *swap = cur; cur = nxt; nxt = swap;
                n_cur = n_nxt;
            }
            if (mark > 0x7ffffff0) { memset(stamp, 0, (size_t)E * sizeof(int32_t)); mark = 0; }
        }
        free(stamp); free(cur); free(nxt);
    }
    level_off[0] = 0;
    for (int64_t c = 0; c < cells; ++c) level_off[c + 1] = level_off[c] + counts[c];
    int64_t N = level_off[cells];
    *entity = (int32_t *)malloc((size_t)(N > 0 ? N : 1) * sizeof(int32_t));
    if (!*entity) failed = 1;
    for (int64_t c = 0; c < cells; ++c) {
        if (!failed && lists[c]) memcpy(*entity + level_off[c], lists[c], (size_t)counts[c] * sizeof(int32_t));
        free(lists[c]);
    }
    free(lists); free(counts); free(first); free(ids);
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------
 * Active triples of one hop of one query (Sec. 3.3, Eq. 5-6).
 *
 *   frontier  : the n_frontier entities with q^(h-1)[e] = 1 (any order, may
 *               repeat)
 *   mask      : the query's relation whitelist (rel_words 64-bit words) or NULL
 *   triple    : malloc'ed by the callee (oracle_free): the indices t with
 *               subj[t] in frontier and rel[t] allowed, ordered by
 *               (subj[t], t)
 * Returns the number of triples, or -1.
 */
typedef struct { int32_t s, t; } subject_triple;

static int cmp_subject_triple(const void *a, const void *b)
{
    const subject_triple *x = (const subject_triple *)a, *y = (const subject_triple *)b;
    if (x->s != y->s) return x->s < y->s ? -1 : 1;
    return (x->t > y->t) - (x->t < y->t);
}

int64_t oracle_active_triples(int64_t T, int32_t E, const int32_t *subj, const int32_t *rel,
                              int64_t n_frontier, const int32_t *frontier, const uint64_t *mask,
                              int32_t **triple)
{
    if (E <= 0 || T < 0 || T > 0x7fffffff || n_frontier < 0) return -1;
    uint8_t *in_q = (uint8_t *)calloc((size_t)E, 1);   /* q^(h-1) as an indicator vector */
    if (!in_q) return -1;
    for (int64_t i = 0; i < n_frontier; ++i) {
        if (frontier[i] < 0 || frontier[i] >= E) { free(in_q); return -1; }
        in_q[frontier[i]] = 1;
    }
    int64_t n = 0;
    for (int64_t t = 0; t < T; ++t)                     /* t^(h)[t] = q^(h-1)[s_t], whitelist applied */
        if (in_q[subj[t]] && relation_allowed(mask, rel[t])) ++n;
    subject_triple *act = (subject_triple *)malloc((size_t)(n > 0 ? n : 1) * sizeof(*act));
    *triple = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    if (!act || !*triple) { free(in_q); free(act); free(*triple); *triple = NULL; return -1; }
    int64_t m = 0;
    for (int64_t t = 0; t < T; ++t)
        if (in_q[subj[t]] && relation_allowed(mask, rel[t])) { act[m].s = subj[t]; act[m].t = (int32_t)t; ++m; }
    qsort(act, (size_t)n, sizeof(*act), cmp_subject_triple);
    for (int64_t i = 0; i < n; ++i) (*triple)[i] = act[i].t;
    free(act);
    free(in_q);
    return n;
}

/* ------------------------------------------------------------------------
 * Walks of exactly pair_len[i] allowed triples from a seed of pair_query[i] to
 * pair_target[i] (Sec. 3.3, "complete paths"), first max_paths in
 * (t_d, .., t_1) order.  count[i] = number written (0 when the target does not
 * end such a walk; 1 empty walk for length 0 at a seed); edges is
 * int32[n_pairs][max_paths][k], -1 padded, each walk written seed -> target.
 */
typedef struct {
    const int32_t *subj, *rel;
    const int64_t *ofirst;
    const int32_t *oids;
    const uint8_t *member;   /* [(k+1)][E]: member[h * E + e] = q^(h)[e] */
    int32_t E;
    const uint64_t *mask;
    int32_t k, d, max_paths, found;
    int32_t *out;
    int32_t *stack;
} walk_ctx;

static void extend_walk(walk_ctx *c, int32_t v, int level)
{
    if (c->found >= c->max_paths) return;
    if (level == 0) {                       /* v is a seed: q^(0)[v] = 1 was checked by the caller */
        int32_t *row = c->out + (size_t)c->found * c->k;
        for (int i = 0; i < c->d; ++i) row[i] = c->stack[c->d - 1 - i];
        c->found++;
        return;
    }
    for (int64_t j = c->ofirst[v]; j < c->ofirst[v + 1]; ++j) {
        int32_t t = c->oids[j];
        if (!c->member[(size_t)(level - 1) * c->E + c->subj[t]]) continue;   /* s_t ends a walk of level-1 triples */
        if (!relation_allowed(c->mask, c->rel[t])) continue;
        c->stack[c->d - level] = t;
        extend_walk(c, c->subj[t], level - 1);
        if (c->found >= c->max_paths) return;
    }
}

int oracle_walk_paths(int64_t T, int32_t E, const int32_t *subj, const int32_t *rel,
                      const int32_t *obj, int32_t Q, const int64_t *seed_off,
                      const int32_t *seeds, int32_t k, const uint64_t *rel_mask,
                      int32_t rel_words, int64_t n_pairs, const int32_t *pair_query,
                      const int32_t *pair_target, const int32_t *pair_len, int32_t max_paths,
                      int32_t *count, int32_t *edges)
{
    if (k < 0 || k > 254 || max_paths < 1 || E <= 0) return -1;
    int64_t *ofirst = NULL;
    int32_t *oids = NULL;
    if (build_index(obj, T, E, &ofirst, &oids) != 0) return -1;
    uint8_t *member = (uint8_t *)malloc((size_t)(k + 1) * (size_t)E);
    int32_t *stack = (int32_t *)malloc((size_t)(k > 0 ? k : 1) * sizeof(int32_t));
    if (!member || !stack) { free(member); free(stack); free(ofirst); free(oids); return -1; }
    for (int64_t i = 0; i < n_pairs * (int64_t)max_paths * k; ++i) edges[i] = -1;
    int32_t cur_q = -1;
    for (int64_t i = 0; i < n_pairs; ++i) {
        int32_t q = pair_query[i], v = pair_target[i], d = pair_len[i];
        count[i] = 0;
        if (q < 0 || q >= Q || v < 0 || v >= E || d < 0 || d > k) continue;
        const uint64_t *mask = rel_mask ? rel_mask + (size_t)q * rel_words : NULL;
        if (q != cur_q) {                   /* q^(0) .. q^(k) of this query, Eq. 4 hop by hop */
            memset(member, 0, (size_t)(k + 1) * (size_t)E);
            for (int64_t a = seed_off[q]; a < seed_off[q + 1]; ++a) member[seeds[a]] = 1;
            for (int h = 1; h <= k; ++h)
                for (int64_t t = 0; t < T; ++t)
                    if (member[(size_t)(h - 1) * E + subj[t]] && relation_allowed(mask, rel[t]))
                        member[(size_t)h * E + obj[t]] = 1;
            cur_q = q;
        }
        if (!member[(size_t)d * E + v]) continue;
        walk_ctx c;
        c.subj = subj; c.rel = rel; c.ofirst = ofirst; c.oids = oids; c.member = member; c.E = E;
        c.mask = mask; c.k = k; c.d = d; c.max_paths = max_paths; c.found = 0;
        c.out = edges + (size_t)i * max_paths * k;
        c.stack = stack;
        extend_walk(&c, v, d);
        count[i] = c.found;
    }
    free(member); free(stack); free(ofirst); free(oids);
    return 0;
}
