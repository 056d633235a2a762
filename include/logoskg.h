/*
 * logoskg.h - C ABI of the MI355X (gfx950) batched k-hop knowledge-graph
 * retrieval library.
 *
 * The operations follow the LogosKG paper's problem statement (Sec. 3.1: a KG
 * is a set of triples (s, r, o); a query is a set of entities; k-hop retrieval
 * returns every entity reachable from a seed within k relational steps) and
 * its incidence-matrix formulation (Sec. 3.2-3.3): the column index t of SUB /
 * row index t of OBJ and REL (Eq. 1-3) is the position of a triple in the
 * arrays given to logoskg_build and is the triple's EDGE ID everywhere below;
 * one hop is q.SUB.OBJ over the boolean semiring (Eq. 4), with the active
 * triples t = q.SUB (Eq. 5-6) additionally filtered by a per-query relation
 * whitelist before the OBJ product.
 *
 * Conventions
 *   - Every call returns a logoskg_status; LOGOSKG_OK is 0.  A short text for
 *     the last failure on the calling thread is kept by logoskg_last_error().
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HBM of the
 *     graph's GPU.  Caller buffers are borrowed for the duration of the call.
 *   - Entity ids are int32 in [0, num_entities), relation ids int32 in
 *     [0, num_relations), num_relations <= 65536, num_triples < 2^31.
 *   - A graph handle runs one call at a time (not thread safe).  Stream
 *     arguments are hipStream_t passed as void* (NULL = the default stream).
 */
#ifndef LOGOSKG_H
#define LOGOSKG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct logoskg_graph logoskg_graph;   /* owns device (and pinned host) memory  */
typedef struct logoskg_result logoskg_result; /* owns the device state of one k-hop call */

typedef enum {
    LOGOSKG_OK = 0,
    LOGOSKG_EINVAL = 1,    /* null pointer, id out of range, k outside [0,254], bad sizes */
    LOGOSKG_ENOMEM = 2,    /* host or device allocation failed, or budget below one shard  */
    LOGOSKG_EDEVICE = 3,   /* a HIP call failed (text in logoskg_last_error)               */
    LOGOSKG_ERANGE = 4,    /* a caller-provided capacity is too small                      */
    LOGOSKG_EINTERNAL = 5,
    LOGOSKG_EIO = 6        /* a shard file could not be written or read                    */
} logoskg_status;

#define LOGOSKG_MAX_QUERIES 1024 /* queries per logoskg_khop call: 16 uint64 words per entity.
                                    A larger workload (the 4,096 queries of the hub-heavy
                                    benchmark shape) is run by the caller as consecutive calls on
                                    slices of its queries, each slice's seed_off rebased to 0:
                                    queries are independent, so the results concatenate.        */
#define LOGOSKG_MAX_K 254
#define LOGOSKG_MAX_PATHS 16

/* ------------------------------------------------------------------ build */

typedef struct {
    uint32_t struct_size;            /* sizeof(logoskg_build_opts); zero the rest for defaults  */
    int32_t device;                  /* HIP device ordinal                                      */
    int32_t num_shards;              /* 0 or 1: whole graph resident in HBM.  >1: degree-aware
                                        partition of the subjects (Sec. 3.4) into this many
                                        shards kept in pinned host memory and cached in HBM      */
    int32_t max_resident_shards;     /* cache capacity in sub-graphs (the paper's n); 0 = no cap.
                                        The cache holds the shards (visited by push hops) and
                                        the sub-graphs by object range that pull hops visit
                                        (logoskg_graph_info.num_object_ranges of them), one per
                                        slot, 6 bytes per triple either way                      */
    uint64_t hbm_shard_budget_bytes; /* cache capacity in bytes; 0 = no cap                      */
    int32_t hub_min_degree;          /* rows with at least this many edges take the
                                        block-per-row kernels; 0 = default (1024).  Never changes
                                        results.                                                 */
    int32_t host_build;              /* 0: the two sorts of the triple list run on the GPU (the
                                        triples are copied to HBM first; a sharded graph's sorted
                                        arrays are copied back to pinned host memory).  1: counting
                                        sorts on the host.  Both give the same arrays.           */
    const char *shard_dir;           /* NULL: the shards stay in pinned host memory.  Else a
                                        directory (it must exist): every shard is written to
                                        <shard_dir>/shard_<i>.lkg at build and read from there
                                        when the cache misses (Sec. 3.4: sub-graphs on disk, the
                                        tau_io of a miss), through one pinned staging buffer per
                                        cache slot.  The files are left in place at
                                        logoskg_graph_free.  Only with num_shards > 1.           */
    /* Optional allocator for the memory the calls on this graph take and give back (bit planes,
     * bitmaps, count tables, list bookkeeping, workspaces: the graph's pool), so that a harness
     * can hand out memory it owns (a framework's caching allocator).  dev_alloc returns device
     * memory on `device`, at least 256-byte aligned, or NULL (reported as LOGOSKG_ENOMEM);
     * dev_free takes back exactly what dev_alloc returned, from logoskg_graph_free at the latest.
     * Both run on the calling thread, never inside a kernel launch sequence that a stream
     * capture could see.  Both NULL (or a struct_size that ends before them): hipMalloc /
     * hipFree.  The graph's own arrays (sorted triples, work lists, cache slots) are allocated
     * with hipMalloc at build either way.                                                      */
    void *(*dev_alloc)(size_t bytes, void *alloc_ctx);
    void (*dev_free)(void *ptr, void *alloc_ctx);
    void *alloc_ctx;
} logoskg_build_opts;

/*
 * Sec. 3.2, Eq. 1-3: turn the triple list into the device form of SUB, OBJ and
 * REL - a subject-sorted CSR (objects and relation ids of each subject's
 * triples) and an object-sorted CSR (subjects, relation ids and edge ids of
 * each object's triples); both sorts are stable, so edge ids ascend inside a
 * row.  Rows are split by degree into a group-per-row class and a
 * block-per-row (hub) class.  With num_shards > 1 the subjects are also
 * assigned to shards by descending degree, each to the currently lightest
 * shard (Sec. 3.4, degree-aware partitioning; map P).
 *
 * subj/rel/obj: host, int32[num_triples].  Duplicated triples are legal (the
 * smaller edge id wins ties); ids are validated (LOGOSKG_EINVAL).
 * *out receives a handle to be released with logoskg_graph_free.
 */
logoskg_status logoskg_build(const int32_t *subj, const int32_t *rel, const int32_t *obj,
                             int64_t num_triples, int32_t num_entities, int32_t num_relations,
                             const logoskg_build_opts *opts, logoskg_graph **out);

void logoskg_graph_free(logoskg_graph *g);

typedef struct {
    int64_t num_triples;
    int32_t num_entities, num_relations;
    int32_t num_shards;
    int32_t hub_min_degree;
    int64_t num_out_rows, num_out_hubs; /* subjects with >= 1 triple / in the hub class */
    int64_t num_in_rows, num_in_hubs;   /* objects  with >= 1 triple / in the hub class */
    int64_t device_bytes;               /* HBM held by the graph (CSR, lists, shard cache) */
    int64_t pinned_host_bytes;          /* pinned host memory held by the shards            */
    int64_t shard_loads, shard_evictions, shard_hits; /* cache counters since build (Sec. 3.4) */
    int64_t shard_bytes_h2d;
    int64_t shard_bytes_disk;           /* bytes read from the shard files (0 without shard_dir) */
    int32_t num_object_ranges;          /* sharded graphs: sub-graphs by object range that pull hops visit
                                           (units of the same cache as the shards); 0 when resident  */
    int32_t cache_slots;                /* sub-graphs the cache can hold at once (0 when resident)       */
} logoskg_graph_info;

logoskg_status logoskg_graph_get_info(const logoskg_graph *g, logoskg_graph_info *out);

/*
 * Per-kernel timing for measurement runs.  enable = 1: every kernel launch of
 * the library is bracketed by HIP events on the caller's stream.  enable = 2:
 * in addition the pull and result kernels count the rows, CSR entries and
 * bit-plane lines they actually touch (a few atomics per wavefront, so time
 * with 1 and count with 2).  logoskg_profile_read drains the finished events:
 * out[i] describes kernel class i (at most `capacity` entries are written,
 * *n_out receives how many exist) and the accumulators restart from zero.
 */
typedef struct {
    char name[32];
    int64_t launches;
    double total_ms, max_ms;
    int64_t rows;   /* rows (entities) the launches worked on                  */
    int64_t edges;  /* CSR entries read                                        */
    int64_t lines;  /* W-word bit-plane lines gathered / updated through edges */
    int64_t items;  /* kernel specific: list entries written, words streamed   */
} logoskg_kernel_profile;

logoskg_status logoskg_profile_enable(logoskg_graph *g, int32_t enable);
logoskg_status logoskg_profile_read(logoskg_graph *g, logoskg_kernel_profile *out, int32_t capacity,
                                    int32_t *n_out);

/*
 * Measurement aid, no part of the retrieval: the line gathers of a dense pull
 * hop (Eq. 4 evaluated per object row on a batch of 1,024 queries) and nothing
 * else.  For every entry of the object-sorted CSR of a resident graph, in
 * order, the 128-byte line lines[16 * subject .. 16 * subject + 15] is loaded
 * with the access shape of the pull kernels and ORed into out16; no row bounds,
 * visited or level lines are touched and nothing else is written, so the time of
 * this call is what the gathers of such a hop cost on this GPU and graph.
 *   lines : device, [num_entities][16] uint64 (any content)
 *   out16 : device, 16 uint64 (the OR of the lines of all subjects, for checks)
 * Asynchronous on `stream`.  LOGOSKG_EINVAL on a sharded graph.
 */
logoskg_status logoskg_probe_gather(const logoskg_graph *g, const uint64_t *lines, uint64_t *out16,
                                    void *stream);

/* Sec. 3.4 metadata map P: shard of each subject entity (-1 for entities that are
 * never a subject), and the number of triples per shard.  host outputs; either
 * may be NULL. */
logoskg_status logoskg_graph_partition(const logoskg_graph *g, int32_t *shard_of_entity /*[E]*/,
                                       int64_t *triples_per_shard /*[num_shards]*/);

/*
 * Sec. 3.4 "On-demand caching", batch processing: queries are grouped by the
 * sub-graphs they need, processed jointly and the results restored afterwards.
 * The need of a query is taken from its seeds through the map P (the sub-graphs
 * its first hop loads).  order[i] = index of the query to run i-th: queries are
 * sorted by their ascending list of distinct shard ids, compared
 * lexicographically (a query none of whose seeds is a subject comes first);
 * queries with the same list keep their input order.  The caller cuts `order`
 * into batches, builds the seed lists of each batch in that order and puts the
 * results back with the same permutation.  seed_off (int64[num_queries + 1]),
 * seeds and order (int32[num_queries]) are HOST arrays; nothing runs on the GPU.
 * On an unsharded graph the order is the identity.
 */
logoskg_status logoskg_schedule_queries(const logoskg_graph *g, const int64_t *seed_off, const int32_t *seeds,
                                        int64_t num_queries, int32_t *order);

/*
 * Sec. 3.4, cache warm-up across batches: asks the shard cache for the given
 * shards, in the given order, as a hop of a batch would (a resident shard is a
 * hit, a missing one is loaded into an empty or the least recently used slot and
 * counted as a load).  The copies run on the graph's copy stream, so a caller who
 * knows the next batch - its seeds' shards through logoskg_graph_partition, or
 * the order of logoskg_schedule_queries - can issue them while the current
 * batch's lists are written.  shards: host int32[n], each in [0, num_shards); at
 * most as many as there are cache slots are useful.  No-op on an unsharded graph.
 */
logoskg_status logoskg_prefetch_shards(logoskg_graph *g, const int32_t *shards, int32_t n);

/* ------------------------------------------------------------------- khop */

#define LOGOSKG_DIR_AUTO 0u       /* choose push or pull per hop from the frontier's edge count */
#define LOGOSKG_DIR_PUSH 1u       /* always expand from the frontier's subject rows             */
#define LOGOSKG_DIR_PULL 2u       /* always gather over the object rows                         */
#define LOGOSKG_DIR_MASK 3u
#define LOGOSKG_NO_COUNTS 4u      /* skip the per-query reached counts (planes only)            */
#define LOGOSKG_WALK_EXACT 8u     /* Eq. 4 iterated literally, without the visited set: level h
                                     = the entities that end a walk of exactly h allowed triples
                                     (an entity may be in several levels).  The reached set and
                                     its offsets are unchanged; hop, pred_edge and paths are not
                                     defined for such a result (LOGOSKG_EINVAL): read the levels
                                     with logoskg_result_level_offsets / _level_fetch.          */

typedef struct {
    uint32_t struct_size;     /* sizeof(logoskg_query_batch)                                  */
    int32_t num_queries;      /* Q in [1, LOGOSKG_MAX_QUERIES]                                */
    int64_t num_seeds;        /* length of seeds                                               */
    const int64_t *seed_off;  /* device int64[Q+1], ascending, seed_off[0]=0, [Q]=num_seeds    */
    const int32_t *seeds;     /* device int32[num_seeds]; repeats inside a query collapse      */
    int32_t k;                /* hops, 0..LOGOSKG_MAX_K                                        */
    uint32_t flags;           /* LOGOSKG_DIR_* | LOGOSKG_NO_COUNTS                             */
    const uint64_t *rel_mask; /* device uint64[Q][ceil(R/64)]: bit r%64 of word r/64 set when
                                 the query may follow relation r; NULL = every relation        */
    void *stream;             /* hipStream_t                                                   */
} logoskg_query_batch;

/*
 * Sec. 3.1 / 3.3 (Eq. 4-6; Algorithm 1 when the graph is sharded): batched
 * k-hop retrieval.  For query j and entity v the result records
 *   hop_j(v)  = the least h <= k at which v is set in q_j^(h) (0 for seeds), and
 *   the reached set {v : hop_j(v) defined}.
 * Device state: one bit plane per hop level, entity-major, W = 1, 4 or 16
 * uint64 words per entity for up to 64 / 256 / 1024 queries (bit j%64 of word j/64 belongs to query j), plus the
 * OR of all levels ("visited").  Unless LOGOSKG_NO_COUNTS is set the per-query
 * reached counts are computed too.  The call returns after the stream has been
 * synchronised; bad seed ids or offsets are detected on the device and
 * reported as LOGOSKG_EINVAL.
 */
logoskg_status logoskg_khop(logoskg_graph *g, const logoskg_query_batch *batch,
                            logoskg_result **out);

typedef struct {
    int32_t num_queries, k;
    int32_t words_per_entity;    /* W */
    int32_t num_levels;          /* k + 1 */
    int64_t padded_entities;     /* rows per plane (num_entities rounded up to 64) */
    const uint64_t *visited;     /* device uint64[padded_entities][W]              */
    const uint64_t *levels;      /* device uint64[k+1][padded_entities][W]         */
    int64_t total_reached;       /* sum over queries (-1 with LOGOSKG_NO_COUNTS)   */
} logoskg_result_info;

logoskg_status logoskg_result_get_info(const logoskg_result *r, logoskg_result_info *out);

typedef struct {
    int32_t direction;        /* LOGOSKG_DIR_PUSH or LOGOSKG_DIR_PULL; 0 = hop not run (empty frontier) */
    int32_t shards_touched;   /* sub-graphs the hop visited: shards with an active subject (push) or
                                 object ranges (pull); 1 for resident graphs                            */
    int64_t active_rows;      /* subjects in the frontier with >= 1 triple                              */
    int64_t frontier_edges;   /* sum of their out-degrees                                               */
    int64_t rows_scanned;     /* pull: object rows visited that were not already complete (profiling on) */
    int64_t edges_scanned;    /* CSR entries read by the expansion kernels (pull: profiling on)          */
    int64_t lines_gathered;   /* pull: frontier lines read (profiling on); push: visited lines read      */
    int64_t entities_reached; /* entities with at least one new query bit at this hop                   */
} logoskg_hop_stats;

/* host out[k]; entry h-1 describes hop h. */
logoskg_status logoskg_result_hop_stats(const logoskg_result *r, logoskg_hop_stats *out);

/* host reached_off[Q+1]: prefix sums of the per-query reached counts. */
logoskg_status logoskg_result_offsets(const logoskg_result *r, int64_t *reached_off);

/*
 * Per-query result lists for queries [q_begin, q_end): query-major, ascending
 * entity id inside a query; position i of query q is
 * reached_off[q] - reached_off[q_begin] + i.  entity, hop and pred_edge are
 * device buffers of reached_off[q_end] - reached_off[q_begin] elements
 * (capacity is checked: LOGOSKG_ERANGE); hop and pred_edge may be NULL.
 *   pred_edge = the smallest edge id t with o_t = v, r_t allowed for the query
 *   and hop(s_t) = hop(v) - 1 (the active triple of Eq. 5-7 that reaches v
 *   first in edge-id order); -1 for seeds.
 * Asynchronous on `stream`: the kernels of a fetch run in turn on it.  (With
 * LOGOSKG_OVERLAP_FETCH=1 in the environment the independent ones run on helper
 * streams - made once per device, shared by all graphs on it, kept until the
 * process ends - and join `stream` before the call returns; measured, no gain.)  The
 * first call on a graph that asks for pred_edge with more than 256 queries
 * allocates a buffer of 4 KiB per object row of more than 32 entries (not
 * above 8 GiB; freed with the graph) and, on a resident graph, 4 bytes per
 * triple for the triple index of every entry of SUB.  On a sharded graph pred_edge streams the
 * object-sorted triples from pinned host memory.
 */
logoskg_status logoskg_result_fetch(logoskg_result *r, int32_t q_begin, int32_t q_end,
                                    int64_t capacity, int32_t *entity, uint8_t *hop,
                                    int32_t *pred_edge, void *stream);

/*
 * Level h of every query, h in [0, k] (Sec. 3.3, the support of q^(h)): with the
 * default search the entities whose minimum hop is exactly h ("at a specific
 * hop"), with LOGOSKG_WALK_EXACT the ends of the walks of exactly h triples.
 * logoskg_result_level_offsets counts the level (level_off: host int64[Q+1],
 * synchronises `stream`); logoskg_result_level_fetch then writes the lists of
 * the queries [q_begin, q_end) of that same level, query-major and ascending in
 * entity id, to the device buffer `entity` (capacity checked: LOGOSKG_ERANGE),
 * asynchronously on `stream`.  One level at a time per result.
 */
logoskg_status logoskg_result_level_offsets(logoskg_result *r, int32_t h, int64_t *level_off,
                                            void *stream);
logoskg_status logoskg_result_level_fetch(logoskg_result *r, int32_t h, int32_t q_begin, int32_t q_end,
                                          int64_t capacity, int32_t *entity, void *stream);

/*
 * Active triples of hop h, h in [1, k] (Sec. 3.3 "Path reconstruction", Eq. 5-7):
 * T_h of query q holds the triples t whose subject is in level h-1 of q (the
 * support of q^(h-1): minimum hop h-1 with the default search, walks of h-1
 * triples with LOGOSKG_WALK_EXACT) and whose relation the query's whitelist
 * allows.  Lists are query-major; inside a query they follow SUB's rows:
 * ascending subject, ascending triple index inside a subject.
 * logoskg_result_triples_offsets prepares the queries [q_begin, q_end) and
 * returns triple_off (host int64[q_end - q_begin + 1], prefix sums of |T_h|;
 * synchronises `stream`); logoskg_result_triples_fetch, called with the same
 * h and range, then writes for position triple_off[q - q_begin] + i the triple
 * index and its components (s_h, r_h, e_h of Eq. 7) to the device buffers
 * triple / subject / relation / object (each int32[capacity] or NULL;
 * capacity checked: LOGOSKG_ERANGE), asynchronously on `stream`.  The calls
 * count level h-1 (they replace the level counted by
 * logoskg_result_level_offsets) and keep the level's entity list, one int64
 * per entry and one or two int64 per 256 triples in device memory until the
 * result is freed or another range is prepared.  The first call on a graph
 * builds the triple indices of SUB's rows (4 bytes per triple in device
 * memory, freed with the graph).  On a sharded graph the kernels read SUB's
 * rows from the pinned host copy of the shards in place; shards kept in files
 * (shard_dir) have no such copy: LOGOSKG_EINVAL.
 */
logoskg_status logoskg_result_triples_offsets(logoskg_result *r, int32_t h, int32_t q_begin, int32_t q_end,
                                              int64_t *triple_off, void *stream);
logoskg_status logoskg_result_triples_fetch(logoskg_result *r, int32_t h, int32_t q_begin, int32_t q_end,
                                            int64_t capacity, int32_t *triple, int32_t *subject,
                                            int32_t *relation, int32_t *object, void *stream);

/*
 * traversed[q][h-1] = number of triples whose subject has hop h-1 for query q
 * (the triples hop h inspects, whatever their relation): the numerator of the
 * per-query "traversed edges per second" figure.  device int64[Q][k].
 */
logoskg_status logoskg_result_traversed(logoskg_result *r, int64_t *traversed, void *stream);

void logoskg_result_free(logoskg_result *r);

/* ------------------------------------------------------------------ paths */

/*
 * Sec. 3.3 "Path reconstruction" (Eq. 5-7), restricted to shortest paths: for
 * pair i = (query_idx[i], target[i]) with hop(target) = d, the paths are the
 * edge-id sequences (t_1..t_d) whose triples chain from a seed to the target
 * through subjects at hops 0..d-1 with allowed relations.  They are ordered
 * lexicographically by (t_d, t_{d-1}, .., t_1) and the first max_paths
 * (1..LOGOSKG_MAX_PATHS) are written seed -> target into
 * path_edges[i][p][0..d), the rest of each row of k entries is -1.
 * path_count[i] = number written (0 if the target is not reached; 1 empty
 * path if it is a seed).  All four arrays are device memory; path_edges is
 * int32[n_pairs][max_paths][k].  On a sharded graph the kernel reads the
 * object rows it walks from pinned host memory, in place.  The call takes its
 * working memory from the graph's pool and returns after `stream` has been
 * synchronised.
 */
logoskg_status logoskg_paths(logoskg_graph *g, const logoskg_result *r, const int32_t *query_idx,
                             const int32_t *target, int64_t n_pairs, int32_t max_paths,
                             int32_t *path_count, int32_t *path_edges, void *stream);

/*
 * Sec. 3.3, complete paths of the plain iteration: for pair i = (query_idx[i],
 * target[i], length[i]) the walks are the sequences (t_1..t_d), d = length[i]
 * in [0, k], of allowed triples that chain from a seed of the query to the
 * target (o_{t_j} = s_{t_{j+1}}; entities may repeat).  Same order
 * ((t_d, .., t_1) lexicographic), limit, layout and memory rules as
 * logoskg_paths; path_count[i] = 0 when the target ends no such walk, 1 empty
 * walk for length 0 at a seed.  `r` must come from a LOGOSKG_WALK_EXACT search
 * (LOGOSKG_EINVAL otherwise); with the targets of logoskg_result_level_fetch(k)
 * and length k this lists every complete path of length k.
 */
logoskg_status logoskg_walks(logoskg_graph *g, const logoskg_result *r, const int32_t *query_idx,
                             const int32_t *target, const int32_t *length, int64_t n_pairs,
                             int32_t max_paths, int32_t *path_count, int32_t *path_edges, void *stream);

/*
 * Sec. 3.3, complete paths in bulk (Eq. 5-7 chained over the hops): EVERY chain
 * (t_1, .., t_d), d = length, of allowed triples of one query with s_{t_1} a
 * seed, o_{t_i} = s_{t_{i+1}} and s_{t_i} in level i-1 -- on a
 * LOGOSKG_WALK_EXACT result all walks of d triples from a seed (the complete
 * paths of length d), on a minimum-hop result all shortest paths to the
 * entities at hop d -- with no bound per target.  The chains are numbered
 * 0 .. total-1: by target (ascending entity id), the chains of one target in
 * the order of logoskg_paths / logoskg_walks ((t_d, .., t_1) lexicographic).
 *
 * logoskg_result_walks_count builds the count tables of (query, length) on the
 * device (8 bytes x (length x num_triples + (length + 2) x padded_entities)
 * from the graph's pool, kept until the result is freed or another
 * (query, length) is counted), returns the number of chains in *total (host)
 * and synchronises `stream`.  LOGOSKG_ERANGE when 2^56 or more chains end in
 * one entity.  logoskg_result_walks_fetch writes the chains
 * [first, first + count) of the (query, length) counted last: walk_edges is
 * device int32[count][length], each chain written seed -> target; walk_target
 * (device int32[count], may be NULL when length > 0) receives the entity each
 * chain ends in.  Asynchronous on `stream`; any page can be asked for in any
 * order, so a caller with a fixed buffer pages through the whole list.  On a
 * sharded graph the kernels read the object-sorted triples from pinned host
 * memory in place.
 */
logoskg_status logoskg_result_walks_count(logoskg_result *r, int32_t query, int32_t length, int64_t *total,
                                          void *stream);
logoskg_status logoskg_result_walks_fetch(logoskg_result *r, int32_t query, int32_t length, int64_t first,
                                          int64_t count, int32_t *walk_edges, int32_t *walk_target, void *stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): logoskg_paths with the
 * same arguments, results and order, whose only working memory - three int32
 * depth-first stacks of n_pairs * max(k, 1) entries - lives in an array that is
 * part of the library's device image (12 MiB per GPU, held until the process
 * ends) instead of a block of the graph's pool.  The call allocates and frees
 * nothing on the device and does not synchronise: it is asynchronous on
 * `stream`.  n_pairs * max(k, 1) above LOGOSKG_STATIC_PATH_SLOTS is refused
 * with LOGOSKG_ERANGE (nothing is launched).  Every call on a GPU uses that
 * GPU's one array: calls that overlap on one GPU (two streams, two threads,
 * two graphs) race; issue them on one stream or wait in between.  Nothing
 * needs clearing between calls (a stack entry is written before it is read).
 */
#define LOGOSKG_STATIC_PATH_SLOTS (1ll << 20)
logoskg_status logoskg_paths_static(logoskg_graph *g, const logoskg_result *r, const int32_t *query_idx,
                                    const int32_t *target, int64_t n_pairs, int32_t max_paths,
                                    int32_t *path_count, int32_t *path_edges, void *stream);

const char *logoskg_last_error(void);
const char *logoskg_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LOGOSKG_H */
