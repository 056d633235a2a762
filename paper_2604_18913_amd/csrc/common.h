// Internal declarations shared by the HIP translation units of liblogoskg.
// Nothing here is part of the public ABI (see include/logoskg.h).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <array>
#include <cstring>
#include <map>
#include <mutex>
#include <memory>
#include <string>
#include <unordered_map>
#include <vector>

#include "logoskg.h"

static_assert(sizeof(logoskg_build_opts) == 64 && sizeof(logoskg_graph_info) == 120,
              "the ctypes binding mirrors these layouts");

namespace lkg {

// ---------------------------------------------------------------- errors
void set_error(const char *fmt, ...);
const char *get_error();

#define LKG_HIP(call)                                                              \
    do {                                                                           \
        hipError_t e_ = (call);                                                    \
        if (e_ != hipSuccess) {                                                    \
            lkg::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_),  \
                           __FILE__, __LINE__);                                    \
            return (e_ == hipErrorOutOfMemory) ? LOGOSKG_ENOMEM : LOGOSKG_EDEVICE; \
        }                                                                          \
    } while (0)

#define LKG_TRY(call)                         \
    do {                                      \
        logoskg_status s_ = (call);           \
        if (s_ != LOGOSKG_OK) return s_;      \
    } while (0)

// ---------------------------------------------------------------- device memory pool
// k-hop calls need several planes of hundreds of MB each; hipMalloc/hipFree of
// that size cost far more than the kernels, so freed blocks are kept and handed
// out again (exact-size match first, else the smallest block that is large
// enough and at most 2x the request).  A block released behind work that may
// still run (release_after) carries an event recorded on that work's stream: a
// later user on another stream waits for it, a user without a stream waits on
// the host.  Such a block can also be marked as holding zeros only.
class DevPool {
public:
    logoskg_status alloc(void **out, size_t bytes) { return alloc(out, bytes, nullptr, false, nullptr); }
    logoskg_status alloc(void **out, size_t bytes, hipStream_t st, bool *zeroed = nullptr) {
        return alloc(out, bytes, st, true, zeroed);
    }
    void release(void *p);  // usable at once (the caller has waited for the block's last use)
    void release_after(void *const *ptrs, const bool *zeroed, int n, hipStream_t st);
    void trim();  // hipFree everything that is not handed out
    size_t bytes_held() const { return held_; }
    // the caller's allocator instead of hipMalloc / hipFree (set before the first alloc)
    void set_allocator(void *(*alloc_fn)(size_t, void *), void (*free_fn)(void *, void *), void *ctx) {
        alloc_fn_ = alloc_fn;
        free_fn_ = free_fn;
        ctx_ = ctx;
    }
    ~DevPool();

private:
    struct After { hipEvent_t ev; hipStream_t stream; };
    struct Block { void *p; std::shared_ptr<After> after; bool zeroed; };
    logoskg_status alloc(void **out, size_t bytes, hipStream_t st, bool have_stream, bool *zeroed);
    std::multimap<size_t, Block> free_;
    std::unordered_map<void *, size_t> live_;
    std::vector<hipEvent_t> spare_events_;
    size_t held_ = 0;
    void *(*alloc_fn_)(size_t, void *) = nullptr;
    void (*free_fn_)(void *, void *) = nullptr;
    void *ctx_ = nullptr;
    bool raw_alloc(void **p, size_t bytes);
    void raw_free(void *p);
};

// ---------------------------------------------------------------- graph
constexpr int kTailMaxDegree = 32;      // rows up to this degree: one W-lane group per row
constexpr int kPullSegment = 1024;      // longer object rows are cut into segments of this many
                                        // entries, one wavefront each
constexpr int kPushSegment = 64;        // same for the subject rows of a push frontier
constexpr int kDefaultHubMin = 1024;    // object rows from this degree: block-per-row predecessor kernel
                                        // (shorter long rows: one wavefront per row)
constexpr int kDensePullPercent = 60;   // from this share of the triples leaving the frontier a hop is taken as dense
constexpr int kPredPushShare = 4;       // a level whose frontier holds at most T / this triples: long rows resolved from the subject side
constexpr int kGiantSegment = 8192;     // a giant row is walked by one 16-wave block per this many entries
constexpr int kGiantRowMin = 8192;      // hub rows from this size get a 16-wave block in the predecessor pass, smaller ones 4 waves
constexpr int kTileEntities = 64;       // entities per result tile (one wavefront of lanes)
constexpr int kSuperTiles = 16;         // tiles per super tile (1024 entities)
constexpr int kPredTiles = 4;           // tiles per block of the 16-word predecessor kernel
constexpr int kPredGroup = 4;           // lanes (= words) per entity in that kernel
constexpr int kMegaSupers = 64;         // super tiles per mega tile (65536 entities)

struct RowSegment {  // part [begin, min(begin + segment, row end)) of one CSR row
    int32_t row;
    uint32_t begin;
};

struct PullSegment {  // a segment [begin, end) of an object row; multi: the row has several segments
    int32_t row;
    uint32_t begin, end;
    uint32_t multi;
};

struct ShortRow {  // a CSR row with its bounds, so that a kernel needs no look-up in the offsets
    int32_t row;
    uint32_t begin, end;
};

struct RowClasses {             // device work lists over the object rows, split by degree
    ShortRow *tail = nullptr;   // rows with 1 .. kTailMaxDegree entries, descending degree
    PullSegment *seg = nullptr;  // segments of the longer rows, longest rows first
    int32_t *multi = nullptr;   // rows cut into more than one segment
    int32_t *longrows = nullptr;  // rows with more than kTailMaxDegree entries, descending degree
                                  // (per streamed chunk when sharded); the first n_hub of them
                                  // have >= hub_min entries
    int64_t n_tail = 0, n_seg = 0, n_multi = 0, n_hub = 0, n_long = 0;
    int64_t n_giant = 0;  // the first n_giant long rows have >= kGiantRowMin entries
    uint32_t *giant_seg_first = nullptr;  // [n_giant + 1] segments of kGiantSegment entries before every giant row
    int64_t n_giant_segs = 0;
};

// ---------------------------------------------------------------- profiling
enum KernelKind {
    KK_CLEAR = 0, KK_SEED, KK_CENSUS, KK_LIVE, KK_PUSH_TAIL, KK_PUSH_SEG, KK_UPDATE, KK_PULL_TAIL,
    KK_PULL_SEG, KK_PULL_FINISH, KK_COUNT, KK_SCAN, KK_LISTS, KK_PRED, KK_PRED_HUB, KK_PRED_MID, KK_TRAVERSED,
    KK_PATHS, KK_SHARD_COPY, KK_TRIPLES, KK_PRED_WALK, KK_NUM
};
extern const char *const kKernelNames[KK_NUM];

// device counter slots (logoskg_graph::d_ctr); the statistics block holds four
// words per kernel class: rows, edges, lines, items
enum {
    C_NTAIL = 0, C_NSEG = 1, C_NROWS = 2, C_FEDGES = 3, C_NACTIVE = 4, C_ERR = 5,
    C_STATS = 8, C_TOTAL = C_STATS + 4 * KK_NUM  // the pinned host mirror holds one word more
};

struct Profiler {
    bool on = false;        // bracket launches with events
    bool counters = false;  // also count rows / edges / lines inside the kernels
    struct Rec { int kind; hipEvent_t a, b; };
    struct Acc { int64_t launches = 0; double total_ms = 0, max_ms = 0; int64_t units[4] = {0, 0, 0, 0}; };
    std::vector<hipEvent_t> spare;
    std::vector<Rec> recs;
    Acc acc[KK_NUM];
    hipEvent_t cur_a = nullptr;
    int cur_kind = -1;
    void begin(int kind, hipStream_t st);
    void end(hipStream_t st);
    void drain();
    void release();
};

struct ProfScope {  // brackets the launches issued during its lifetime
    Profiler &p; hipStream_t st;
    ProfScope(Profiler &p_, int kind, hipStream_t st_) : p(p_), st(st_) { p.begin(kind, st); }
    ~ProfScope() { p.end(st); }
};

}  // namespace lkg

struct logoskg_graph {
    int device = 0;
    int32_t E = 0, R = 0;
    int64_t Epad = 0;  // E rounded up to a multiple of 64
    int64_t T = 0;
    int hub_min = lkg::kDefaultHubMin;
    int num_shards = 1;

    // subject-sorted CSR (SUB): row s -> objects / relations of its triples
    uint32_t *out_off = nullptr;  // [E+1]
    uint32_t *row_begin = nullptr;    // [E] start of each subject's triples in the edge arrays
                                      // (== out_off when resident; shard-grouped order otherwise)
    uint8_t *shard_of_dev = nullptr;  // [Epad] device copy of the map P (255 = no shard)
    int32_t *out_obj = nullptr;   // [T]
    uint16_t *out_rel = nullptr;  // [T]
    // object-sorted CSR (OBJ): row v -> subjects / relations / edge ids of its triples
    uint32_t *in_off = nullptr;  // [E+1]
    int32_t *in_sub = nullptr;   // [T]
    uint16_t *in_rel = nullptr;  // [T]
    int32_t *in_eid = nullptr;   // [T]
    int32_t *out_eid = nullptr;  // [T] triple index of every entry of the subject-sorted CSR; built on
                                 // first use by the active-triple export
    lkg::RowClasses in_rows;     // static row lists for the pull kernels
    int64_t n_out_rows = 0, n_out_hubs = 0;

    // frontier work lists rebuilt every hop from the level's active bitmap
    int32_t *fr_tail = nullptr;          // [E] frontier rows of degree <= kTailMaxDegree
    lkg::RowSegment *fr_seg = nullptr;   // [fr_seg_cap] segments of the longer frontier rows
    int64_t fr_seg_cap = 0;
    unsigned long long *d_ctr = nullptr;  // device counters (see khop.hip)
    unsigned long long *h_ctr = nullptr;  // pinned host mirror

    std::vector<int32_t> shard_of;  // host copy of the map P (empty when unsharded)
    std::vector<int64_t> shard_triples;
    void *shards = nullptr;  // lkg::ShardSet* when num_shards > 1

    // predecessor pass with 16-word planes: the kernels of the long object rows leave their
    // results in row_pred[row index][query] and the tile kernel moves them into the lists
    int32_t *long_index = nullptr;  // [E] position of a long row's entity in in_rows.longrows
    int32_t *row_pred = nullptr;    // [row_pred_rows][1024]
    int64_t row_pred_rows = 0;
    bool row_pred_tried = false;
    unsigned long long *plane_buf = nullptr;  // plane words of the bit-sliced predecessor pass (same first use)
    size_t plane_buf_bytes = 0;
    hipEvent_t ev_rows = nullptr;

    // the device's helper streams (default priority; shared by all graphs on the device) on which the
    // independent result kernels of a fetch can overlap (LOGOSKG_OVERLAP_FETCH=1)
    hipStream_t side[2] = {nullptr, nullptr};
    hipEvent_t ev_fork = nullptr, ev_join[2] = {nullptr, nullptr};

    lkg::DevPool pool;
    lkg::Profiler prof;
    size_t static_bytes = 0;
    size_t pinned_bytes = 0;
};

struct logoskg_result {
    logoskg_graph *g = nullptr;
    int Q = 0, k = 0, W = 0;
    int64_t Epad = 0;
    bool has_mask = false;
    bool has_counts = false;
    bool walk_exact = false;  // levels hold q^(h) of the plain iteration (no visited filter)
    unsigned long long *visited = nullptr;  // [Epad][W]
    unsigned long long *levels = nullptr;   // [k+1][Epad][W]
    uint32_t *act = nullptr;      // [k+1][Epad/32]: entity has a non-zero line in that level
    unsigned long long *allow = nullptr;    // [R][W] relation -> queries that may follow it
    unsigned long long *live = nullptr;     // [k+1][16] queries whose level-h frontier has an out-edge
    // result-list bookkeeping (count pass): for every query, the number of reached
    // entities below a tile, as three nested exclusive prefixes
    uint16_t *tile_base = nullptr;  // [ntiles][64W]  tiles (64 entities) inside their super tile
    uint32_t *super_base = nullptr; // [nsuper][64W]  super tiles (1024 entities) inside their mega tile
    uint32_t *mega_base = nullptr;  // [nmega][64W]   mega tiles (65536 entities)
    long long *d_reached_off = nullptr;  // [64W+1]
    // active entities (a bit in some level), ascending, and the place of each in that list; the
    // tiles of the count / list / predecessor kernels are cut from it (resident graphs)
    int32_t *tile_ent = nullptr;   // [Epad + 64], -1 behind the last id
    int32_t *cpos = nullptr;       // [Epad], defined for the listed entities
    uint32_t *act_chunk = nullptr; // per 2,048-entity chunk: listed entities before it; then *d_nact
    unsigned long long *d_nact = nullptr;
    long long n_active = -1;       // length of the list (known after the count pass)
    std::vector<int64_t> reached_off;  // host copy [Q+1]
    // the same bookkeeping for one level plane (logoskg_result_level_offsets)
    int level_counted = -1;
    uint16_t *lvl_tile_base = nullptr;
    uint32_t *lvl_super_base = nullptr, *lvl_mega_base = nullptr;
    long long *d_level_off = nullptr;
    std::vector<int64_t> level_off;
    // active triples of one hop for one query range (logoskg_result_triples_offsets)
    int trip_h = -1, trip_q0 = 0, trip_q1 = 0;
    int64_t trip_n = 0;            // entries of level trip_h - 1 over the range
    int64_t trip_total = 0;        // length of the concatenation of their rows of SUB
    int32_t *trip_ent = nullptr;   // [trip_n] those entities, query-major
    long long *trip_off = nullptr; // [trip_n + 1] where every entry's row starts in that concatenation
    long long *trip_chunk_entry = nullptr;  // [chunks + 1] entry behind the first position of every 256-position chunk
    long long *trip_chunk_first = nullptr;  // [chunks + 1] with a whitelist: allowed triples before the chunk
    std::vector<int64_t> trip_off_host;  // [trip_q1 - trip_q0 + 1]
    // chain-count tables of one (query, length) (logoskg_result_walks_count)
    int walk_q = -1, walk_d = -1;
    int64_t walk_total = 0;
    unsigned long long *walk_cnt = nullptr;   // [walk_d + 1][Epad] chains that end in the entity after h triples
    unsigned long long *walk_cum = nullptr;   // [walk_d][T] per hop: running sums inside the rows of OBJ
    unsigned long long *walk_pref = nullptr;  // [E + 1] chains that end in a smaller entity
    std::vector<logoskg_hop_stats> stats;
    mutable hipStream_t last_stream = nullptr;  // stream of the latest call that used the result
    bool complete = false;  // logoskg_khop ran to its end: every non-zero line of the planes has its bit in act
};

namespace lkg {

// device-side helpers -------------------------------------------------------
__device__ __forceinline__ int lane() { return (int)__lane_id(); }

// True when any lane of the caller's aligned W-lane group has `p` set.  Every
// lane of the group must be active at the call.
template <int W>
__device__ __forceinline__ bool group_any(bool p) {
    if constexpr (W == 1) {
        return p;
    } else {
        unsigned long long b = __ballot(p);
        int g0 = lane() & ~(W - 1);
        return ((b >> g0) & ((1ull << W) - 1ull)) != 0ull;
    }
}

__device__ __forceinline__ bool wave_any(bool p) { return __ballot(p) != 0ull; }

__device__ __forceinline__ unsigned long long shfl64(unsigned long long v, int src) {
    int lo = __shfl((int)(unsigned)(v & 0xffffffffull), src);
    int hi = __shfl((int)(unsigned)(v >> 32), src);
    return ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo;
}

__device__ __forceinline__ unsigned long long shfl_xor64(unsigned long long v, int m) {
    int lo = __shfl_xor((int)(unsigned)(v & 0xffffffffull), m);
    int hi = __shfl_xor((int)(unsigned)(v >> 32), m);
    return ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo;
}

__device__ __forceinline__ unsigned long long shfl_up64(unsigned long long v, int d) {
    int lo = __shfl_up((int)(unsigned)(v & 0xffffffffull), d);
    int hi = __shfl_up((int)(unsigned)(v >> 32), d);
    return ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo;
}

// exclusive prefix sum over the lanes of a wavefront; `total` receives the sum
__device__ __forceinline__ int wave_excl_scan(int v, int &total) {
    int x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int y = __shfl_up(x, d);
        if (lane() >= d) x += y;
    }
    total = __shfl(x, 63);
    return x - v;
}

__device__ __forceinline__ long long wave_sum(long long v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += (long long)shfl_xor64((unsigned long long)v, m);
    return v;
}

// 64x64 bit-matrix transpose across a wavefront: on entry lane r holds row r
// (bit c = M[r][c]); on return lane c holds column c (bit r = M[r][c]).  Six
// butterfly steps; in step j the off-diagonal j x j blocks of every 2j x 2j block
// change places.
__device__ __forceinline__ unsigned long long transpose64(unsigned long long x) {
    const unsigned long long lowmask[6] = {0x00000000FFFFFFFFull, 0x0000FFFF0000FFFFull, 0x00FF00FF00FF00FFull,
                                           0x0F0F0F0F0F0F0F0Full, 0x3333333333333333ull, 0x5555555555555555ull};
#pragma unroll
    for (int s = 0; s < 6; ++s) {
        const int j = 32 >> s;
        const unsigned long long m = lowmask[s];
        unsigned long long y = shfl_xor64(x, j);
        if (lane() & j) x = ((y >> j) & m) | (x & ~m);
        else x = (x & m) | ((y & m) << j);
    }
    return x;
}

// bits of word w (0..W-1) that belong to queries < Q
__device__ __forceinline__ unsigned long long query_bits(int Q, int w) {
    int lo = w * 64;
    if (Q >= lo + 64) return ~0ull;
    if (Q <= lo) return 0ull;
    return (1ull << (Q - lo)) - 1ull;
}

inline int words_for_queries(int Q) { return Q <= 64 ? 1 : (Q <= 256 ? 4 : 16); }

// arguments of the list / predecessor kernels (result.hip)
struct FillArgs {
    int32_t E;
    int Q, k, q0, q1, hub_min;
    long long ntiles;
    const int32_t *tile_ent;  // the tiles' entities (list of active entities) or NULL: tile i = ids 64 i ..
    const int32_t *cpos;      // entity -> place in tile_ent (garbage for entities not in the list), or NULL
    long long n_listed;       // length of tile_ent's list
    unsigned long long *plane_buf;  // bit-sliced plane words between k_pred_walk and k_pred_emit, or NULL
    size_t plane_buf_bytes;
    int emit_eid_cap, emit_line_cap;  // capacities of k_pred_emit's two LDS tables (entries / lines)
    uint32_t push_levels;   // bit h: level h of the long rows is resolved from the subject side (k_pred_push), the row
                            // kernels leave it out; host_graph / host_result are what the host code needs for that
    void *host_graph, *host_result;
    uint32_t dense_levels;  // bit h: nearly every triple leaves level h - 1, so the predecessor kernels gather the
                            // line of every entry of a row at level h without asking for its frontier bit first
    void *ev_rows;                    // host side: event between the block-per-row kernel and the list writer
    long long tile_begin, tile_count;  // tiles this predecessor launch covers
    long long plane;   // words per plane
    long long actw;    // uint32 words per active bitmap
    const unsigned long long *visited, *levels, *allow;
    const uint32_t *act;
    const uint16_t *tile_base;
    const uint32_t *super_base, *mega_base;
    const long long *reached_off;
    const uint32_t *in_off;
    const int32_t *in_sub, *in_eid;
    const uint16_t *in_rel;
    const int32_t *rows;  // long object rows of this predecessor launch
    long long row_base;   // position of rows[0] in the graph's list of long rows
    const int32_t *long_index;  // entity -> position in that list (long rows only)
    int32_t *row_pred;    // [rows of the launch][1024] results of the row kernels, or NULL: they
                          // write the lists themselves
    int32_t *entity;
    uint8_t *hop;
    int32_t *pred;
    unsigned long long *stats_pred, *stats_hub, *stats_mid;  // rows / edges / lines counters or NULL
    int fuse_lists;  // the 16-word tile kernel also writes the entity and hop lists
    long long n_giant_rows;  // hub rows of the launch that get a 16-wave block (the first ones); -1 = all
    const uint32_t *giant_seg_first;  // [n_giant_rows + 1] or NULL: a block per giant row instead of one per segment
    long long n_giant_segs;
};

logoskg_status build_csr_on_device(logoskg_graph *g, const int32_t *subj, const int32_t *rel, const int32_t *obj,
                                   std::vector<uint32_t> *ooff, std::vector<uint32_t> *ioff);
struct TripleSorter;  // the triple list on the device during a sharded build (build_device.hip)
logoskg_status sorter_create(logoskg_graph *g, const int32_t *subj, const int32_t *rel, const int32_t *obj,
                             TripleSorter **out);
void sorter_destroy(TripleSorter *s);
logoskg_status sorter_offsets(TripleSorter *s, bool by_object, std::vector<uint32_t> *off);
logoskg_status sorter_subject_order(TripleSorter *s, const uint32_t *d_row_begin, int32_t *h_obj, uint16_t *h_rel);
logoskg_status sorter_object_order(TripleSorter *s, int32_t *h_sub, uint16_t *h_rel, int32_t *h_eid);
logoskg_status ensure_out_eid(logoskg_graph *g, hipStream_t st);
void drop_walk_tables(logoskg_result *r);
void launch_lists(Profiler &prof, const FillArgs &a, int W, hipStream_t st);
void launch_pred(Profiler &prof, const FillArgs &a, int W, long long n_hub_rows, long long n_other_rows, bool mask,
                 hipStream_t st_tiles, hipStream_t st_rows);
logoskg_status sharded_pred(logoskg_graph *g, FillArgs *a, int W, bool mask, hipStream_t st);
long long max_chunk_rows(const logoskg_graph *g);
logoskg_status census(logoskg_graph *g, logoskg_result *r, int h, int shard, bool write_lists, hipStream_t st);
// (prof_kind: the kernel class the launch is timed under)
logoskg_status census_lists(logoskg_graph *g, logoskg_result *r, int h, int shard, hipStream_t st,
                            int prof_kind = KK_CENSUS);
void launch_push_lists(logoskg_graph *g, logoskg_result *r, int h, const unsigned long long *hc,
                       const int32_t *obj, const uint16_t *rel, bool update, const int32_t *list_tail,
                       const lkg::RowSegment *list_seg, const unsigned long long *ctr, hipStream_t st);
void shard_info(const logoskg_graph *g, logoskg_graph_info *o);
bool shard_out_arrays(const logoskg_graph *g, const int32_t **obj, const uint16_t **rel);
bool shard_in_arrays(const logoskg_graph *g, const int32_t **sub, const uint16_t **rel, const int32_t **eid);
void launch_pull_range(logoskg_graph *g, logoskg_result *r, int h, const RowClasses &rc, const int32_t *in_sub,
                       const uint16_t *in_rel, const unsigned long long *hc, bool want_stats, bool first,
                       hipStream_t st);
logoskg_status run_sharded_hop(logoskg_graph *g, logoskg_result *r, int h, bool pull, bool want_stats,
                               const unsigned long long *hc, hipStream_t st, logoskg_hop_stats *hs);
void free_shards(logoskg_graph *g);
// build.hip: per-device helper streams shared by all graphs (which = 0, 1: fetch side work; 2: shard copies)
hipStream_t helper_stream(int device, int which);
logoskg_status build_shards(logoskg_graph *g, const int32_t *subj, const int32_t *rel,
                            const int32_t *obj, const logoskg_build_opts *opts, const std::vector<uint32_t> &ooff,
                            TripleSorter *sorter);

}  // namespace lkg
