// Graphs larger than the HBM budget (paper Sec. 3.4, Algorithm 1).
//
// Degree-aware partitioning: the subjects are sorted by (out-degree descending,
// id ascending) and each is given to the shard that holds the fewest triples so
// far (ties: lowest shard index), so high-degree subjects spread evenly and all
// triples of a subject stay together.  The map P (shard of each subject) lives
// in HBM; the triples (objects, relations) are kept in pinned host memory,
// grouped by shard, and move into a fixed number of HBM slots on demand under a
// least-recently-used policy.  A push hop = for every shard that has an active
// subject (ascending shard index on odd hops, descending on even ones): make it
// resident (hit, or load and maybe evict), restrict the frontier to its
// subjects, push, OR into the global next level (object ids are global, so
// "map back" is free).  The next shard's load is issued on a copy stream while
// the current one computes.
//
// A dense hop pulls instead, as on a resident graph: the same triples cut a
// second way, by object range, into sub-graphs that hold whole rows of OBJ (the
// chunks the predecessor pass streams).  They are units of the same cache: a
// pull hop visits every object range in turn (subjects and relation ids of its
// rows in a cache slot), gathers the frontier lines of each row's subjects and
// writes that range's part of the next level, without atomics.
#include <fcntl.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <cerrno>
#include <queue>
#include <string>

#include "common.h"

namespace lkg {

struct ShardSet {
    int n = 0;
    std::vector<int64_t> edge_begin;  // [n+1] positions in the shard-grouped edge arrays
    int32_t *h_obj = nullptr;         // pinned host, [T] grouped by shard
    uint16_t *h_rel = nullptr;        // pinned host, [T]
    // cache
    int n_slots = 0;
    size_t slot_edges = 0;  // capacity of a slot = largest shard
    std::vector<int32_t *> slot_obj;
    std::vector<uint16_t *> slot_rel;
    std::vector<int> slot_shard, shard_slot;
    std::vector<uint64_t> slot_used;
    std::vector<hipEvent_t> slot_ready, slot_idle;
    uint64_t tick = 0;
    hipStream_t copy_stream = nullptr;
    int64_t loads = 0, evictions = 0, hits = 0, bytes_h2d = 0;
    // sub-graphs on disk (build option shard_dir): one file per shard instead of h_obj / h_rel,
    // read on a miss into the slot's pinned staging buffer and copied from there
    std::vector<int> fd;
    std::vector<int32_t *> host_obj;   // [n_slots] pinned, slot_edges entries
    std::vector<uint16_t *> host_rel;
    int64_t bytes_disk = 0;
    unsigned long long *d_route = nullptr, *h_route = nullptr;  // [kRouteWords], see k_route_count
    // object-sorted triples (for predecessor edges): pinned host arrays, streamed through two
    // staging buffers in chunks of whole 64-entity tiles
    int32_t *h_in_sub = nullptr, *h_in_eid = nullptr;
    uint16_t *h_in_rel = nullptr;
    struct Chunk { long long tile_begin, tile_count; int64_t edge_begin, edge_count; long long row_begin, hub_count, row_count; };
    std::vector<Chunk> chunks;
    // pull work lists of every chunk (object range), concatenated on the device
    std::vector<RowClasses> pull_lists;
    ShortRow *d_tail = nullptr;
    PullSegment *d_seg = nullptr;
    int32_t *d_multi = nullptr;
    // cacheable units: the shards, then the object ranges (subjects + relation ids of their rows of
    // OBJ), then the triple indices of the object ranges (read by the predecessor pass only)
    int units() const { return n + 2 * (int)chunks.size(); }
    int range_unit(int c) const { return n + c; }
    int index_unit(int c) const { return n + (int)chunks.size() + c; }
    size_t stage_edges = 0;
    int32_t *stage_sub[2] = {nullptr, nullptr}, *stage_eid[2] = {nullptr, nullptr};
    uint16_t *stage_rel[2] = {nullptr, nullptr};
    hipEvent_t stage_ready[2] = {nullptr, nullptr}, stage_idle[2] = {nullptr, nullptr};
    int64_t in_bytes_h2d = 0;
};

// Routing of a hop (Algorithm 1, line 2) in two passes over the entities, whatever the number of
// shards.  Layout of `route` (unsigned long long, kRouteWords entries):
//   [0,128) active subject rows per shard   [128,256) their triples
//   [256,384) rows of up to 32 triples       [384,512) 256-triple segments of the longer rows
//   [512,640) first place of the shard in the short-row list   [640,768) in the segment list
//   [768,1024) append cursors, two per shard (short rows, segments); after k_route_lists they are
//              the counts the push kernels read
constexpr int kRouteWords = 1024, kRouteBase = 512, kRouteCursor = 768;

// The lanes of a wavefront that hold a subject of the same shard, one shard after the other.
template <typename F>
__device__ __forceinline__ void for_each_shard(bool has, int shard, F body) {
    unsigned long long todo = __ballot(has);
    while (todo) {  // wave-uniform
        const int leader = __ffsll((long long)todo) - 1;
        const int s0 = __shfl(shard, leader);
        const bool mine = has && shard == s0;
        todo &= ~__ballot(mine);
        body(s0, mine, leader);
    }
}

__global__ void __launch_bounds__(256)
k_route_count(const uint32_t *__restrict__ act, int32_t E, const uint32_t *__restrict__ out_off,
              const uint8_t *__restrict__ shard_of, unsigned long long *route) {
    __shared__ unsigned long long sh[4][128];
    for (int i = threadIdx.x; i < 512; i += blockDim.x) sh[i >> 7][i & 127] = 0;
    __syncthreads();
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long base = (long long)blockIdx.x * blockDim.x; base < E; base += stride) {  // block-uniform trip count
        const long long e = base + threadIdx.x;
        uint32_t d = 0;
        int shard = 0;
        if (e < E && ((act[e >> 5] >> (e & 31)) & 1u)) {
            d = out_off[e + 1] - out_off[e];
            if (d) shard = shard_of[e] & 127;
        }
        const bool tail = d > 0 && d <= (uint32_t)kTailMaxDegree;
        const long long segs = d > (uint32_t)kTailMaxDegree ? (d + kPushSegment - 1) / kPushSegment : 0;
        for_each_shard(d > 0, shard, [&](int s0, bool mine, int leader) {
            const long long rows = __popcll(__ballot(mine)), tails = __popcll(__ballot(mine && tail));
            const long long edges = wave_sum(mine ? (long long)d : 0), sg = wave_sum(mine ? segs : 0);
            if (lane() == leader) {
                atomicAdd(&sh[0][s0], (unsigned long long)rows);
                atomicAdd(&sh[1][s0], (unsigned long long)edges);
                if (tails) atomicAdd(&sh[2][s0], (unsigned long long)tails);
                if (sg) atomicAdd(&sh[3][s0], (unsigned long long)sg);
            }
        });
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 512; i += blockDim.x)
        if (sh[i >> 7][i & 127]) atomicAdd(&route[i], sh[i >> 7][i & 127]);
}

// Every block owns a contiguous run of entities: it counts its list entries per shard, reserves
// their places with one atomic per shard and list, and then writes them (the run is read twice;
// an atomic per wavefront and shard on sixteen global cursors would serialise).
__global__ void __launch_bounds__(256)
k_route_lists(const uint32_t *__restrict__ act, int32_t E, const uint32_t *__restrict__ out_off,
              const uint32_t *__restrict__ row_begin, const uint8_t *__restrict__ shard_of,
              unsigned long long *route, int32_t *list_tail, RowSegment *list_seg) {
    __shared__ unsigned int cnt[2][128];           // entries of this block per shard: short rows, segments
    __shared__ unsigned long long first[2][128];   // first place of the block's entries in the two lists
    for (int i = threadIdx.x; i < 256; i += blockDim.x) cnt[i >> 7][i & 127] = 0;
    __syncthreads();
    const long long chunk = (((long long)E + gridDim.x - 1) / gridDim.x + 255) / 256 * 256;
    const long long begin = (long long)blockIdx.x * chunk, end = min((long long)E, begin + chunk);
    auto classify = [&](long long e, uint32_t &d, int &shard) {
        d = 0;
        shard = 0;
        if (e < end && ((act[e >> 5] >> (e & 31)) & 1u)) {
            d = out_off[e + 1] - out_off[e];
            if (d) shard = shard_of[e] & 127;
        }
    };
    for (long long base = begin; base < end; base += blockDim.x) {  // block-uniform trip count
        uint32_t d;
        int shard;
        classify(base + threadIdx.x, d, shard);
        const bool tail = d > 0 && d <= (uint32_t)kTailMaxDegree;
        const int segs = d > (uint32_t)kTailMaxDegree ? (int)((d + kPushSegment - 1) / kPushSegment) : 0;
        for_each_shard(d > 0, shard, [&](int s0, bool mine, int leader) {
            const int tails = __popcll(__ballot(mine && tail));
            const int sg = (int)wave_sum(mine ? (long long)segs : 0);
            if (lane() == leader) {
                if (tails) atomicAdd(&cnt[0][s0], (unsigned)tails);
                if (sg) atomicAdd(&cnt[1][s0], (unsigned)sg);
            }
        });
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 256; i += blockDim.x) {
        const int which = i >> 7, s0 = i & 127;
        unsigned long long f = 0;
        if (cnt[which][s0])
            f = route[kRouteBase + 128 * which + s0] +
                atomicAdd(&route[kRouteCursor + 2 * s0 + which], (unsigned long long)cnt[which][s0]);
        first[which][s0] = f;
        cnt[which][s0] = 0;  // from here on: entries written so far
    }
    __syncthreads();
    for (long long base = begin; base < end; base += blockDim.x) {
        const long long e = base + threadIdx.x;
        uint32_t d;
        int shard;
        classify(e, d, shard);
        const bool tail = d > 0 && d <= (uint32_t)kTailMaxDegree;
        const int segs = d > (uint32_t)kTailMaxDegree ? (int)((d + kPushSegment - 1) / kPushSegment) : 0;
        for_each_shard(d > 0, shard, [&](int s0, bool mine, int leader) {
            const unsigned long long tmask = __ballot(mine && tail);
            int ts;
            const int ps = wave_excl_scan(mine ? segs : 0, ts);
            unsigned bt = 0, bs = 0;
            if (lane() == leader) {
                if (tmask) bt = atomicAdd(&cnt[0][s0], (unsigned)__popcll(tmask));
                if (ts) bs = atomicAdd(&cnt[1][s0], (unsigned)ts);
            }
            const unsigned long long at = first[0][s0] + (unsigned)__shfl((int)bt, leader);
            const unsigned long long as = first[1][s0] + (unsigned)__shfl((int)bs, leader);
            if (mine && tail) list_tail[at + __popcll(tmask & ((1ull << lane()) - 1ull))] = (int32_t)e;
            if (mine && segs) {
                const uint32_t lo = row_begin[e];
                for (int i = 0; i < segs; ++i)
                    list_seg[as + ps + i] = RowSegment{(int32_t)e, lo + (uint32_t)i * kPushSegment};
            }
        });
    }
}

void free_shards(logoskg_graph *g) {
    ShardSet *ss = (ShardSet *)g->shards;
    if (!ss) return;
    if (ss->copy_stream) (void)hipStreamSynchronize(ss->copy_stream);
    for (auto p : ss->slot_obj) if (p) (void)hipFree(p);
    for (auto p : ss->slot_rel) if (p) (void)hipFree(p);
    for (auto e : ss->slot_ready) if (e) (void)hipEventDestroy(e);
    for (auto e : ss->slot_idle) if (e) (void)hipEventDestroy(e);
    for (int i = 0; i < 2; ++i) {
        if (ss->stage_sub[i]) (void)hipFree(ss->stage_sub[i]);
        if (ss->stage_eid[i]) (void)hipFree(ss->stage_eid[i]);
        if (ss->stage_rel[i]) (void)hipFree(ss->stage_rel[i]);
        if (ss->stage_ready[i]) (void)hipEventDestroy(ss->stage_ready[i]);
        if (ss->stage_idle[i]) (void)hipEventDestroy(ss->stage_idle[i]);
    }
    if (ss->h_in_sub) (void)hipHostFree(ss->h_in_sub);
    if (ss->h_in_eid) (void)hipHostFree(ss->h_in_eid);
    if (ss->h_in_rel) (void)hipHostFree(ss->h_in_rel);
    if (ss->h_obj) (void)hipHostFree(ss->h_obj);
    if (ss->h_rel) (void)hipHostFree(ss->h_rel);
    for (auto p : ss->host_obj) if (p) (void)hipHostFree(p);
    for (auto p : ss->host_rel) if (p) (void)hipHostFree(p);
    for (int f : ss->fd) if (f >= 0) (void)close(f);
    if (ss->d_route) (void)hipFree(ss->d_route);
    if (ss->h_route) (void)hipHostFree(ss->h_route);
    if (ss->d_tail) (void)hipFree(ss->d_tail);
    if (ss->d_seg) (void)hipFree(ss->d_seg);
    if (ss->d_multi) (void)hipFree(ss->d_multi);
    if (g->row_begin && g->row_begin != g->out_off) (void)hipFree(g->row_begin);
    if (g->shard_of_dev) (void)hipFree(g->shard_of_dev);
    g->row_begin = nullptr;
    g->shard_of_dev = nullptr;
    delete ss;
    g->shards = nullptr;
}

// Object-sorted triples for the predecessor pass of a sharded graph: offsets and
// the hub list stay in HBM, the per-triple arrays go to pinned host memory and
// are cut into chunks of whole tiles holding about T / num_shards triples each.
static logoskg_status build_in_chunks(logoskg_graph *g, ShardSet *ss, const int32_t *subj, const int32_t *rel,
                                      const int32_t *obj, TripleSorter *sorter) {
    const int32_t E = g->E;
    const int64_t T = g->T;
    std::vector<uint32_t> ioff;
    if (sorter) {
        LKG_TRY(sorter_offsets(sorter, true, &ioff));
    } else {
        ioff.assign((size_t)E + 1, 0);
        for (int64_t t = 0; t < T; ++t) ioff[(size_t)obj[t] + 1]++;
        for (int32_t e = 0; e < E; ++e) ioff[(size_t)e + 1] += ioff[e];
    }
    std::vector<int32_t> longrows;  // rows of more than kTailMaxDegree entries, chunk by chunk
    size_t n4 = std::max<int64_t>(T, 1) * sizeof(int32_t), n2 = std::max<int64_t>(T, 1) * sizeof(uint16_t);
    if (hipHostMalloc((void **)&ss->h_in_sub, n4, hipHostMallocDefault) != hipSuccess ||
        hipHostMalloc((void **)&ss->h_in_eid, n4, hipHostMallocDefault) != hipSuccess ||
        hipHostMalloc((void **)&ss->h_in_rel, n2, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        set_error("pinned host allocation of %zu bytes failed", 2 * n4 + n2);
        return LOGOSKG_ENOMEM;
    }
    g->pinned_bytes += 2 * n4 + n2;
    if (sorter) {
        LKG_TRY(sorter_object_order(sorter, ss->h_in_sub, ss->h_in_rel, ss->h_in_eid));
    } else {
        std::vector<uint32_t> cur(ioff.begin(), ioff.end() - 1);
        for (int64_t t = 0; t < T; ++t) {
            uint32_t p = cur[obj[t]]++;
            ss->h_in_sub[p] = subj[t];
            ss->h_in_rel[p] = (uint16_t)rel[t];
            ss->h_in_eid[p] = (int32_t)t;
        }
    }
    LKG_HIP(hipMalloc((void **)&g->in_off, ((size_t)E + 1) * sizeof(uint32_t)));
    LKG_HIP(hipMemcpy(g->in_off, ioff.data(), ((size_t)E + 1) * sizeof(uint32_t), hipMemcpyHostToDevice));
    g->static_bytes += ((size_t)E + 1) * sizeof(uint32_t);
    // chunks of whole tiles
    const long long ntiles = g->Epad / kTileEntities;
    const int64_t target = std::max<int64_t>(1, (T + g->num_shards - 1) / g->num_shards);
    long long t0 = 0;
    while (t0 < ntiles) {
        long long t1 = t0;
        int64_t e_begin = ioff[(size_t)std::min<long long>(t0 * 64, E)], e_end = e_begin;
        while (t1 < ntiles) {  // chunks begin on a multiple of kPredTiles tiles
            const long long t2 = std::min<long long>(t1 + kPredTiles, ntiles);
            int64_t nxt = ioff[(size_t)std::min<long long>(t2 * 64, E)];
            if (t1 > t0 && nxt - e_begin > target) break;
            e_end = nxt;
            t1 = t2;
        }
        ShardSet::Chunk c;
        c.tile_begin = t0; c.tile_count = t1 - t0; c.edge_begin = e_begin; c.edge_count = e_end - e_begin;
        c.row_begin = (long long)longrows.size();
        c.hub_count = 0;
        for (long long e = t0 * 64; e < std::min<long long>(t1 * 64, E); ++e) {
            uint32_t d = ioff[(size_t)e + 1] - ioff[(size_t)e];
            if (d > (uint32_t)kTailMaxDegree) longrows.push_back((int32_t)e);
            if (d >= (uint32_t)g->hub_min) c.hub_count++;
        }
        std::stable_sort(longrows.begin() + c.row_begin, longrows.end(), [&](int32_t x, int32_t y) {
            return ioff[(size_t)x + 1] - ioff[x] > ioff[(size_t)y + 1] - ioff[y];
        });
        c.row_count = (long long)longrows.size() - c.row_begin;
        g->in_rows.n_hub += c.hub_count;
        ss->chunks.push_back(c);
        ss->stage_edges = std::max(ss->stage_edges, (size_t)c.edge_count);
        t0 = t1;
    }
    {   // pull work lists per chunk: short rows by descending length, segments of the long rows
        // (already longest first), rows with several segments
        std::vector<ShortRow> tail;
        std::vector<PullSegment> seg;
        std::vector<int32_t> multi;
        std::vector<std::vector<int32_t>> bucket(kTailMaxDegree + 1);
        struct First { size_t tail, seg, multi; };
        std::vector<First> first;  // where every chunk's lists begin in the concatenations
        for (const ShardSet::Chunk &c : ss->chunks) {
            RowClasses rc;
            const size_t t_begin = tail.size(), s_begin = seg.size(), m_begin = multi.size();
            for (auto &b : bucket) b.clear();
            for (long long e = c.tile_begin * 64; e < std::min<long long>((c.tile_begin + c.tile_count) * 64, E); ++e) {
                const uint32_t d = ioff[(size_t)e + 1] - ioff[(size_t)e];
                if (d >= 1 && d <= (uint32_t)kTailMaxDegree) bucket[d].push_back((int32_t)e);
            }
            for (int d = kTailMaxDegree; d >= 1; --d)
                for (int32_t v : bucket[d]) tail.push_back({v, ioff[(size_t)v], ioff[(size_t)v + 1]});
            for (long long i = 0; i < c.row_count; ++i) {
                const int32_t v = longrows[(size_t)(c.row_begin + i)];
                const uint32_t lo = ioff[(size_t)v], hi = ioff[(size_t)v + 1];
                const bool several = hi - lo > (uint32_t)kPullSegment;
                if (several) multi.push_back(v);
                for (uint32_t j = lo; j < hi; j += kPullSegment)
                    seg.push_back({v, j, std::min(j + (uint32_t)kPullSegment, hi), several ? 1u : 0u});
            }
            rc.n_tail = (int64_t)(tail.size() - t_begin);
            rc.n_seg = (int64_t)(seg.size() - s_begin);
            rc.n_multi = (int64_t)(multi.size() - m_begin);
            first.push_back({t_begin, s_begin, m_begin});
            ss->pull_lists.push_back(rc);
        }
        LKG_HIP(hipMalloc((void **)&ss->d_tail, std::max<size_t>(tail.size(), 1) * sizeof(ShortRow)));
        LKG_HIP(hipMalloc((void **)&ss->d_seg, std::max<size_t>(seg.size(), 1) * sizeof(PullSegment)));
        LKG_HIP(hipMalloc((void **)&ss->d_multi, std::max<size_t>(multi.size(), 1) * sizeof(int32_t)));
        if (!tail.empty()) LKG_HIP(hipMemcpy(ss->d_tail, tail.data(), tail.size() * sizeof(ShortRow), hipMemcpyHostToDevice));
        if (!seg.empty()) LKG_HIP(hipMemcpy(ss->d_seg, seg.data(), seg.size() * sizeof(PullSegment), hipMemcpyHostToDevice));
        if (!multi.empty()) LKG_HIP(hipMemcpy(ss->d_multi, multi.data(), multi.size() * sizeof(int32_t), hipMemcpyHostToDevice));
        g->static_bytes += tail.size() * sizeof(ShortRow) + seg.size() * sizeof(PullSegment) + multi.size() * sizeof(int32_t);
        for (size_t i = 0; i < ss->pull_lists.size(); ++i) {
            ss->pull_lists[i].tail = ss->d_tail + first[i].tail;
            ss->pull_lists[i].seg = ss->d_seg + first[i].seg;
            ss->pull_lists[i].multi = ss->d_multi + first[i].multi;
        }
        g->in_rows.n_tail = (int64_t)tail.size();
        g->in_rows.n_seg = (int64_t)seg.size();
        g->in_rows.n_multi = (int64_t)multi.size();
    }
    g->in_rows.n_long = (int64_t)longrows.size();
    LKG_HIP(hipMalloc((void **)&g->in_rows.longrows, std::max<size_t>(longrows.size(), 1) * sizeof(int32_t)));
    if (!longrows.empty())
        LKG_HIP(hipMemcpy(g->in_rows.longrows, longrows.data(), longrows.size() * sizeof(int32_t),
                          hipMemcpyHostToDevice));
    ss->stage_edges = std::max<size_t>(ss->stage_edges, 1);
    return LOGOSKG_OK;
}

long long max_chunk_rows(const logoskg_graph *g) {
    const ShardSet *ss = (const ShardSet *)g->shards;
    long long m = 0;
    if (ss)
        for (const ShardSet::Chunk &c : ss->chunks) m = std::max(m, c.row_count);
    return m;
}

static logoskg_status acquire(logoskg_graph *g, ShardSet *ss, int shard, hipStream_t compute, int *slot_out);

// The two staging buffers of the streamed predecessor pass, allocated at its first use.
static logoskg_status ensure_staging(logoskg_graph *g, ShardSet *ss) {
    if (ss->stage_sub[0]) return LOGOSKG_OK;
    for (int i = 0; i < 2; ++i) {
        LKG_HIP(hipMalloc((void **)&ss->stage_sub[i], ss->stage_edges * sizeof(int32_t)));
        LKG_HIP(hipMalloc((void **)&ss->stage_eid[i], ss->stage_edges * sizeof(int32_t)));
        LKG_HIP(hipMalloc((void **)&ss->stage_rel[i], ss->stage_edges * sizeof(uint16_t)));
        g->static_bytes += ss->stage_edges * 10;
        LKG_HIP(hipEventCreateWithFlags(&ss->stage_ready[i], hipEventDisableTiming));
        LKG_HIP(hipEventCreateWithFlags(&ss->stage_idle[i], hipEventDisableTiming));
    }
    return LOGOSKG_OK;
}

// Predecessor pass of a sharded graph, object range after object range.  When the cache can hold
// every unit, the rows of OBJ come through it: a range's subjects and relation ids (the unit the
// pull hops use) and its triple indices (a unit of their own) are made resident like a shard, so
// a cache that holds the graph serves every fetch without a copy.  A smaller cache would only
// thrash, and push out what the hops need (measured: 17 slots for 26 units, 284 ms per step with
// the pass through the cache): then the three arrays are streamed through two staging buffers
// (the next range copies while this one runs) and the cache is left to the hops.
logoskg_status sharded_pred(logoskg_graph *g, FillArgs *a, int W, bool mask, hipStream_t st) {
    ShardSet *ss = (ShardSet *)g->shards;
    if (!ss) { set_error("graph has no shards"); return LOGOSKG_EINTERNAL; }
    auto launch = [&](const ShardSet::Chunk &c, const int32_t *sub, const uint16_t *rel, const int32_t *eid) {
        FillArgs x = *a;
        x.in_sub = sub - c.edge_begin;
        x.in_eid = eid - c.edge_begin;
        x.in_rel = rel - c.edge_begin;
        x.tile_begin = c.tile_begin;
        x.tile_count = c.tile_count;
        x.rows = g->in_rows.longrows + c.row_begin;
        x.row_base = c.row_begin;
        launch_pred(g->prof, x, W, c.hub_count, c.row_count - c.hub_count, mask, st, st);
    };
    if (ss->n_slots >= ss->units()) {
        const size_t nc = ss->chunks.size();
        std::vector<int> s_range(nc, -1), s_index(nc, -1);
        auto make_resident = [&](size_t ci) -> logoskg_status {
            if (ss->chunks[ci].edge_count == 0 || s_range[ci] >= 0) return LOGOSKG_OK;
            LKG_TRY(acquire(g, ss, ss->range_unit((int)ci), st, &s_range[ci]));
            LKG_TRY(acquire(g, ss, ss->index_unit((int)ci), st, &s_index[ci]));
            return LOGOSKG_OK;
        };
        for (size_t ci = 0; ci < nc; ++ci) {
            const ShardSet::Chunk &c = ss->chunks[ci];
            LKG_TRY(make_resident(ci));
            if (c.edge_count > 0) {
                LKG_HIP(hipStreamWaitEvent(st, ss->slot_ready[s_range[ci]], 0));
                LKG_HIP(hipStreamWaitEvent(st, ss->slot_ready[s_index[ci]], 0));
            }
            const int a_slot = c.edge_count > 0 ? s_range[ci] : 0, b_slot = c.edge_count > 0 ? s_index[ci] : 0;
            launch(c, ss->slot_obj[a_slot], ss->slot_rel[a_slot], ss->slot_obj[b_slot]);
            LKG_HIP(hipGetLastError());
            if (c.edge_count > 0) {
                LKG_HIP(hipEventRecord(ss->slot_idle[s_range[ci]], st));
                LKG_HIP(hipEventRecord(ss->slot_idle[s_index[ci]], st));
            }
            // the next range's two units are asked for while this one runs (nothing is evicted: every
            // unit has a slot)
            if (ci + 1 < nc) LKG_TRY(make_resident(ci + 1));
        }
        return LOGOSKG_OK;
    }
    LKG_TRY(ensure_staging(g, ss));
    auto issue = [&](size_t ci) -> logoskg_status {
        const ShardSet::Chunk &c = ss->chunks[ci];
        const int b = (int)(ci & 1);
        LKG_HIP(hipStreamWaitEvent(ss->copy_stream, ss->stage_idle[b], 0));
        if (c.edge_count > 0) {
            g->prof.begin(KK_SHARD_COPY, ss->copy_stream);
            LKG_HIP(hipMemcpyAsync(ss->stage_sub[b], ss->h_in_sub + c.edge_begin, (size_t)c.edge_count * 4,
                                   hipMemcpyHostToDevice, ss->copy_stream));
            LKG_HIP(hipMemcpyAsync(ss->stage_eid[b], ss->h_in_eid + c.edge_begin, (size_t)c.edge_count * 4,
                                   hipMemcpyHostToDevice, ss->copy_stream));
            if (mask)
                LKG_HIP(hipMemcpyAsync(ss->stage_rel[b], ss->h_in_rel + c.edge_begin, (size_t)c.edge_count * 2,
                                       hipMemcpyHostToDevice, ss->copy_stream));
            g->prof.end(ss->copy_stream);
            ss->in_bytes_h2d += c.edge_count * (mask ? 10 : 8);
        }
        LKG_HIP(hipEventRecord(ss->stage_ready[b], ss->copy_stream));
        return LOGOSKG_OK;
    };
    if (!ss->chunks.empty()) LKG_TRY(issue(0));
    for (size_t ci = 0; ci < ss->chunks.size(); ++ci) {
        const ShardSet::Chunk &c = ss->chunks[ci];
        const int b = (int)(ci & 1);
        if (ci + 1 < ss->chunks.size()) LKG_TRY(issue(ci + 1));
        LKG_HIP(hipStreamWaitEvent(st, ss->stage_ready[b], 0));
        launch(c, ss->stage_sub[b], ss->stage_rel[b], ss->stage_eid[b]);
        LKG_HIP(hipGetLastError());
        LKG_HIP(hipEventRecord(ss->stage_idle[b], st));
    }
    return LOGOSKG_OK;
}

// Shard file: 32-byte header (magic, shard index, number of triples, 0), then the objects
// (int32) and the relation ids (uint16) of the shard's triples in the shard-grouped order.
struct ShardFileHeader {
    char magic[8];
    int64_t shard, count, reserved;
};
static const char kShardMagic[8] = {'L', 'K', 'G', 'S', 'H', 'R', 'D', '1'};

static bool write_all(int fd, const void *buf, size_t bytes) {
    const char *p = (const char *)buf;
    while (bytes > 0) {
        ssize_t w = write(fd, p, std::min<size_t>(bytes, (size_t)1 << 30));
        if (w < 0) {
            if (errno == EINTR) continue;
            return false;
        }
        p += w;
        bytes -= (size_t)w;
    }
    return true;
}

static bool read_all_at(int fd, void *buf, size_t bytes, off_t at) {
    char *p = (char *)buf;
    while (bytes > 0) {
        ssize_t r = pread(fd, p, std::min<size_t>(bytes, (size_t)1 << 30), at);
        if (r < 0 && errno == EINTR) continue;
        if (r <= 0) return false;
        p += r;
        at += r;
        bytes -= (size_t)r;
    }
    return true;
}

// Sec. 3.4, sub-graphs on disk: writes every shard to <dir>/shard_<i>.lkg, releases the pinned
// copy of all shards and keeps one pinned staging buffer per cache slot instead.
static logoskg_status shards_to_disk(logoskg_graph *g, ShardSet *ss, const char *dir) {
    ss->fd.assign((size_t)ss->n, -1);
    for (int s = 0; s < ss->n; ++s) {
        const std::string path = std::string(dir) + "/shard_" + std::to_string(s) + ".lkg";
        const int64_t b = ss->edge_begin[s], cnt = ss->edge_begin[(size_t)s + 1] - b;
        int fd = open(path.c_str(), O_CREAT | O_TRUNC | O_WRONLY, 0644);
        ShardFileHeader h;
        memcpy(h.magic, kShardMagic, 8);
        h.shard = s;
        h.count = cnt;
        h.reserved = 0;
        const bool ok = fd >= 0 && write_all(fd, &h, sizeof(h)) &&
                        write_all(fd, ss->h_obj + b, (size_t)cnt * sizeof(int32_t)) &&
                        write_all(fd, ss->h_rel + b, (size_t)cnt * sizeof(uint16_t));
        if (fd >= 0 && close(fd) != 0 && ok) { set_error("closing %s failed: %s", path.c_str(), strerror(errno)); return LOGOSKG_EIO; }
        if (!ok) { set_error("writing %s failed: %s", path.c_str(), strerror(errno)); return LOGOSKG_EIO; }
        ss->fd[s] = open(path.c_str(), O_RDONLY);
        if (ss->fd[s] < 0) { set_error("opening %s failed: %s", path.c_str(), strerror(errno)); return LOGOSKG_EIO; }
    }
    const size_t all = std::max<int64_t>(g->T, 1) * (sizeof(int32_t) + sizeof(uint16_t));
    (void)hipHostFree(ss->h_obj);
    (void)hipHostFree(ss->h_rel);
    ss->h_obj = nullptr;
    ss->h_rel = nullptr;
    g->pinned_bytes -= all;
    ss->host_obj.assign((size_t)ss->n_slots, nullptr);
    ss->host_rel.assign((size_t)ss->n_slots, nullptr);
    for (int i = 0; i < ss->n_slots; ++i) {
        if (hipHostMalloc((void **)&ss->host_obj[i], ss->slot_edges * sizeof(int32_t), hipHostMallocDefault) != hipSuccess ||
            hipHostMalloc((void **)&ss->host_rel[i], ss->slot_edges * sizeof(uint16_t), hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            set_error("pinned staging buffer of %zu bytes failed", ss->slot_edges * 6);
            return LOGOSKG_ENOMEM;
        }
        g->pinned_bytes += ss->slot_edges * (sizeof(int32_t) + sizeof(uint16_t));
    }
    return LOGOSKG_OK;
}

logoskg_status build_shards(logoskg_graph *g, const int32_t *subj, const int32_t *rel, const int32_t *obj,
                            const logoskg_build_opts *opts, const std::vector<uint32_t> &ooff, TripleSorter *sorter) {
    const int n = g->num_shards;
    const int32_t E = g->E;
    const int64_t T = g->T;
    ShardSet *ss = new (std::nothrow) ShardSet();
    if (!ss) { set_error("out of host memory"); return LOGOSKG_ENOMEM; }
    g->shards = ss;
    ss->n = n;

    // out-degrees
    std::vector<uint32_t> deg((size_t)E, 0);
    for (int32_t e = 0; e < E; ++e) deg[e] = ooff[(size_t)e + 1] - ooff[e];
    // subjects by (degree desc, id asc); counting sort on the degree keeps it O(E + maxdeg)
    uint32_t maxdeg = 0;
    for (int32_t e = 0; e < E; ++e) maxdeg = std::max(maxdeg, deg[e]);
    std::vector<int64_t> first((size_t)maxdeg + 2, 0);
    for (int32_t e = 0; e < E; ++e) if (deg[e]) first[deg[e]]++;
    {   // positions for descending degree
        int64_t run = 0;
        for (int64_t d = maxdeg; d >= 1; --d) { int64_t c = first[d]; first[d] = run; run += c; }
    }
    std::vector<int32_t> order((size_t)g->n_out_rows);
    for (int32_t e = 0; e < E; ++e) if (deg[e]) order[(size_t)first[deg[e]]++] = e;
    // greedy: lightest shard so far, ties to the lowest index
    g->shard_of.assign((size_t)E, -1);
    g->shard_triples.assign((size_t)n, 0);
    typedef std::pair<int64_t, int> Load;  // (triples, shard)
    std::priority_queue<Load, std::vector<Load>, std::greater<Load>> heap;
    for (int s = 0; s < n; ++s) heap.push(Load(0, s));
    for (int32_t e : order) {
        Load l = heap.top();
        heap.pop();
        g->shard_of[e] = l.second;
        l.first += deg[e];
        g->shard_triples[(size_t)l.second] = l.first;
        heap.push(l);
    }
    ss->edge_begin.assign((size_t)n + 1, 0);
    for (int s = 0; s < n; ++s) ss->edge_begin[(size_t)s + 1] = ss->edge_begin[s] + g->shard_triples[s];
    // row_begin: subjects of a shard in ascending id inside the shard's range
    std::vector<uint32_t> row_begin((size_t)E, 0);
    {
        std::vector<int64_t> cur(ss->edge_begin.begin(), ss->edge_begin.end() - 1);
        for (int32_t e = 0; e < E; ++e) {
            int s = g->shard_of[e];
            if (s < 0) continue;
            row_begin[e] = (uint32_t)cur[s];
            cur[s] += deg[e];
        }
    }
    size_t ob = std::max<int64_t>(T, 1) * sizeof(int32_t), rb = std::max<int64_t>(T, 1) * sizeof(uint16_t);
    if (hipHostMalloc((void **)&ss->h_obj, ob, hipHostMallocDefault) != hipSuccess ||
        hipHostMalloc((void **)&ss->h_rel, rb, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        set_error("pinned host allocation of %zu bytes failed", ob + rb);
        return LOGOSKG_ENOMEM;
    }
    g->pinned_bytes += ob + rb;
    // device metadata: row_begin and the map P
    LKG_HIP(hipMalloc((void **)&g->row_begin, (size_t)E * sizeof(uint32_t)));
    LKG_HIP(hipMemcpy(g->row_begin, row_begin.data(), (size_t)E * sizeof(uint32_t), hipMemcpyHostToDevice));
    g->static_bytes += (size_t)E * sizeof(uint32_t);
    if (sorter) {
        LKG_TRY(sorter_subject_order(sorter, g->row_begin, ss->h_obj, ss->h_rel));
    } else {
        std::vector<uint32_t> cur(row_begin);
        for (int64_t t = 0; t < T; ++t) {
            uint32_t p = cur[subj[t]]++;
            ss->h_obj[p] = obj[t];
            ss->h_rel[p] = (uint16_t)rel[t];
        }
    }
    {
        std::vector<uint8_t> p8((size_t)g->Epad, 255);
        for (int32_t e = 0; e < E; ++e) if (g->shard_of[e] >= 0) p8[e] = (uint8_t)g->shard_of[e];
        LKG_HIP(hipMalloc((void **)&g->shard_of_dev, (size_t)g->Epad));
        LKG_HIP(hipMemcpy(g->shard_of_dev, p8.data(), (size_t)g->Epad, hipMemcpyHostToDevice));
        g->static_bytes += (size_t)g->Epad;
    }
    LKG_TRY(build_in_chunks(g, ss, subj, rel, obj, sorter));
    // cache slots: each holds one sub-graph, a subject shard (objects + relation ids) or an object
    // range (subjects + relation ids): 6 bytes per triple either way
    int64_t largest = 1;
    for (int s = 0; s < n; ++s) largest = std::max(largest, g->shard_triples[s]);
    for (const ShardSet::Chunk &c : ss->chunks) largest = std::max<int64_t>(largest, c.edge_count);
    ss->slot_edges = (size_t)largest;
    size_t slot_bytes = ss->slot_edges * (sizeof(int32_t) + sizeof(uint16_t));
    int slots = ss->units();
    if (opts->max_resident_shards > 0) slots = std::min(slots, opts->max_resident_shards);
    if (opts->hbm_shard_budget_bytes > 0) {
        uint64_t fit = opts->hbm_shard_budget_bytes / slot_bytes;
        if (fit == 0) {
            set_error("hbm_shard_budget_bytes = %llu is smaller than one shard (%zu bytes)",
                      (unsigned long long)opts->hbm_shard_budget_bytes, slot_bytes);
            return LOGOSKG_ENOMEM;
        }
        slots = (int)std::min<uint64_t>((uint64_t)slots, fit);
    }
    ss->n_slots = slots;
    ss->slot_obj.assign((size_t)slots, nullptr);
    ss->slot_rel.assign((size_t)slots, nullptr);
    ss->slot_shard.assign((size_t)slots, -1);
    ss->shard_slot.assign((size_t)ss->units(), -1);
    ss->slot_used.assign((size_t)slots, 0);
    ss->slot_ready.assign((size_t)slots, nullptr);
    ss->slot_idle.assign((size_t)slots, nullptr);
    for (int i = 0; i < slots; ++i) {
        LKG_HIP(hipMalloc((void **)&ss->slot_obj[i], ss->slot_edges * sizeof(int32_t)));
        LKG_HIP(hipMalloc((void **)&ss->slot_rel[i], ss->slot_edges * sizeof(uint16_t)));
        g->static_bytes += slot_bytes;
        LKG_HIP(hipEventCreateWithFlags(&ss->slot_ready[i], hipEventDisableTiming));
        LKG_HIP(hipEventCreateWithFlags(&ss->slot_idle[i], hipEventDisableTiming));
    }
    if (!(ss->copy_stream = helper_stream(g->device, 2))) {
        set_error("could not create the copy stream");
        return LOGOSKG_EDEVICE;
    }
    if (opts->shard_dir && opts->shard_dir[0]) LKG_TRY(shards_to_disk(g, ss, opts->shard_dir));
    LKG_HIP(hipMalloc((void **)&ss->d_route, 1024 * sizeof(unsigned long long)));
    if (hipHostMalloc((void **)&ss->h_route, 1024 * sizeof(unsigned long long), hipHostMallocDefault) != hipSuccess) {
        set_error("hipHostMalloc failed");
        return LOGOSKG_ENOMEM;
    }
    return LOGOSKG_OK;
}

// Makes a sub-graph resident and returns its slot: a hit refreshes its use stamp; a
// miss takes an empty slot or evicts the least recently used one and starts the
// copy on the copy stream (after the kernels that last read the slot).  Units below
// ss->n are subject shards, the others object ranges (always kept in pinned memory).
static logoskg_status acquire(logoskg_graph *g, ShardSet *ss, int shard, hipStream_t compute, int *slot_out) {
    const int nc = (int)ss->chunks.size();
    const bool range = shard >= ss->n;
    const bool index = shard >= ss->n + nc;           // triple indices of an object range: 4 bytes per triple
    const int chunk = range ? (shard - ss->n) % std::max(nc, 1) : 0;
    int slot = ss->shard_slot[shard];
    if (slot >= 0) {
        ss->hits++;
    } else {
        slot = -1;
        for (int i = 0; i < ss->n_slots; ++i)
            if (ss->slot_shard[i] < 0) { slot = i; break; }
        if (slot < 0) {
            slot = 0;
            for (int i = 1; i < ss->n_slots; ++i)
                if (ss->slot_used[i] < ss->slot_used[slot]) slot = i;
            ss->shard_slot[ss->slot_shard[slot]] = -1;
            ss->evictions++;
        }
        int64_t b = range ? ss->chunks[(size_t)chunk].edge_begin : ss->edge_begin[shard];
        int64_t cnt = range ? ss->chunks[(size_t)chunk].edge_count : ss->edge_begin[(size_t)shard + 1] - b;
        const int32_t *src_obj = index ? ss->h_in_eid + b : range ? ss->h_in_sub + b : (ss->h_obj ? ss->h_obj + b : nullptr);
        const uint16_t *src_rel = index ? nullptr : range ? ss->h_in_rel + b : (ss->h_rel ? ss->h_rel + b : nullptr);
        if (!range && !ss->fd.empty()) {  // the shard comes from its file, through the slot's staging buffer
            LKG_HIP(hipEventSynchronize(ss->slot_ready[slot]));  // the buffer's last copy has left it
            ShardFileHeader h;
            const bool ok = read_all_at(ss->fd[shard], &h, sizeof(h), 0) && memcmp(h.magic, kShardMagic, 8) == 0 &&
                            h.shard == shard && h.count == cnt &&
                            (cnt == 0 ||
                             (read_all_at(ss->fd[shard], ss->host_obj[slot], (size_t)cnt * sizeof(int32_t), sizeof(h)) &&
                              read_all_at(ss->fd[shard], ss->host_rel[slot], (size_t)cnt * sizeof(uint16_t),
                                          (off_t)(sizeof(h) + (size_t)cnt * sizeof(int32_t)))));
            if (!ok) {
                set_error("reading the file of shard %d failed (missing, truncated or not written by this build)", shard);
                return LOGOSKG_EIO;
            }
            src_obj = ss->host_obj[slot];
            src_rel = ss->host_rel[slot];
            ss->bytes_disk += (int64_t)sizeof(h) + cnt * (int64_t)(sizeof(int32_t) + sizeof(uint16_t));
        }
        LKG_HIP(hipStreamWaitEvent(ss->copy_stream, ss->slot_idle[slot], 0));
        if (cnt > 0) {
            g->prof.begin(KK_SHARD_COPY, ss->copy_stream);
            LKG_HIP(hipMemcpyAsync(ss->slot_obj[slot], src_obj, (size_t)cnt * sizeof(int32_t),
                                   hipMemcpyHostToDevice, ss->copy_stream));
            if (src_rel)
                LKG_HIP(hipMemcpyAsync(ss->slot_rel[slot], src_rel, (size_t)cnt * sizeof(uint16_t),
                                       hipMemcpyHostToDevice, ss->copy_stream));
            g->prof.end(ss->copy_stream);
        }
        LKG_HIP(hipEventRecord(ss->slot_ready[slot], ss->copy_stream));
        ss->slot_shard[slot] = shard;
        ss->shard_slot[shard] = slot;
        ss->loads++;
        ss->bytes_h2d += cnt * (int64_t)(sizeof(int32_t) + (src_rel ? sizeof(uint16_t) : 0));
    }
    ss->slot_used[slot] = ++ss->tick;
    (void)compute;
    *slot_out = slot;
    return LOGOSKG_OK;
}

// A pull hop: every object range in turn (down on even hops, up on odd ones, like the shards of
// a push hop), its rows of OBJ in a cache slot.
static logoskg_status run_sharded_pull(logoskg_graph *g, ShardSet *ss, logoskg_result *r, int h, bool want_stats,
                                       const unsigned long long *hc, hipStream_t st, logoskg_hop_stats *hs) {
    std::vector<int> order;
    for (int c = 0; c < (int)ss->chunks.size(); ++c)
        if (ss->chunks[(size_t)c].edge_count > 0) order.push_back(c);
    if ((h & 1) == 0) std::reverse(order.begin(), order.end());
    hs->shards_touched = (int)order.size();
    std::vector<int> slot_of(order.size(), -1);
    for (size_t i = 0; i < order.size(); ++i) {
        const int c = order[i];
        if (slot_of[i] < 0) LKG_TRY(acquire(g, ss, ss->range_unit(c), st, &slot_of[i]));
        const int slot = slot_of[i];
        LKG_HIP(hipStreamWaitEvent(st, ss->slot_ready[slot], 0));
        const int64_t b = ss->chunks[(size_t)c].edge_begin;
        launch_pull_range(g, r, h, ss->pull_lists[(size_t)c], ss->slot_obj[slot] - b, ss->slot_rel[slot] - b, hc,
                          want_stats, i == 0, st);
        LKG_HIP(hipGetLastError());
        LKG_HIP(hipEventRecord(ss->slot_idle[slot], st));
        if (i + 1 < order.size() && ss->n_slots >= 2 && slot_of[i + 1] < 0)
            LKG_TRY(acquire(g, ss, ss->range_unit(order[i + 1]), st, &slot_of[i + 1]));
    }
    return LOGOSKG_OK;
}

logoskg_status run_sharded_hop(logoskg_graph *g, logoskg_result *r, int h, bool pull, bool want_stats,
                               const unsigned long long *hc_in, hipStream_t st, logoskg_hop_stats *hs) {
    ShardSet *ss = (ShardSet *)g->shards;
    if (!ss) { set_error("graph has no shards"); return LOGOSKG_EINTERNAL; }
    if (pull) return run_sharded_pull(g, ss, r, h, want_stats, hc_in, st, hs);
    const long long nwords = r->Epad / 32;
    const uint32_t *act_prev = r->act + (size_t)nwords * (h - 1);
    const unsigned nb = (unsigned)std::min<long long>(1024, std::max<long long>(1, ((long long)g->E + 255) / 256));
    // routing: rows, triples and list sizes of every shard in one pass
    LKG_HIP(hipMemsetAsync(ss->d_route, 0, kRouteWords * sizeof(unsigned long long), st));
    {
        ProfScope ps(g->prof, KK_CENSUS, st);
        k_route_count<<<dim3(nb), dim3(256), 0, st>>>(act_prev, g->E, g->out_off, g->shard_of_dev, ss->d_route);
    }
    LKG_HIP(hipGetLastError());
    LKG_HIP(hipMemcpyAsync(ss->h_route, ss->d_route, 512 * sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
    LKG_HIP(hipStreamSynchronize(st));
    std::vector<int> active;
    unsigned long long tail_run = 0, seg_run = 0;
    for (int s = 0; s < ss->n; ++s) {
        if (ss->h_route[s] > 0) active.push_back(s);
        ss->h_route[kRouteBase + s] = tail_run;
        ss->h_route[kRouteBase + 128 + s] = seg_run;
        tail_run += ss->h_route[256 + s];
        seg_run += ss->h_route[384 + s];
    }
    hs->shards_touched = (int)active.size();
    if (active.empty()) return LOGOSKG_OK;
    // Alg. 1 leaves the order of the shards open.  Even hops go down, odd hops up: the shards a
    // hop ends with are the ones the next hop begins with, so a cache smaller than the graph
    // still hits (a fixed order would evict every shard just before its next use).
    if ((h & 1) == 0) std::reverse(active.begin(), active.end());
    // the work lists of all shards, shard after shard, in a second pass
    LKG_HIP(hipMemcpyAsync(ss->d_route + kRouteBase, ss->h_route + kRouteBase, 256 * sizeof(unsigned long long),
                           hipMemcpyHostToDevice, st));
    {
        ProfScope ps(g->prof, KK_CENSUS, st);
        k_route_lists<<<dim3(nb), dim3(256), 0, st>>>(act_prev, g->E, g->out_off, g->row_begin, g->shard_of_dev,
                                                      ss->d_route, g->fr_tail, g->fr_seg);
    }
    LKG_HIP(hipGetLastError());
    std::vector<int> slot_of((size_t)active.size(), -1);
    for (size_t i = 0; i < active.size(); ++i) {
        const int shard = active[i];
        if (slot_of[i] < 0) LKG_TRY(acquire(g, ss, shard, st, &slot_of[i]));
        const int slot = slot_of[i];
        unsigned long long hc[C_TOTAL] = {};
        hc[C_NTAIL] = ss->h_route[256 + shard];
        hc[C_NSEG] = ss->h_route[384 + shard];
        LKG_HIP(hipStreamWaitEvent(st, ss->slot_ready[slot], 0));
        const int64_t b = ss->edge_begin[shard];
        launch_push_lists(g, r, h, hc, ss->slot_obj[slot] - b, ss->slot_rel[slot] - b, i + 1 == active.size(),
                          g->fr_tail + ss->h_route[kRouteBase + shard], g->fr_seg + ss->h_route[kRouteBase + 128 + shard],
                          ss->d_route + kRouteCursor + 2 * shard, st);
        LKG_HIP(hipGetLastError());
        LKG_HIP(hipEventRecord(ss->slot_idle[slot], st));
        // with at least two slots the next shard's access is issued now, while this one is being
        // expanded (a shard file is read by the calling thread): it never evicts the shard in use,
        // which is the most recently used
        if (i + 1 < active.size() && ss->n_slots >= 2 && slot_of[i + 1] < 0)
            LKG_TRY(acquire(g, ss, active[i + 1], st, &slot_of[i + 1]));
    }
    return LOGOSKG_OK;
}

// The object-sorted triples of a sharded graph (pinned host memory, which kernels can read in
// place over the host link): for the few rows a path listing walks.
bool shard_in_arrays(const logoskg_graph *g, const int32_t **sub, const uint16_t **rel, const int32_t **eid) {
    const ShardSet *ss = (const ShardSet *)g->shards;
    if (!ss || !ss->h_in_sub || !ss->h_in_eid || !ss->h_in_rel) return false;
    *sub = ss->h_in_sub;
    *rel = ss->h_in_rel;
    *eid = ss->h_in_eid;
    return true;
}

// The subject-sorted triples of a sharded graph in the shard-grouped order (pinned host memory;
// absent when the shards live in files): for the rows an active-triple export copies.
bool shard_out_arrays(const logoskg_graph *g, const int32_t **obj, const uint16_t **rel) {
    const ShardSet *ss = (const ShardSet *)g->shards;
    if (!ss || !ss->h_obj || !ss->h_rel) return false;
    *obj = ss->h_obj;
    *rel = ss->h_rel;
    return true;
}

void shard_info(const logoskg_graph *g, logoskg_graph_info *o) {
    const ShardSet *ss = (const ShardSet *)g->shards;
    if (!ss) return;
    o->shard_loads = ss->loads;
    o->shard_evictions = ss->evictions;
    o->shard_hits = ss->hits;
    o->shard_bytes_h2d = ss->bytes_h2d + ss->in_bytes_h2d;
    o->shard_bytes_disk = ss->bytes_disk;
    o->num_object_ranges = (int32_t)ss->chunks.size();
    o->cache_slots = ss->n_slots;
}

}  // namespace lkg

using namespace lkg;

extern "C" logoskg_status logoskg_graph_get_info(const logoskg_graph *g, logoskg_graph_info *o) {
    if (!g || !o) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    memset(o, 0, sizeof(*o));
    o->num_triples = g->T;
    o->num_entities = g->E;
    o->num_relations = g->R;
    o->num_shards = g->num_shards;
    o->hub_min_degree = g->hub_min;
    o->num_out_rows = g->n_out_rows;
    o->num_out_hubs = g->n_out_hubs;
    o->num_in_rows = g->in_rows.n_tail + g->in_rows.n_long;
    o->num_in_hubs = g->in_rows.n_hub;
    o->device_bytes = (int64_t)(g->static_bytes + g->pool.bytes_held());
    o->pinned_host_bytes = (int64_t)g->pinned_bytes;
    shard_info(g, o);
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_graph_partition(const logoskg_graph *g, int32_t *shard_of_entity,
                                                  int64_t *triples_per_shard) {
    if (!g) { set_error("NULL graph"); return LOGOSKG_EINVAL; }
    if (g->num_shards <= 1) {
        if (shard_of_entity) {
            std::vector<uint32_t> off((size_t)g->E + 1);
            LKG_HIP(hipMemcpy(off.data(), g->out_off, off.size() * 4, hipMemcpyDeviceToHost));
            for (int32_t e = 0; e < g->E; ++e) shard_of_entity[e] = off[(size_t)e + 1] > off[e] ? 0 : -1;
        }
        if (triples_per_shard) triples_per_shard[0] = g->T;
        return LOGOSKG_OK;
    }
    if (shard_of_entity) memcpy(shard_of_entity, g->shard_of.data(), (size_t)g->E * sizeof(int32_t));
    if (triples_per_shard)
        memcpy(triples_per_shard, g->shard_triples.data(), (size_t)g->num_shards * sizeof(int64_t));
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_prefetch_shards(logoskg_graph *g, const int32_t *shards, int32_t n) {
    if (!g || n < 0 || (n > 0 && !shards)) { set_error("bad argument"); return LOGOSKG_EINVAL; }
    if (g->num_shards <= 1 || n == 0) return LOGOSKG_OK;
    ShardSet *ss = (ShardSet *)g->shards;
    if (!ss) { set_error("graph has no shards"); return LOGOSKG_EINTERNAL; }
    for (int32_t i = 0; i < n; ++i)
        if (shards[i] < 0 || shards[i] >= ss->n) {
            set_error("shard %d outside [0, %d)", shards[i], ss->n);
            return LOGOSKG_EINVAL;
        }
    LKG_HIP(hipSetDevice(g->device));
    for (int32_t i = 0; i < n; ++i) {
        int slot = -1;
        LKG_TRY(acquire(g, ss, shards[i], nullptr, &slot));
    }
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_schedule_queries(const logoskg_graph *g, const int64_t *seed_off,
                                                   const int32_t *seeds, int64_t num_queries, int32_t *order) {
    if (!g || !seed_off || !order || num_queries < 0 || num_queries > 0x7fffffff) {
        set_error("bad argument");
        return LOGOSKG_EINVAL;
    }
    if (seed_off[0] != 0) { set_error("seed_off[0] must be 0"); return LOGOSKG_EINVAL; }
    for (int64_t q = 0; q < num_queries; ++q)
        if (seed_off[q + 1] < seed_off[q]) { set_error("seed_off decreases at query %lld", (long long)q); return LOGOSKG_EINVAL; }
    if (seed_off[num_queries] > 0 && !seeds) { set_error("NULL seeds"); return LOGOSKG_EINVAL; }
    for (int64_t i = 0; i < seed_off[num_queries]; ++i)
        if ((uint32_t)seeds[i] >= (uint32_t)g->E) {
            set_error("seed %d at position %lld is out of range", seeds[i], (long long)i);
            return LOGOSKG_EINVAL;
        }
    for (int64_t q = 0; q < num_queries; ++q) order[q] = (int32_t)q;
    if (g->num_shards <= 1) return LOGOSKG_OK;
    // the sub-graphs every query's seeds live in, ascending and distinct
    std::vector<std::vector<int32_t>> need((size_t)num_queries);
    for (int64_t q = 0; q < num_queries; ++q) {
        std::vector<int32_t> &v = need[(size_t)q];
        for (int64_t i = seed_off[q]; i < seed_off[q + 1]; ++i) {
            const int32_t sh = g->shard_of[(size_t)seeds[i]];
            if (sh >= 0) v.push_back(sh);
        }
        std::sort(v.begin(), v.end());
        v.erase(std::unique(v.begin(), v.end()), v.end());
    }
    std::stable_sort(order, order + num_queries,
                     [&](int32_t a, int32_t b) { return need[(size_t)a] < need[(size_t)b]; });
    return LOGOSKG_OK;
}

