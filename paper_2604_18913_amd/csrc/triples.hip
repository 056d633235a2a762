// Active-triple export (Sec. 3.3 "Path reconstruction", Eq. 5-7): T_h of a
// query = the triples whose subject is in level h-1 and whose relation the
// query's whitelist allows, written out with their components.
//
// The level's entity lists (query-major, ascending entity id) come from the
// level-list path; every list entry stands for one row of SUB, and the output
// is the concatenation of those rows with the entries a whitelist forbids
// removed: a stream compaction over the concatenated rows.  So the work is cut
// by position, not by row, and a hub row of 100,000 triples costs as much per
// triple as a row of three:
//   1. row_first[i] = exclusive prefix sum of the row lengths (rocPRIM);
//   2. chunk_entry[c] = the list entry that holds concatenated position
//      c * 256 (written by the entries themselves);
//   3. with a whitelist: every 256-position chunk counts its allowed triples,
//      a second prefix sum gives the chunk's first output position;
//   4. one block per chunk: a thread finds its entry by a binary search between
//      chunk_entry[c] and chunk_entry[c + 1], reads its triple and writes it at
//      its output position (its own position without a whitelist).
// Reads of a row and all writes are contiguous across the lanes of a wavefront.
// The output order is (query, subject, triple index).
#include <cstring>

#include <rocprim/device/device_scan.hpp>

#include "common.h"

namespace lkg {

namespace {

constexpr int kBlock = 256;               // threads per block = concatenated positions per chunk
constexpr long long kMaxBlocks = 1 << 20;
constexpr int kExpandChunks = 8;  // chunks a block of the copy kernel takes together (1: 3.0, 2: 4.0, 4: 4.8, 8: 5.1 TB/s)

// The query whose list holds position pos of the concatenated level lists: the
// last q in [qa, qb] with level_off[q] <= pos (queries with empty lists share
// their offset with the next one and are skipped that way).
__device__ __forceinline__ int query_of(const long long *__restrict__ level_off, int qa, int qb, long long pos) {
    int lo = qa, hi = qb;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (level_off[mid] <= pos) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

__device__ __forceinline__ bool allowed(const unsigned long long *__restrict__ allow, int W, int r, int q) {
    return (allow[(size_t)r * W + (q >> 6)] >> (q & 63)) & 1ull;
}

// len[i] = number of triples of entry i's subject; len[n] = 0 (the prefix sum leaves the total there)
__global__ void k_row_length(const int32_t *__restrict__ ent, long long n, const uint32_t *__restrict__ out_off,
                             long long *len) {
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i <= n;
         i += (long long)gridDim.x * blockDim.x) {
        long long d = 0;
        if (i < n) {
            const int32_t s = ent[i];
            d = (long long)(out_off[s + 1] - out_off[s]);
        }
        len[i] = d;
    }
}

// chunk_entry[c] = the entry whose row holds concatenated position c * kBlock, c = 0 .. nchunks - 1;
// every such position lies in exactly one non-empty row.  chunk_entry[nchunks] = n - 1.
__global__ void k_chunk_entry(const long long *__restrict__ row_first, long long n, long long nchunks,
                              long long *chunk_entry) {
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (long long)gridDim.x * blockDim.x) {
        const long long a = row_first[i], b = row_first[i + 1];
        for (long long c = (a + kBlock - 1) / kBlock; c * kBlock < b; ++c) chunk_entry[c] = i;
        if (i == n - 1) chunk_entry[nchunks] = n - 1;
    }
}

// What the thread at concatenated position x has to copy.
struct Position {
    long long entry;  // list entry, -1 beyond the end
    int32_t s;        // its subject
    uint32_t p;       // index into the arrays of SUB's rows
};

__device__ __forceinline__ Position locate(long long x, long long total, long long c,
                                           const long long *__restrict__ chunk_entry,
                                           const long long *__restrict__ row_first,
                                           const int32_t *__restrict__ ent, const uint32_t *__restrict__ out_off) {
    Position r{-1, 0, 0};
    if (x >= total) return r;
    // the last entry in [chunk_entry[c], chunk_entry[c + 1]] whose row starts at or before x
    long long lo = chunk_entry[c], hi = chunk_entry[c + 1];
    while (lo < hi) {
        const long long mid = (lo + hi + 1) >> 1;
        if (row_first[mid] <= x) lo = mid;
        else hi = mid - 1;
    }
    r.entry = lo;
    r.s = ent[lo];
    r.p = out_off[r.s] + (uint32_t)(x - row_first[lo]);
    return r;
}

// Whitelist test of the triple at position x: the query comes from the entry's place in the level lists.
__device__ __forceinline__ bool position_allowed(const Position &r, const uint16_t *__restrict__ out_rel,
                                                 const unsigned long long *__restrict__ allow, int W,
                                                 const long long *__restrict__ level_off, int q0, int q1) {
    if (r.entry < 0) return false;
    const int q = query_of(level_off, q0, q1 - 1, level_off[q0] + r.entry);
    return allowed(allow, W, out_rel[r.p], q);
}

// The copy of a position is a chain of dependent loads (chunk bounds, search steps, subject, row
// start, with a whitelist the entry's query, then the triple itself), and a kernel with one
// position per thread runs at the rate that latency allows, not at the rate of its bytes.  So a
// thread takes the same position of U consecutive chunks and walks their chains together.
template <int U>
struct Chains {
    long long x[U];    // concatenated position
    long long lo[U];   // its list entry
    bool ok[U];        // the position exists
    int32_t sub[U];    // subject of the entry
    uint32_t p[U];     // index into the arrays of SUB's rows
};

template <int U>
__device__ __forceinline__ void walk_chains(long long c0, long long total, long long nchunks,
                                            const long long *__restrict__ chunk_entry,
                                            const long long *__restrict__ row_first,
                                            const int32_t *__restrict__ ent, const uint32_t *__restrict__ out_off,
                                            Chains<U> &k) {
    long long hi[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const long long c = c0 + u;
        k.x[u] = c * kBlock + threadIdx.x;
        k.ok[u] = c < nchunks && k.x[u] < total;
        k.lo[u] = k.ok[u] ? chunk_entry[c] : 0;
        hi[u] = k.ok[u] ? chunk_entry[c + 1] : 0;
    }
    // the last entry in [lo, hi] whose row starts at or before x
    for (bool open = true; open;) {
        open = false;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (k.lo[u] < hi[u]) {
                const long long mid = (k.lo[u] + hi[u] + 1) >> 1;
                if (row_first[mid] <= k.x[u]) k.lo[u] = mid;
                else hi[u] = mid - 1;
                open |= k.lo[u] < hi[u];
            }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) k.sub[u] = k.ok[u] ? ent[k.lo[u]] : 0;
#pragma unroll
    for (int u = 0; u < U; ++u) k.p[u] = k.ok[u] ? out_off[k.sub[u]] + (uint32_t)(k.x[u] - row_first[k.lo[u]]) : 0u;
}

// ok[u] &= the relation rel[u] of position u is on the whitelist of the entry's query (the last q
// in [q0, q1 - 1] with level_off[q] <= the entry's place in the level lists)
template <int U>
__device__ __forceinline__ void filter_chains(Chains<U> &k, const int32_t *rel,
                                              const unsigned long long *__restrict__ allow, int W,
                                              const long long *__restrict__ level_off, int q0, int q1) {
    int ql[U], qh[U];
    const long long first = level_off[q0];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        ql[u] = q0;
        qh[u] = k.ok[u] ? q1 - 1 : q0;
    }
    for (bool open = true; open;) {
        open = false;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (ql[u] < qh[u]) {
                const int mid = (ql[u] + qh[u] + 1) >> 1;
                if (level_off[mid] <= first + k.lo[u]) ql[u] = mid;
                else qh[u] = mid - 1;
                open |= ql[u] < qh[u];
            }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (k.ok[u]) k.ok[u] = allowed(allow, W, rel[u], ql[u]);
}

// chunk_count[c] = allowed triples among the positions of chunk c; chunk_count[nchunks] = 0
__global__ void __launch_bounds__(kBlock)
k_chunk_count(long long total, long long nchunks, const long long *__restrict__ chunk_entry,
              const long long *__restrict__ row_first, const int32_t *__restrict__ ent,
              const uint32_t *__restrict__ out_off, const uint16_t *__restrict__ out_rel,
              const unsigned long long *__restrict__ allow, int W, const long long *__restrict__ level_off, int q0,
              int q1, long long *chunk_count) {
    constexpr int U = kExpandChunks;
    __shared__ int wave_count[U][kBlock / 64];
    for (long long c0 = (long long)blockIdx.x * U; c0 <= nchunks; c0 += (long long)gridDim.x * U) {  // block-uniform
        Chains<U> k;
        walk_chains<U>(c0, total, nchunks, chunk_entry, row_first, ent, out_off, k);
        int32_t rel[U];
#pragma unroll
        for (int u = 0; u < U; ++u) rel[u] = k.ok[u] ? out_rel[k.p[u]] : 0;
        filter_chains<U>(k, rel, allow, W, level_off, q0, q1);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned long long b = __ballot(k.ok[u]);
            if (lane() == 0) wave_count[u][threadIdx.x >> 6] = __popcll(b);
        }
        __syncthreads();
        if (threadIdx.x < U && c0 + threadIdx.x <= nchunks) {
            int sum = 0;
            for (int w = 0; w < kBlock / 64; ++w) sum += wave_count[threadIdx.x][w];
            chunk_count[c0 + threadIdx.x] = sum;
        }
        __syncthreads();
    }
}

// picked[j] = output position of the first triple of query q0 + j (j = q1 - q0: the total).  Without a
// whitelist that is row_first of the query's first entry; with one, the allowed triples before it.
template <bool MASK>
__global__ void __launch_bounds__(kBlock)
k_pick_offsets(long long total, long long nchunks, const long long *__restrict__ chunk_entry,
               const long long *__restrict__ row_first, const long long *__restrict__ chunk_first,
               const int32_t *__restrict__ ent, const uint32_t *__restrict__ out_off,
               const uint16_t *__restrict__ out_rel, const unsigned long long *__restrict__ allow, int W,
               const long long *__restrict__ level_off, int q0, int q1, long long *picked) {
    __shared__ int wave_count[kBlock / 64];
    const int j = blockIdx.x;  // one block per boundary
    const long long x = row_first[level_off[q0 + j] - level_off[q0]];
    if (!MASK) {
        if (threadIdx.x == 0) picked[j] = x;
        return;
    }
    const long long c = x / kBlock;  // allowed triples of the chunk's positions below x are added
    bool ok = false;
    if (c < nchunks && c * kBlock + threadIdx.x < x) {
        const Position r = locate(c * kBlock + threadIdx.x, total, c, chunk_entry, row_first, ent, out_off);
        ok = position_allowed(r, out_rel, allow, W, level_off, q0, q1);
    }
    const unsigned long long b = __ballot(ok);
    if (lane() == 0) wave_count[threadIdx.x >> 6] = __popcll(b);
    __syncthreads();
    if (threadIdx.x == 0) {
        long long sum = chunk_first[c < nchunks ? c : nchunks];
        for (int w = 0; w < kBlock / 64; ++w) sum += wave_count[w];
        picked[j] = sum;
    }
}

// One block per chunk of kBlock concatenated positions: every thread copies its triple.
template <bool MASK>
__global__ void __launch_bounds__(kBlock)
k_triple_expand(long long total, long long nchunks, const long long *__restrict__ chunk_entry,
                const long long *__restrict__ row_first, const long long *__restrict__ chunk_first,
                const int32_t *__restrict__ ent, const uint32_t *__restrict__ out_off,
                const int32_t *__restrict__ out_obj, const uint16_t *__restrict__ out_rel,
                const int32_t *__restrict__ out_eid, const unsigned long long *__restrict__ allow, int W,
                const long long *__restrict__ level_off, int q0, int q1, int32_t *__restrict__ triple,
                int32_t *__restrict__ subject, int32_t *__restrict__ relation, int32_t *__restrict__ object) {
    constexpr int U = kExpandChunks;
    __shared__ int wave_count[MASK ? U : 1][kBlock / 64];
    for (long long c0 = (long long)blockIdx.x * U; c0 < nchunks; c0 += (long long)gridDim.x * U) {  // block-uniform
        Chains<U> k;
        walk_chains<U>(c0, total, nchunks, chunk_entry, row_first, ent, out_off, k);
        int32_t ve[U], vr[U], vo[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            ve[u] = vr[u] = vo[u] = 0;
            if (k.ok[u]) {
                if (triple) ve[u] = out_eid[k.p[u]];
                if (MASK || relation) vr[u] = out_rel[k.p[u]];
                if (object) vo[u] = out_obj[k.p[u]];
            }
        }
        long long pos[U];
#pragma unroll
        for (int u = 0; u < U; ++u) pos[u] = k.x[u];
        if constexpr (MASK) {
            filter_chains<U>(k, vr, allow, W, level_off, q0, q1);
            unsigned long long b[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                b[u] = __ballot(k.ok[u]);
                if (lane() == 0) wave_count[u][threadIdx.x >> 6] = __popcll(b[u]);
            }
            __syncthreads();
#pragma unroll
            for (int u = 0; u < U; ++u) {
                pos[u] = (c0 + u < nchunks ? chunk_first[c0 + u] : 0) + __popcll(b[u] & ((1ull << lane()) - 1ull));
                for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) pos[u] += wave_count[u][w];
            }
            __syncthreads();  // the counts are rewritten by the next turn
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (k.ok[u]) {
                if (triple) triple[pos[u]] = ve[u];
                if (subject) subject[pos[u]] = k.sub[u];
                if (relation) relation[pos[u]] = vr[u];
                if (object) object[pos[u]] = vo[u];
            }
    }
}

unsigned blocks_for(long long items, int per_block) {
    long long b = (items + per_block - 1) / per_block;
    return (unsigned)std::max<long long>(1, std::min<long long>(b, kMaxBlocks));
}

void drop_prepared(logoskg_result *r) {
    for (void *p : {(void *)r->trip_ent, (void *)r->trip_off, (void *)r->trip_chunk_entry, (void *)r->trip_chunk_first})
        r->g->pool.release(p);
    r->trip_ent = nullptr;
    r->trip_off = nullptr;
    r->trip_chunk_entry = nullptr;
    r->trip_chunk_first = nullptr;
    r->trip_h = -1;
    r->trip_n = 0;
    r->trip_total = 0;
    r->trip_off_host.clear();
}

}  // namespace

}  // namespace lkg

using namespace lkg;

extern "C" logoskg_status logoskg_result_triples_offsets(logoskg_result *r, int32_t h, int32_t q0, int32_t q1,
                                                         int64_t *triple_off, void *stream) {
    if (!r || !triple_off) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    if (h < 1 || h > r->k) { set_error("hop %d outside [1, %d]", h, r->k); return LOGOSKG_EINVAL; }
    if (q0 < 0 || q1 > r->Q || q0 > q1) { set_error("bad query range [%d, %d)", q0, q1); return LOGOSKG_EINVAL; }
    logoskg_graph *g = r->g;
    const int32_t *out_obj = g->out_obj;
    const uint16_t *out_rel = g->out_rel;
    if (g->num_shards > 1 && !shard_out_arrays(g, &out_obj, &out_rel)) {
        set_error("active triples of a sharded graph need its shards in pinned host memory (not in files)");
        return LOGOSKG_EINVAL;
    }
    LKG_HIP(hipSetDevice(g->device));
    hipStream_t st = (hipStream_t)stream;
    r->last_stream = st;
    drop_prepared(r);
    LKG_TRY(ensure_out_eid(g, st));
    // level h-1 of every query, then the lists of the range
    std::vector<int64_t> level_off((size_t)r->Q + 1);
    LKG_TRY(logoskg_result_level_offsets(r, h - 1, level_off.data(), stream));
    const int64_t n = level_off[(size_t)q1] - level_off[(size_t)q0];
    const int nq = q1 - q0;
    const bool mask = r->has_mask;

    long long *d_len = nullptr, *d_count = nullptr, *d_picked = nullptr;
    void *d_tmp = nullptr;
    auto done = [&](logoskg_status s) {
        for (void *p : {(void *)d_len, (void *)d_count, (void *)d_picked, d_tmp}) g->pool.release(p);
        if (s != LOGOSKG_OK) drop_prepared(r);
        return s;
    };
    auto check = [&](hipError_t e, const char *what) {
        if (e == hipSuccess) return LOGOSKG_OK;
        set_error("%s failed: %s", what, hipGetErrorString(e));
        return e == hipErrorOutOfMemory ? LOGOSKG_ENOMEM : LOGOSKG_EDEVICE;
    };
    // exclusive prefix sum of `count` int64 values through rocPRIM, temporary storage from the pool
    auto prefix_sum = [&](long long *in, long long *out, size_t count) -> logoskg_status {
        size_t bytes = 0;
        logoskg_status s2 = check(rocprim::exclusive_scan(nullptr, bytes, in, out, 0ll, count,
                                                          rocprim::plus<long long>(), st), "sizing the prefix sum");
        if (s2 != LOGOSKG_OK) return s2;
        g->pool.release(d_tmp);
        d_tmp = nullptr;
        if ((s2 = g->pool.alloc(&d_tmp, std::max<size_t>(bytes, 8))) != LOGOSKG_OK) return s2;
        return check(rocprim::exclusive_scan(d_tmp, bytes, in, out, 0ll, count, rocprim::plus<long long>(), st),
                     "prefix sum");
    };
    logoskg_status s;
    if ((s = g->pool.alloc((void **)&r->trip_ent, std::max<int64_t>(n, 1) * sizeof(int32_t))) != LOGOSKG_OK ||
        (s = g->pool.alloc((void **)&r->trip_off, (size_t)(n + 1) * sizeof(long long))) != LOGOSKG_OK ||
        (s = g->pool.alloc((void **)&d_len, (size_t)(n + 1) * sizeof(long long))) != LOGOSKG_OK ||
        (s = g->pool.alloc((void **)&d_picked, (size_t)(nq + 1) * sizeof(long long))) != LOGOSKG_OK)
        return done(s);
    if ((s = logoskg_result_level_fetch(r, h - 1, q0, q1, n, r->trip_ent, stream)) != LOGOSKG_OK) return done(s);

    // 1. where every entry's row starts in the concatenation of the rows
    k_row_length<<<dim3(blocks_for(n + 1, kBlock)), dim3(kBlock), 0, st>>>(r->trip_ent, n, g->out_off, d_len);
    if ((s = prefix_sum(d_len, r->trip_off, (size_t)n + 1)) != LOGOSKG_OK) return done(s);
    long long total = 0;
    if ((s = check(hipMemcpyAsync(&total, r->trip_off + n, sizeof(total), hipMemcpyDeviceToHost, st), "copy")) !=
            LOGOSKG_OK ||
        (s = check(hipStreamSynchronize(st), "row lengths")) != LOGOSKG_OK)
        return done(s);
    const long long nchunks = (total + kBlock - 1) / kBlock;
    // 2. the entry behind the first position of every chunk
    if ((s = g->pool.alloc((void **)&r->trip_chunk_entry, (size_t)(nchunks + 1) * sizeof(long long))) != LOGOSKG_OK)
        return done(s);
    if (n > 0)
        k_chunk_entry<<<dim3(blocks_for(n, kBlock)), dim3(kBlock), 0, st>>>(r->trip_off, n, nchunks,
                                                                            r->trip_chunk_entry);
    // 3. with a whitelist: allowed triples per chunk and their prefix sums
    if (mask) {
        if ((s = g->pool.alloc((void **)&d_count, (size_t)(nchunks + 1) * sizeof(long long))) != LOGOSKG_OK ||
            (s = g->pool.alloc((void **)&r->trip_chunk_first, (size_t)(nchunks + 1) * sizeof(long long))) != LOGOSKG_OK)
            return done(s);
        k_chunk_count<<<dim3(blocks_for((nchunks + kExpandChunks) / kExpandChunks, 1)), dim3(kBlock), 0, st>>>(
            total, nchunks, r->trip_chunk_entry, r->trip_off, r->trip_ent, g->row_begin, out_rel, r->allow, r->W,
            r->d_level_off, q0, q1, d_count);
        if ((s = prefix_sum(d_count, r->trip_chunk_first, (size_t)nchunks + 1)) != LOGOSKG_OK) return done(s);
        k_pick_offsets<true><<<dim3(nq + 1), dim3(kBlock), 0, st>>>(
            total, nchunks, r->trip_chunk_entry, r->trip_off, r->trip_chunk_first, r->trip_ent, g->row_begin, out_rel,
            r->allow, r->W, r->d_level_off, q0, q1, d_picked);
    } else {
        k_pick_offsets<false><<<dim3(nq + 1), dim3(kBlock), 0, st>>>(
            total, nchunks, r->trip_chunk_entry, r->trip_off, nullptr, r->trip_ent, g->row_begin, out_rel, nullptr,
            r->W, r->d_level_off, q0, q1, d_picked);
    }
    std::vector<long long> picked((size_t)nq + 1, 0);
    if ((s = check(hipGetLastError(), "launch")) != LOGOSKG_OK ||
        (s = check(hipMemcpyAsync(picked.data(), d_picked, (size_t)(nq + 1) * sizeof(long long),
                                  hipMemcpyDeviceToHost, st), "copy")) != LOGOSKG_OK ||
        (s = check(hipStreamSynchronize(st), "counting the active triples")) != LOGOSKG_OK)
        return done(s);
    r->trip_off_host.assign(picked.begin(), picked.end());
    r->trip_h = h;
    r->trip_q0 = q0;
    r->trip_q1 = q1;
    r->trip_n = n;
    r->trip_total = total;
    for (int j = 0; j <= nq; ++j) triple_off[j] = (int64_t)picked[(size_t)j];
    return done(LOGOSKG_OK);
}

extern "C" logoskg_status logoskg_result_triples_fetch(logoskg_result *r, int32_t h, int32_t q0, int32_t q1,
                                                       int64_t capacity, int32_t *triple, int32_t *subject,
                                                       int32_t *relation, int32_t *object, void *stream) {
    if (!r) { set_error("NULL result"); return LOGOSKG_EINVAL; }
    if (r->trip_h != h || r->trip_q0 != q0 || r->trip_q1 != q1 || h < 1) {
        set_error("hop %d of the queries [%d, %d) was not prepared: call logoskg_result_triples_offsets for it first",
                  h, q0, q1);
        return LOGOSKG_EINVAL;
    }
    if (r->level_counted != h - 1) {
        set_error("level %d was counted again after the active triples of hop %d were prepared", r->level_counted, h);
        return LOGOSKG_EINVAL;
    }
    const int64_t need = r->trip_off_host.back();
    if (capacity < need) {
        set_error("capacity %lld < %lld triples", (long long)capacity, (long long)need);
        return LOGOSKG_ERANGE;
    }
    if (need == 0 || (!triple && !subject && !relation && !object)) return LOGOSKG_OK;
    logoskg_graph *g = r->g;
    LKG_HIP(hipSetDevice(g->device));
    hipStream_t st = (hipStream_t)stream;
    r->last_stream = st;
    const long long total = r->trip_total, nchunks = (total + kBlock - 1) / kBlock;
    const int32_t *out_obj = g->out_obj;
    const uint16_t *out_rel = g->out_rel;
    if (g->num_shards > 1 && !shard_out_arrays(g, &out_obj, &out_rel)) {
        set_error("active triples of a sharded graph need its shards in pinned host memory (not in files)");
        return LOGOSKG_EINVAL;
    }
    dim3 grid(blocks_for((nchunks + kExpandChunks - 1) / kExpandChunks, 1)), block(kBlock);
    {
        ProfScope ps(g->prof, KK_TRIPLES, st);
        if (r->has_mask)
            k_triple_expand<true><<<grid, block, 0, st>>>(total, nchunks, r->trip_chunk_entry, r->trip_off,
                                                          r->trip_chunk_first, r->trip_ent, g->row_begin, out_obj,
                                                          out_rel, g->out_eid, r->allow, r->W, r->d_level_off, q0,
                                                          q1, triple, subject, relation, object);
        else
            k_triple_expand<false><<<grid, block, 0, st>>>(total, nchunks, r->trip_chunk_entry, r->trip_off, nullptr,
                                                           r->trip_ent, g->row_begin, out_obj, out_rel, g->out_eid,
                                                           nullptr, r->W, r->d_level_off, q0, q1, triple, subject,
                                                           relation, object);
    }
    LKG_HIP(hipGetLastError());
    if (g->prof.on) {
        g->prof.acc[KK_TRIPLES].units[0] += r->trip_n;  // rows of SUB copied
        g->prof.acc[KK_TRIPLES].units[1] += total;      // triples read
        g->prof.acc[KK_TRIPLES].units[3] += need;       // triples written
    }
    return LOGOSKG_OK;
}
