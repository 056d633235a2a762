// Active-triple export (Sec. 3.3 "Path reconstruction", Eq. 5-7): T_h of a
// query = the triples whose subject is in level h-1 and whose relation the
// query's whitelist allows, written out with their components.
//
// The level's entity lists (query-major, ascending entity id) come from the
// level-list path; every list entry then stands for one row of SUB.  A degree
// kernel counts the allowed triples of every entry, a device-wide exclusive
// prefix sum (rocPRIM) turns the counts into output positions, and an expansion
// kernel copies the rows: one wavefront per entry, 64 triples per step,
// compacted with a ballot when a whitelist removes some.  The output order is
// therefore (query, subject, triple index).
#include <cstring>

#include <rocprim/device/device_scan.hpp>

#include "common.h"

namespace lkg {

namespace {

constexpr int kBlock = 256;
constexpr long long kMaxBlocks = 1 << 16;

// The query whose list holds position pos of the concatenated level lists: the
// last q in [q0, q1) with level_off[q] <= pos (queries with empty lists share
// their offset with the next one and are skipped that way).
__device__ __forceinline__ int query_of(const long long *__restrict__ level_off, int q0, int q1, long long pos) {
    int lo = q0, hi = q1 - 1;
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

// deg[i] = number of triples of entry i's subject (no whitelist): one thread per entry
__global__ void k_triple_degree(const int32_t *__restrict__ ent, long long n, const uint32_t *__restrict__ out_off,
                                long long *deg) {
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i <= n;
         i += (long long)gridDim.x * blockDim.x) {
        long long d = 0;
        if (i < n) {
            const int32_t s = ent[i];
            d = (long long)(out_off[s + 1] - out_off[s]);
        }
        deg[i] = d;  // deg[n] = 0: the prefix sum leaves the total there
    }
}

// the same with a whitelist: one wavefront per entry counts the allowed triples of the row
__global__ void k_triple_degree_masked(const int32_t *__restrict__ ent, long long n,
                                       const uint32_t *__restrict__ out_off, const uint16_t *__restrict__ out_rel,
                                       const unsigned long long *__restrict__ allow, int W,
                                       const long long *__restrict__ level_off, int q0, int q1, long long *deg) {
    const long long waves = (long long)gridDim.x * (blockDim.x >> 6);
    for (long long i = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6); i <= n; i += waves) {
        long long cnt = 0;
        if (i < n) {
            const int32_t s = ent[i];
            const int q = query_of(level_off, q0, q1, level_off[q0] + i);
            const uint32_t lo = out_off[s], hi = out_off[s + 1];
            for (uint32_t p = lo + (uint32_t)lane(); p < hi; p += 64) cnt += allowed(allow, W, out_rel[p], q) ? 1 : 0;
            cnt = wave_sum(cnt);
        }
        if (lane() == 0) deg[i] = cnt;
    }
}

// picked[j] = first[level_off[q0 + j] - level_off[q0]], j = 0 .. q1 - q0
__global__ void k_pick_offsets(const long long *__restrict__ first, const long long *__restrict__ level_off, int q0,
                               int q1, long long *picked) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j <= q1 - q0) picked[j] = first[level_off[q0 + j] - level_off[q0]];
}

// One wavefront per list entry: copy the (allowed) triples of the subject's row to first[i]..
template <bool MASK>
__global__ void __launch_bounds__(kBlock)
k_triple_expand(const int32_t *__restrict__ ent, long long n, const long long *__restrict__ first,
                const uint32_t *__restrict__ out_off, const int32_t *__restrict__ out_obj,
                const uint16_t *__restrict__ out_rel, const int32_t *__restrict__ out_eid,
                const unsigned long long *__restrict__ allow, int W, const long long *__restrict__ level_off, int q0,
                int q1, int32_t *triple, int32_t *subject, int32_t *relation, int32_t *object) {
    const long long waves = (long long)gridDim.x * (blockDim.x >> 6);
    for (long long i = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6); i < n; i += waves) {
        const int32_t s = ent[i];
        const uint32_t lo = out_off[s], hi = out_off[s + 1];
        long long w = first[i];
        int q = 0;
        if (MASK) q = query_of(level_off, q0, q1, level_off[q0] + i);
        for (uint32_t p0 = lo; p0 < hi; p0 += 64) {
            const uint32_t p = p0 + (uint32_t)lane();
            bool ok = p < hi;
            int rr = 0;
            if (ok) {
                rr = out_rel[p];
                if (MASK) ok = allowed(allow, W, rr, q);
            }
            const unsigned long long b = __ballot(ok);
            if (ok) {
                const long long pos = w + __popcll(b & ((1ull << lane()) - 1ull));
                if (triple) triple[pos] = out_eid[p];
                if (subject) subject[pos] = s;
                if (relation) relation[pos] = rr;
                if (object) object[pos] = out_obj[p];
            }
            w += __popcll(b);
        }
    }
}

unsigned blocks_for(long long items, int per_block) {
    long long b = (items + per_block - 1) / per_block;
    return (unsigned)std::max<long long>(1, std::min<long long>(b, kMaxBlocks));
}

void drop_prepared(logoskg_result *r) {
    r->g->pool.release(r->trip_ent);
    r->g->pool.release(r->trip_off);
    r->trip_ent = nullptr;
    r->trip_off = nullptr;
    r->trip_h = -1;
    r->trip_n = 0;
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
    if (g->num_shards > 1) { set_error("active triples need a resident (unsharded) graph"); return LOGOSKG_EINVAL; }
    LKG_HIP(hipSetDevice(g->device));
    hipStream_t st = (hipStream_t)stream;
    drop_prepared(r);
    LKG_TRY(ensure_out_eid(g, st));
    // level h-1 of every query, then the lists of the range
    std::vector<int64_t> level_off((size_t)r->Q + 1);
    LKG_TRY(logoskg_result_level_offsets(r, h - 1, level_off.data(), stream));
    const int64_t n = level_off[(size_t)q1] - level_off[(size_t)q0];
    const int nq = q1 - q0;
    LKG_TRY(g->pool.alloc((void **)&r->trip_ent, std::max<int64_t>(n, 1) * sizeof(int32_t)));
    LKG_TRY(g->pool.alloc((void **)&r->trip_off, (size_t)(n + 1) * sizeof(long long)));
    LKG_TRY(logoskg_result_level_fetch(r, h - 1, q0, q1, n, r->trip_ent, stream));

    long long *d_deg = nullptr, *d_picked = nullptr;
    void *d_tmp = nullptr;
    auto done = [&](logoskg_status s) {
        g->pool.release(d_deg);
        g->pool.release(d_picked);
        g->pool.release(d_tmp);
        if (s != LOGOSKG_OK) drop_prepared(r);
        return s;
    };
    logoskg_status s;
    if ((s = g->pool.alloc((void **)&d_deg, (size_t)(n + 1) * sizeof(long long))) != LOGOSKG_OK) return done(s);
    if ((s = g->pool.alloc((void **)&d_picked, (size_t)(nq + 1) * sizeof(long long))) != LOGOSKG_OK) return done(s);
    size_t tmp_bytes = 0;
    hipError_t e = rocprim::exclusive_scan(nullptr, tmp_bytes, d_deg, r->trip_off, 0ll, (size_t)(n + 1),
                                           rocprim::plus<long long>(), st);
    if (e == hipSuccess && (s = g->pool.alloc(&d_tmp, std::max<size_t>(tmp_bytes, 8))) != LOGOSKG_OK) return done(s);
    if (e == hipSuccess) {
        if (r->has_mask)
            k_triple_degree_masked<<<dim3(blocks_for(n + 1, kBlock / 64)), dim3(kBlock), 0, st>>>(
                r->trip_ent, n, g->out_off, g->out_rel, r->allow, r->W, r->d_level_off, q0, q1, d_deg);
        else
            k_triple_degree<<<dim3(blocks_for(n + 1, kBlock)), dim3(kBlock), 0, st>>>(r->trip_ent, n, g->out_off,
                                                                                      d_deg);
        e = rocprim::exclusive_scan(d_tmp, tmp_bytes, d_deg, r->trip_off, 0ll, (size_t)(n + 1),
                                    rocprim::plus<long long>(), st);
    }
    std::vector<long long> picked((size_t)nq + 1, 0);
    if (e == hipSuccess) {
        k_pick_offsets<<<dim3((nq + 1 + kBlock - 1) / kBlock), dim3(kBlock), 0, st>>>(r->trip_off, r->d_level_off, q0,
                                                                                      q1, d_picked);
        e = hipGetLastError();
    }
    if (e == hipSuccess)
        e = hipMemcpyAsync(picked.data(), d_picked, (size_t)(nq + 1) * sizeof(long long), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
        set_error("counting the active triples failed: %s", hipGetErrorString(e));
        return done(LOGOSKG_EDEVICE);
    }
    r->trip_off_host.assign(picked.begin(), picked.end());
    r->trip_h = h;
    r->trip_q0 = q0;
    r->trip_q1 = q1;
    r->trip_n = n;
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
    const long long n = r->trip_n;
    dim3 grid(blocks_for(n, kBlock / 64)), block(kBlock);
    {
        ProfScope ps(g->prof, KK_TRIPLES, st);
        if (r->has_mask)
            k_triple_expand<true><<<grid, block, 0, st>>>(r->trip_ent, n, r->trip_off, g->out_off, g->out_obj,
                                                          g->out_rel, g->out_eid, r->allow, r->W, r->d_level_off, q0,
                                                          q1, triple, subject, relation, object);
        else
            k_triple_expand<false><<<grid, block, 0, st>>>(r->trip_ent, n, r->trip_off, g->out_off, g->out_obj,
                                                           g->out_rel, g->out_eid, nullptr, r->W, r->d_level_off, q0,
                                                           q1, triple, subject, relation, object);
    }
    LKG_HIP(hipGetLastError());
    if (g->prof.on) g->prof.acc[KK_TRIPLES].units[3] += need;
    return LOGOSKG_OK;
}
