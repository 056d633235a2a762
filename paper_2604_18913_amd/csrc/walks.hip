// Bulk export of complete paths (paper Sec. 3.3, "Path reconstruction": the
// active triples of hop 1 are extended hop by hop, whenever the object of a
// triple is the subject of a triple of the next hop, into complete paths of
// length k; Eq. 5-7).
//
// For one query and a length d this file lists EVERY chain (t_1, .., t_d) of
// allowed triples with s_{t_1} a seed, o_{t_i} = s_{t_{i+1}} and the subject of
// t_i in level i-1 -- on a LOGOSKG_WALK_EXACT result all walks of d triples from
// a seed, on a minimum-hop result all shortest paths to the entities at hop d --
// without a bound per target: the chains are numbered, and a caller fetches any
// range of numbers (a page) into a buffer of its own.
//
// Order: by target (ascending entity id), chains of one target ordered
// lexicographically by (t_d, t_{d-1}, .., t_1), the order of logoskg_paths and
// logoskg_walks.  Numbering needs no enumeration: c_0[v] = 1 for the seeds,
// c_h[v] = sum over the allowed triples (s, r, v) of c_{h-1}[s] counts the chains
// that end in v after h triples (c_{h-1} is zero outside level h-1), and the
// running sums of a row of OBJ say which chain numbers pass through each of its
// triples.  Chain number x is then decoded by d binary searches, one thread per
// chain, whatever the degree of the entities on it.
#include <rocprim/device/device_scan.hpp>

#include "common.h"

namespace lkg {

// counts stay below 2^56 (7.2 x 10^16): 64 of them add up without wrapping, so one check per
// 64 row entries is enough
constexpr unsigned long long kWalkCountLimit = 1ull << 56;

__device__ __forceinline__ unsigned long long wave_incl_scan64(unsigned long long v) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long y = shfl_up64(v, d);
        if (lane() >= d) v += y;
    }
    return v;
}

__global__ void __launch_bounds__(256)
k_walk_seeds(int32_t E, int W, int w, unsigned long long bit, const unsigned long long *__restrict__ level0,
             unsigned long long *__restrict__ cnt0) {
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < E) cnt0[e] = (level0[(size_t)e * W + w] & bit) ? 1ull : 0ull;
}

// One hop of the count: a wavefront takes 64 consecutive entities, and walks the object row of each
// one that is in level h of the query, 64 entries at a time.  cum[j] = chains that pass through the
// row's entries before j (exclusive running sum inside the row), cnt_cur[v] = the row's total.
template <bool MASK>
__global__ void __launch_bounds__(256)
k_walk_count(int32_t E, int W, int w, unsigned long long bit, const unsigned long long *__restrict__ level_h,
             const unsigned long long *__restrict__ allow, const uint32_t *__restrict__ in_off,
             const int32_t *__restrict__ in_sub, const uint16_t *__restrict__ in_rel,
             const unsigned long long *__restrict__ cnt_prev, unsigned long long *__restrict__ cnt_cur,
             unsigned long long *__restrict__ cum, unsigned int *overflow) {
    const long long waves = (long long)gridDim.x * (blockDim.x >> 6);
    const long long groups = ((long long)E + 63) / 64;
    for (long long gidx = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6); gidx < groups; gidx += waves) {
        const long long e = gidx * 64 + lane();
        const bool in = e < E && (level_h[(size_t)e * W + w] & bit) != 0ull;
        unsigned long long todo = __ballot(in);
        while (todo) {  // wave-uniform
            const int l = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            const long long v = gidx * 64 + l;
            const uint32_t lo = in_off[v], hi = in_off[v + 1];
            unsigned long long running = 0;
            for (uint32_t j0 = lo; j0 < hi; j0 += 64) {
                const uint32_t j = j0 + (uint32_t)lane();
                unsigned long long c = 0;
                if (j < hi) {
                    bool ok = true;
                    if (MASK) ok = (allow[(size_t)in_rel[j] * W + w] & bit) != 0ull;
                    if (ok) c = cnt_prev[in_sub[j]];
                }
                const unsigned long long incl = wave_incl_scan64(c);
                if (j < hi) cum[j] = running + (incl - c);
                running += shfl64(incl, 63);
                if (running >= kWalkCountLimit) {  // reported by the host; the tables are not used then
                    running = kWalkCountLimit - 1;
                    if (lane() == 0) atomicOr(overflow, 1u);
                }
            }
            if (lane() == 0) cnt_cur[v] = running;
        }
    }
}

// pref[0] = 0 and the running sum over the entities must not have wrapped
__global__ void __launch_bounds__(256)
k_walk_check_prefix(int32_t E, unsigned long long *pref, unsigned int *overflow) {
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e == 0) pref[0] = 0ull;
    if (e >= 1 && e < E && pref[e + 1] < pref[e]) atomicOr(overflow, 1u);
}

// One thread per chain of the page: the target from the prefix over the entities, then one
// triple per hop, from the last to the first, by a binary search in the running sums of the row.
__global__ void __launch_bounds__(256)
k_walk_page(long long first, long long count, int d, int32_t E, long long T, const unsigned long long *__restrict__ pref,
            const unsigned long long *__restrict__ cum, const uint32_t *__restrict__ in_off,
            const int32_t *__restrict__ in_sub, const int32_t *__restrict__ in_eid, int32_t *__restrict__ walk_edges,
            int32_t *__restrict__ walk_target) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    unsigned long long x = (unsigned long long)(first + i);
    // the last entity whose prefix is <= x (it has at least one chain: x < pref[E])
    long long a = 0, b = E;  // pref[a] <= x < pref[b]
    while (b - a > 1) {
        const long long m = (a + b) >> 1;
        if (pref[m] <= x) a = m; else b = m;
    }
    int32_t v = (int32_t)a;
    x -= pref[a];
    if (walk_target) walk_target[i] = v;
    for (int h = d; h >= 1; --h) {
        const unsigned long long *c = cum + (size_t)(h - 1) * (size_t)T;
        uint32_t lo = in_off[v], hi = in_off[v + 1];  // c[lo] = 0 <= x, and x < the row's total
        while (hi - lo > 1) {
            const uint32_t m = lo + ((hi - lo) >> 1);
            if (c[m] <= x) lo = m; else hi = m;
        }
        walk_edges[(size_t)i * d + (h - 1)] = in_eid[lo];
        x -= c[lo];
        v = in_sub[lo];
    }
}

void drop_walk_tables(logoskg_result *r) {
    logoskg_graph *g = r->g;
    r->walk_q = r->walk_d = -1;
    r->walk_total = 0;
    if (!r->walk_cnt && !r->walk_cum && !r->walk_pref) return;
    void *ptrs[] = {r->walk_cnt, r->walk_cum, r->walk_pref};
    const bool zeroed[3] = {false, false, false};
    g->pool.release_after(ptrs, zeroed, 3, r->last_stream);
    r->walk_cnt = r->walk_cum = r->walk_pref = nullptr;
}

static logoskg_status prepare_walk_tables(logoskg_result *r, int q, int d, hipStream_t st) {
    logoskg_graph *g = r->g;
    if (r->walk_q == q && r->walk_d == d) return LOGOSKG_OK;
    drop_walk_tables(r);
    const int W = r->W, w = q >> 6;
    const unsigned long long bit = 1ull << (q & 63);
    const int32_t E = g->E;
    const size_t Epad = (size_t)r->Epad, T = (size_t)std::max<int64_t>(g->T, 1);
    const int32_t *in_sub = g->in_sub, *in_eid = g->in_eid;
    const uint16_t *in_rel = g->in_rel;
    if (g->num_shards > 1 && !shard_in_arrays(g, &in_sub, &in_rel, &in_eid)) {
        set_error("the object-sorted triples of the sharded graph are not available");
        return LOGOSKG_EINTERNAL;
    }
    // cnt: d + 1 levels, then one word of flags; cum: d rows of T; pref: E + 1
    LKG_TRY(g->pool.alloc((void **)&r->walk_cnt, ((size_t)(d + 1) * Epad + 8) * 8, st));
    LKG_TRY(g->pool.alloc((void **)&r->walk_cum, (size_t)std::max(d, 1) * T * 8, st));
    LKG_TRY(g->pool.alloc((void **)&r->walk_pref, (Epad + 8) * 8, st));
    unsigned int *overflow = (unsigned int *)(r->walk_cnt + (size_t)(d + 1) * Epad);
    LKG_HIP(hipMemsetAsync(r->walk_cnt, 0, ((size_t)(d + 1) * Epad + 8) * 8, st));
    const size_t plane = Epad * (size_t)W;
    {
        ProfScope ps(g->prof, KK_PATHS, st);
        k_walk_seeds<<<dim3((unsigned)((E + 255) / 256)), dim3(256), 0, st>>>(E, W, w, bit, r->levels, r->walk_cnt);
        const unsigned nb = (unsigned)std::min<long long>(4096, std::max<long long>(1, ((long long)E + 255) / 256));
        for (int h = 1; h <= d; ++h) {
            const unsigned long long *lvl = r->levels + plane * (size_t)h;
            unsigned long long *prev = r->walk_cnt + (size_t)(h - 1) * Epad, *cur = r->walk_cnt + (size_t)h * Epad;
            unsigned long long *cum = r->walk_cum + (size_t)(h - 1) * T;
            if (r->has_mask)
                k_walk_count<true><<<dim3(nb), dim3(256), 0, st>>>(E, W, w, bit, lvl, r->allow, g->in_off, in_sub, in_rel,
                                                                   prev, cur, cum, overflow);
            else
                k_walk_count<false><<<dim3(nb), dim3(256), 0, st>>>(E, W, w, bit, lvl, nullptr, g->in_off, in_sub, in_rel,
                                                                    prev, cur, cum, overflow);
        }
    }
    LKG_HIP(hipGetLastError());
    // pref[e + 1] = chains that end in an entity <= e
    const unsigned long long *last = r->walk_cnt + (size_t)d * Epad;
    size_t bytes = 0;
    auto check = [&](hipError_t e, const char *what) -> logoskg_status {
        if (e != hipSuccess) { set_error("%s failed: %s", what, hipGetErrorString(e)); return LOGOSKG_EDEVICE; }
        return LOGOSKG_OK;
    };
    LKG_TRY(check(rocprim::inclusive_scan(nullptr, bytes, last, r->walk_pref + 1, (size_t)E,
                                          rocprim::plus<unsigned long long>(), st), "sizing the prefix sum"));
    void *tmp = nullptr;
    LKG_TRY(g->pool.alloc(&tmp, std::max<size_t>(bytes, 8), st));
    logoskg_status s = check(rocprim::inclusive_scan(tmp, bytes, last, r->walk_pref + 1, (size_t)E,
                                                     rocprim::plus<unsigned long long>(), st), "prefix sum");
    {
        void *ptrs[] = {tmp};
        const bool z[1] = {false};
        g->pool.release_after(ptrs, z, 1, st);
    }
    LKG_TRY(s);
    k_walk_check_prefix<<<dim3((unsigned)((E + 255) / 256)), dim3(256), 0, st>>>(E, r->walk_pref, overflow);
    LKG_HIP(hipGetLastError());
    unsigned long long total = 0;
    unsigned int ovf = 0;
    LKG_HIP(hipMemcpyAsync(&total, r->walk_pref + E, 8, hipMemcpyDeviceToHost, st));
    LKG_HIP(hipMemcpyAsync(&ovf, overflow, 4, hipMemcpyDeviceToHost, st));
    LKG_HIP(hipStreamSynchronize(st));
    if (ovf || total >= (1ull << 62)) {
        drop_walk_tables(r);
        set_error("query %d has 2^56 or more chains of %d triples into one entity: too many to number", q, d);
        return LOGOSKG_ERANGE;
    }
    r->walk_q = q;
    r->walk_d = d;
    r->walk_total = (int64_t)total;
    return LOGOSKG_OK;
}

}  // namespace lkg

using namespace lkg;

extern "C" logoskg_status logoskg_result_walks_count(logoskg_result *r, int32_t query, int32_t length, int64_t *total,
                                                     void *stream) {
    if (!r || !total) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    if (query < 0 || query >= r->Q) { set_error("query %d outside [0, %d)", query, r->Q); return LOGOSKG_EINVAL; }
    if (length < 0 || length > r->k) { set_error("length %d outside [0, %d]", length, r->k); return LOGOSKG_EINVAL; }
    logoskg_graph *g = r->g;
    LKG_HIP(hipSetDevice(g->device));
    hipStream_t st = (hipStream_t)stream;
    r->last_stream = st;
    LKG_TRY(prepare_walk_tables(r, query, length, st));
    *total = r->walk_total;
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_result_walks_fetch(logoskg_result *r, int32_t query, int32_t length, int64_t first,
                                                     int64_t count, int32_t *walk_edges, int32_t *walk_target,
                                                     void *stream) {
    if (!r) { set_error("NULL result"); return LOGOSKG_EINVAL; }
    if (r->walk_q != query || r->walk_d != length || query < 0) {
        set_error("the chains of %d triples of query %d were not counted: call logoskg_result_walks_count for them first",
                  length, query);
        return LOGOSKG_EINVAL;
    }
    if (first < 0 || count < 0 || first + count > r->walk_total) {
        set_error("chains [%lld, %lld) outside [0, %lld)", (long long)first, (long long)(first + count),
                  (long long)r->walk_total);
        return LOGOSKG_ERANGE;
    }
    if (count == 0) return LOGOSKG_OK;
    if (count > (1ll << 36)) { set_error("at most 2^36 chains per call"); return LOGOSKG_ERANGE; }
    if ((length > 0 && !walk_edges) || (length == 0 && !walk_target)) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    logoskg_graph *g = r->g;
    LKG_HIP(hipSetDevice(g->device));
    hipStream_t st = (hipStream_t)stream;
    r->last_stream = st;
    const int32_t *in_sub = g->in_sub, *in_eid = g->in_eid;
    const uint16_t *in_rel = g->in_rel;
    if (g->num_shards > 1 && !shard_in_arrays(g, &in_sub, &in_rel, &in_eid)) {
        set_error("the object-sorted triples of the sharded graph are not available");
        return LOGOSKG_EINTERNAL;
    }
    ProfScope ps(g->prof, KK_PATHS, st);
    k_walk_page<<<dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st>>>(
        first, count, length, g->E, std::max<int64_t>(g->T, 1), r->walk_pref, r->walk_cum, g->in_off, in_sub, in_eid,
        walk_edges, walk_target);
    LKG_HIP(hipGetLastError());
    return LOGOSKG_OK;
}
