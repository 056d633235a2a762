// Result side of logoskg_khop: per-query reached counts, the query-major
// (entity, hop, predecessor edge) lists, and the per-query traversed-edge
// counts.
//
// The level planes are entity-major bit matrices; the lists are their
// transpose.  Entities are cut into tiles of 64 (one wavefront of lanes) and
// super tiles of 64 tiles.  A wavefront owns (tile, word): lane v holds the
// word of entity 64*tile+v, and for each of the 64 queries of the word a
// ballot gives the mask of tile entities that query reached - its popcount is
// the tile's count, and the population below a lane is that entity's rank
// inside the tile's run of the query's list.
//
// The predecessor edge (smallest edge id whose subject sits one hop closer and
// whose relation the query allows; the first active triple of Eq. 5-7 in
// edge-id order) is found by walking the object row of the entity in ascending
// edge id with a mask of still unresolved queries, so every (query, entity)
// pair is written once.
#include <algorithm>
#include <climits>

#include "common.h"

namespace lkg {

template <int W>
__device__ __forceinline__ unsigned long long stage_word(unsigned long long (*stage)[W + 1],
                                                         const unsigned long long *__restrict__ plane_tile,
                                                         int wave) {
    // coalesced load of a 64-entity tile of one plane, then lane v takes word `wave` of entity v
    int t = threadIdx.x;
    __syncthreads();
    stage[t / W][t % W] = plane_tile[t];
    __syncthreads();
    return stage[lane()][wave];
}

template <int W>
__global__ void k_count(const unsigned long long *__restrict__ visited, int Qp, uint8_t *tile_cnt) {
    __shared__ unsigned long long stage[64][W + 1];
    long long tile = blockIdx.x;
    int wave = threadIdx.x >> 6;
    unsigned long long x = stage_word<W>(stage, visited + (size_t)tile * 64 * W, wave);
    int mine = 0;
    for (int qq = 0; qq < 64; ++qq) {
        unsigned long long m = __ballot((x >> qq) & 1ull);
        if (lane() == qq) mine = __popcll(m);
    }
    tile_cnt[(size_t)tile * Qp + threadIdx.x] = (uint8_t)mine;
}

__global__ void k_scan_tiles(long long ntiles, int Qp, const uint8_t *__restrict__ tile_cnt,
                             uint16_t *tile_base, uint32_t *super_sum) {
    long long st = blockIdx.x;
    for (int q = threadIdx.x; q < Qp; q += blockDim.x) {
        uint32_t run = 0;
        for (int t = 0; t < kSuperTiles; ++t) {
            long long tile = st * kSuperTiles + t;
            if (tile >= ntiles) break;
            tile_base[(size_t)tile * Qp + q] = (uint16_t)run;
            run += tile_cnt[(size_t)tile * Qp + q];
        }
        super_sum[(size_t)st * Qp + q] = run;
    }
}

// one block: prefix over super tiles for every query, then the prefix over queries
__global__ void k_scan_super(long long nsuper, int Q, int Qp, uint32_t *super_base, long long *reached_off) {
    __shared__ long long total[1024];
    for (int q = threadIdx.x; q < Qp; q += blockDim.x) {
        uint32_t run = 0;
        for (long long st = 0; st < nsuper; ++st) {
            uint32_t x = super_base[(size_t)st * Qp + q];
            super_base[(size_t)st * Qp + q] = run;
            run += x;
        }
        total[q] = q < Q ? (long long)run : 0;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        long long run = 0;
        for (int q = 0; q < Q; ++q) {
            reached_off[q] = run;
            run += total[q];
        }
        for (int q = Q; q <= Qp; ++q) reached_off[q] = run;
    }
}

__device__ __forceinline__ unsigned long long range_bits(int q0, int q1, int w) {
    return query_bits(q1, w) & ~query_bits(q0, w);
}

// Output position of (query q, tile entity vi) given the tile's reached mask of q.
__device__ __forceinline__ long long slot_of(const long long *base, const unsigned long long *mT, int q, int vi) {
    return base[q] + __popcll(mT[q] & ((1ull << vi) - 1ull));
}

struct FillArgs {
    int32_t E;
    int Q, k, q0, q1, hub_min;
    long long plane;   // words per plane
    long long actw;    // uint32 words per active bitmap
    const unsigned long long *visited, *levels, *allow;
    const uint32_t *act;
    const uint16_t *tile_base;
    const uint32_t *super_base;
    const long long *reached_off;
    const uint32_t *in_off;
    const int32_t *in_sub, *in_eid;
    const uint16_t *in_rel;
    const int32_t *hubs;
    long long n_hubs;
    int32_t *entity;
    uint8_t *hop;
    int32_t *pred;
    long long *hub_slot;
    unsigned long long *stats_fill, *stats_hub;  // rows / edges / lines counters or NULL
};

// Ordered walk over 64 in-edges [j0, j0+64) of entity row: resolves bits of
// `rem` (lanes < W hold one word each) in ascending edge order.  `emit(hit,
// eid)` is called by lanes whose word has newly resolved bits.
template <int W, bool MASK, typename Emit>
__device__ __forceinline__ int pred_chunk(uint32_t j0, uint32_t hi, const FillArgs &a,
                                           const uint32_t *__restrict__ act_prev,
                                           const unsigned long long *__restrict__ prev,
                                           unsigned long long &rem, Emit emit) {
    uint32_t j = j0 + lane();
    int s = 0;
    bool cand = false;
    if (j < hi) {
        s = a.in_sub[j];
        cand = (act_prev[s >> 5] >> (s & 31)) & 1u;
    }
    unsigned long long cm = __ballot(cand);
    int gathered = 0;
    while (cm) {
        int c = __ffsll((long long)cm) - 1;
        cm &= cm - 1;
        int sc = __shfl(s, c);
        ++gathered;
        unsigned long long hit = 0;
        if (lane() < W) {
            unsigned long long ln = prev[(size_t)sc * W + lane()];
            if (MASK) ln &= a.allow[(size_t)a.in_rel[j0 + c] * W + lane()];
            hit = ln & rem;
            rem &= ~hit;
        }
        if (wave_any(hit != 0)) {
            int eid = a.in_eid[j0 + c];
            if (hit) emit(hit, eid);
            if (!wave_any(rem != 0)) break;
        }
    }
    return gathered;
}

template <int W, int NB, bool MASK>
__global__ void k_fill(FillArgs a) {
    constexpr int Qp = 64 * W;
    __shared__ unsigned long long stage[64][W + 1];
    __shared__ unsigned long long mT[Qp];
    __shared__ long long base[Qp];
    const long long tile = blockIdx.x;
    const int t = threadIdx.x, wave = t >> 6, v = lane();
    const int e = (int)(tile * 64) + v;

    {   // start of this tile's run in every query's list
        int q = t;
        long long b = 0;
        if (q >= a.q0 && q < a.q1)
            b = a.reached_off[q] - a.reached_off[a.q0] + a.super_base[(size_t)(tile / kSuperTiles) * Qp + q] +
                a.tile_base[(size_t)tile * Qp + q];
        base[q] = b;
    }
    unsigned long long visw = stage_word<W>(stage, a.visited + (size_t)tile * 64 * W, wave);
    unsigned long long hb[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) hb[b] = 0;
    for (int h = 0; h <= a.k; ++h) {  // hop of each bit, bit-sliced: hb[b] = OR of levels with bit b of h set
        unsigned long long x = stage_word<W>(stage, a.levels + (size_t)h * a.plane + (size_t)tile * 64 * W, wave);
#pragma unroll
        for (int b = 0; b < NB; ++b)
            if ((h >> b) & 1) hb[b] |= x;
    }
    unsigned long long mine = 0;
    for (int qq = 0; qq < 64; ++qq) {
        int q = wave * 64 + qq;
        if (q < a.q0 || q >= a.q1) continue;
        bool bit = (visw >> qq) & 1ull;
        unsigned long long m = __ballot(bit);
        if (v == qq) mine = m;
        if (bit) {
            long long pos = base[q] + __popcll(m & ((1ull << v) - 1ull));
            a.entity[pos] = e;
            int hv = 0;
#pragma unroll
            for (int b = 0; b < NB; ++b) hv |= (int)((hb[b] >> qq) & 1ull) << b;
            if (a.hop) a.hop[pos] = (uint8_t)hv;
            if (a.pred && hv == 0) a.pred[pos] = -1;
        }
    }
    mT[t] = mine;
    __syncthreads();
    if (!a.pred) return;

    // predecessor edges: one wavefront per entity of the tile
    const int nwaves = blockDim.x >> 6;
    long long n_rows = 0, n_edges = 0, n_lines = 0;
    for (int vi = wave; vi < 64; vi += nwaves) {
        int ev = (int)(tile * 64) + vi;
        if (ev >= a.E) break;
        uint32_t lo = a.in_off[ev], hi = a.in_off[ev + 1];
        if (lo == hi) continue;
        bool hubrow = (hi - lo) >= (uint32_t)a.hub_min;
        long long hidx = 0;
        if (hubrow) {  // position of ev in the ascending hub list
            long long l = 0, r = a.n_hubs - 1;
            while (l < r) {
                long long mid = (l + r) >> 1;
                if (a.hubs[mid] < ev) l = mid + 1; else r = mid;
            }
            hidx = l;
        }
        for (int h = 1; h <= a.k; ++h) {
            unsigned long long rem = 0;
            if (v < W) rem = a.levels[(size_t)h * a.plane + (size_t)ev * W + v] & range_bits(a.q0, a.q1, v);
            if (!wave_any(rem != 0)) continue;
            if (hubrow) {  // the block-per-hub kernel resolves these; give it the slots
                for (unsigned long long m = rem; m; m &= m - 1) {
                    int q = v * 64 + (__ffsll((long long)m) - 1);
                    long long pos = slot_of(base, mT, q, vi);
                    a.pred[pos] = INT_MAX;
                    a.hub_slot[(size_t)hidx * Qp + q] = pos;
                }
                continue;
            }
            const uint32_t *act_prev = a.act + (size_t)(h - 1) * a.actw;
            const unsigned long long *prev = a.levels + (size_t)(h - 1) * a.plane;
            ++n_rows;
            for (uint32_t j0 = lo; j0 < hi; j0 += 64) {
                n_lines += pred_chunk<W, MASK>(j0, hi, a, act_prev, prev, rem, [&](unsigned long long hit, int eid) {
                    for (unsigned long long m = hit; m; m &= m - 1) {
                        int q = v * 64 + (__ffsll((long long)m) - 1);
                        a.pred[slot_of(base, mT, q, vi)] = eid;
                    }
                });
                n_edges += min((uint32_t)64, hi - j0);
                if (!wave_any(rem != 0)) break;
            }
        }
    }
    if (a.stats_fill && v == 0) {
        if (n_rows) atomicAdd(&a.stats_fill[0], (unsigned long long)n_rows);
        if (n_edges) atomicAdd(&a.stats_fill[1], (unsigned long long)n_edges);
        if (n_lines) atomicAdd(&a.stats_fill[2], (unsigned long long)n_lines);
    }
}

// Hub object rows: one block per row.  The row is walked in steps of
// (waves x 64) edges; inside a step the waves work on disjoint edge ranges in
// parallel and merge with atomicMin, between steps the resolved bits are
// removed, so later steps never override earlier (smaller) edge ids.
template <int W, bool MASK>
__global__ void __launch_bounds__(512) k_pred_hub(FillArgs a) {
    constexpr int Qp = 64 * W;
    __shared__ unsigned long long srem[16];
    const long long hidx = blockIdx.x;
    const int ev = a.hubs[hidx];
    const int t = threadIdx.x, wave = t >> 6, nw = blockDim.x >> 6;
    const uint32_t lo = a.in_off[ev], hi = a.in_off[ev + 1];
    long long n_rows = 0, n_edges = 0, n_lines = 0;
    for (int h = 1; h <= a.k; ++h) {
        __syncthreads();
        if (t < 16)
            srem[t] = t < W ? a.levels[(size_t)h * a.plane + (size_t)ev * W + t] & range_bits(a.q0, a.q1, t) : 0ull;
        __syncthreads();
        const uint32_t *act_prev = a.act + (size_t)(h - 1) * a.actw;
        const unsigned long long *prev = a.levels + (size_t)(h - 1) * a.plane;
        for (uint32_t s0 = lo; s0 < hi; s0 += 64u * nw) {
            unsigned long long rem = lane() < W ? srem[lane()] : 0ull;
            if (!wave_any(rem != 0)) break;  // same decision in every wave
            if (s0 == lo && wave == 0) ++n_rows;
            unsigned long long before = rem;
            uint32_t j0 = s0 + 64u * wave;
            if (j0 < hi) {
                n_lines += pred_chunk<W, MASK>(j0, hi, a, act_prev, prev, rem, [&](unsigned long long hit, int eid) {
                    for (unsigned long long m = hit; m; m &= m - 1) {
                        int q = lane() * 64 + (__ffsll((long long)m) - 1);
                        atomicMin(&a.pred[a.hub_slot[(size_t)hidx * Qp + q]], eid);
                    }
                });
                n_edges += min((uint32_t)64, hi - j0);
            }
            unsigned long long resolved = before & ~rem;
            __syncthreads();
            if (resolved) atomicAnd(&srem[lane()], ~resolved);
            __syncthreads();
        }
    }
    if (a.stats_hub && lane() == 0) {
        if (n_rows) atomicAdd(&a.stats_hub[0], (unsigned long long)n_rows);
        if (n_edges) atomicAdd(&a.stats_hub[1], (unsigned long long)n_edges);
        if (n_lines) atomicAdd(&a.stats_hub[2], (unsigned long long)n_lines);
    }
}

// traversed[q][h] += out-degree of every entity whose level-h bit of q is set
template <int W>
__global__ void k_traversed(int32_t E, int Q, int k, long long plane, long long ntiles,
                            const unsigned long long *__restrict__ levels,
                            const uint32_t *__restrict__ out_off, unsigned long long *trav) {
    __shared__ unsigned long long stage[64][W + 1];
    __shared__ uint32_t sdeg[64];
    const int t = threadIdx.x, w = t >> 6, b = t & 63;
    const long long st = blockIdx.x;
    for (int h = 0; h < k; ++h) {
        unsigned long long acc = 0;
        for (int tt = 0; tt < kSuperTiles; ++tt) {
            long long tile = st * kSuperTiles + tt;
            if (tile >= ntiles) break;
            __syncthreads();
            stage[t / W][t % W] = levels[(size_t)h * plane + (size_t)tile * 64 * W + t];
            if (t < 64) {
                long long e = tile * 64 + t;
                sdeg[t] = e < E ? out_off[e + 1] - out_off[e] : 0u;
            }
            __syncthreads();
            for (int v = 0; v < 64; ++v)
                if ((stage[v][w] >> b) & 1ull) acc += sdeg[v];
        }
        if (acc && t < Q) atomicAdd(&trav[(size_t)t * k + h], acc);
    }
}

logoskg_status count_reached(logoskg_result *r, hipStream_t st) {
    logoskg_graph *g = r->g;
    const int W = r->W, Qp = 64 * W;
    const long long ntiles = r->Epad / kTileEntities;
    const long long nsuper = (ntiles + kSuperTiles - 1) / kSuperTiles;
    LKG_TRY(g->pool.alloc((void **)&r->tile_cnt, (size_t)ntiles * Qp));
    LKG_TRY(g->pool.alloc((void **)&r->tile_base, (size_t)ntiles * Qp * 2));
    LKG_TRY(g->pool.alloc((void **)&r->super_base, (size_t)nsuper * Qp * 4));
    LKG_TRY(g->pool.alloc((void **)&r->d_reached_off, (size_t)(Qp + 1) * 8));
    dim3 grid((unsigned)ntiles), block(Qp);
    {
        ProfScope ps(g->prof, KK_COUNT, st);
        switch (W) {
            case 1: k_count<1><<<grid, block, 0, st>>>(r->visited, Qp, r->tile_cnt); break;
            case 4: k_count<4><<<grid, block, 0, st>>>(r->visited, Qp, r->tile_cnt); break;
            default: k_count<16><<<grid, block, 0, st>>>(r->visited, Qp, r->tile_cnt); break;
        }
        g->prof.acc[KK_COUNT].units[3] += g->prof.on ? r->Epad * W : 0;
    }
    {
        ProfScope ps(g->prof, KK_SCAN, st);
        k_scan_tiles<<<dim3((unsigned)nsuper), dim3(std::min(Qp, 256)), 0, st>>>(ntiles, Qp, r->tile_cnt,
                                                                             r->tile_base, r->super_base);
        k_scan_super<<<dim3(1), dim3(Qp), 0, st>>>(nsuper, r->Q, Qp, r->super_base, (long long *)r->d_reached_off);
    }
    LKG_HIP(hipGetLastError());
    r->reached_off.assign((size_t)r->Q + 1, 0);
    LKG_HIP(hipMemcpyAsync(r->reached_off.data(), r->d_reached_off, (size_t)(r->Q + 1) * 8,
                           hipMemcpyDeviceToHost, st));
    LKG_HIP(hipStreamSynchronize(st));
    r->has_counts = true;
    return LOGOSKG_OK;
}

template <int W, int NB>
static void launch_fill(Profiler &prof, const FillArgs &a, bool mask, long long ntiles, hipStream_t st) {
    dim3 grid((unsigned)ntiles), block(64 * W);
    {
        ProfScope ps(prof, KK_FILL, st);
        if (mask) k_fill<W, NB, true><<<grid, block, 0, st>>>(a);
        else k_fill<W, NB, false><<<grid, block, 0, st>>>(a);
    }
    if (a.pred && a.n_hubs > 0) {
        ProfScope ps(prof, KK_PRED_HUB, st);
        if (mask) k_pred_hub<W, true><<<dim3((unsigned)a.n_hubs), dim3(512), 0, st>>>(a);
        else k_pred_hub<W, false><<<dim3((unsigned)a.n_hubs), dim3(512), 0, st>>>(a);
    }
}

template <int W>
static void launch_fill_w(Profiler &prof, const FillArgs &a, bool mask, long long ntiles, hipStream_t st) {
    int nb = 1;
    while ((1 << nb) <= a.k) ++nb;
    if (nb <= 2) launch_fill<W, 2>(prof, a, mask, ntiles, st);
    else if (nb <= 4) launch_fill<W, 4>(prof, a, mask, ntiles, st);
    else launch_fill<W, 8>(prof, a, mask, ntiles, st);
}

}  // namespace lkg

using namespace lkg;

extern "C" logoskg_status logoskg_result_offsets(const logoskg_result *r, int64_t *reached_off) {
    if (!r || !reached_off) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    if (!r->has_counts) { set_error("result was computed with LOGOSKG_NO_COUNTS"); return LOGOSKG_EINVAL; }
    memcpy(reached_off, r->reached_off.data(), (size_t)(r->Q + 1) * sizeof(int64_t));
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_result_fetch(logoskg_result *r, int32_t q0, int32_t q1, int64_t capacity,
                                               int32_t *entity, uint8_t *hop, int32_t *pred, void *stream) {
    if (!r) { set_error("NULL result"); return LOGOSKG_EINVAL; }
    if (!r->has_counts) { set_error("result was computed with LOGOSKG_NO_COUNTS"); return LOGOSKG_EINVAL; }
    if (q0 < 0 || q1 > r->Q || q0 > q1) { set_error("bad query range [%d, %d)", q0, q1); return LOGOSKG_EINVAL; }
    int64_t need = r->reached_off[(size_t)q1] - r->reached_off[(size_t)q0];
    if (capacity < need) {
        set_error("capacity %lld < %lld entries", (long long)capacity, (long long)need);
        return LOGOSKG_ERANGE;
    }
    if (need == 0) return LOGOSKG_OK;
    if (!entity) { set_error("entity buffer is NULL"); return LOGOSKG_EINVAL; }
    logoskg_graph *g = r->g;
    if (pred && g->num_shards > 1) {
        set_error("predecessor edges need a resident graph");
        return LOGOSKG_EINVAL;
    }
    LKG_HIP(hipSetDevice(g->device));
    hipStream_t st = (hipStream_t)stream;
    const int W = r->W, Qp = 64 * W;
    if (pred && g->in_rows.n_hub > 0 && !r->hub_slot)
        LKG_TRY(g->pool.alloc((void **)&r->hub_slot, (size_t)g->in_rows.n_hub * Qp * 8));
    FillArgs a;
    a.E = g->E; a.Q = r->Q; a.k = r->k; a.q0 = q0; a.q1 = q1; a.hub_min = g->hub_min;
    a.plane = r->Epad * W; a.actw = r->Epad / 32;
    a.visited = (const unsigned long long *)r->visited;
    a.levels = (const unsigned long long *)r->levels;
    a.allow = (const unsigned long long *)r->allow;
    a.act = r->act; a.tile_base = r->tile_base; a.super_base = r->super_base;
    a.reached_off = (const long long *)r->d_reached_off;
    a.in_off = g->in_off; a.in_sub = g->in_sub; a.in_eid = g->in_eid; a.in_rel = g->in_rel;
    a.hubs = g->in_rows.hub; a.n_hubs = g->in_rows.n_hub;
    a.entity = entity; a.hop = hop; a.pred = pred; a.hub_slot = (long long *)r->hub_slot;
    const bool counting = g->prof.counters;
    a.stats_fill = counting ? g->d_ctr + C_STATS + 4 * KK_FILL : nullptr;
    a.stats_hub = counting ? g->d_ctr + C_STATS + 4 * KK_PRED_HUB : nullptr;
    if (counting) LKG_HIP(hipMemsetAsync(g->d_ctr + C_STATS, 0, 4 * KK_NUM * sizeof(unsigned long long), st));
    const long long ntiles = r->Epad / kTileEntities;
    switch (W) {
        case 1: launch_fill_w<1>(g->prof, a, r->has_mask, ntiles, st); break;
        case 4: launch_fill_w<4>(g->prof, a, r->has_mask, ntiles, st); break;
        default: launch_fill_w<16>(g->prof, a, r->has_mask, ntiles, st); break;
    }
    LKG_HIP(hipGetLastError());
    if (g->prof.on) g->prof.acc[KK_FILL].units[3] += need;
    if (counting) {  // measurement mode only: wait for the counters
        LKG_HIP(hipMemcpyAsync(g->h_ctr, g->d_ctr, C_TOTAL * sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
        LKG_HIP(hipStreamSynchronize(st));
        for (int kind : {KK_FILL, KK_PRED_HUB})
            for (int u = 0; u < 3; ++u) g->prof.acc[kind].units[u] += (long long)g->h_ctr[C_STATS + 4 * kind + u];
    }
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_result_traversed(logoskg_result *r, int64_t *traversed, void *stream) {
    if (!r || (r->k > 0 && !traversed)) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    if (r->k == 0) return LOGOSKG_OK;
    logoskg_graph *g = r->g;
    LKG_HIP(hipSetDevice(g->device));
    hipStream_t st = (hipStream_t)stream;
    const int W = r->W;
    const long long ntiles = r->Epad / kTileEntities;
    const long long nsuper = (ntiles + kSuperTiles - 1) / kSuperTiles;
    LKG_HIP(hipMemsetAsync(traversed, 0, (size_t)r->Q * r->k * 8, st));
    dim3 grid((unsigned)nsuper), block(64 * W);
    ProfScope ps(g->prof, KK_TRAVERSED, st);
    unsigned long long *tr = (unsigned long long *)traversed;
    const unsigned long long *lv = (const unsigned long long *)r->levels;
    switch (W) {
        case 1: k_traversed<1><<<grid, block, 0, st>>>(g->E, r->Q, r->k, r->Epad * W, ntiles, lv, g->out_off, tr); break;
        case 4: k_traversed<4><<<grid, block, 0, st>>>(g->E, r->Q, r->k, r->Epad * W, ntiles, lv, g->out_off, tr); break;
        default: k_traversed<16><<<grid, block, 0, st>>>(g->E, r->Q, r->k, r->Epad * W, ntiles, lv, g->out_off, tr); break;
    }
    LKG_HIP(hipGetLastError());
    return LOGOSKG_OK;
}
