// Result side of logoskg_khop: per-query reached counts, the query-major
// (entity, hop, predecessor edge) lists, and the per-query traversed-edge
// counts.
//
// The level planes are entity-major bit matrices; the lists are their
// transpose.  Entities are cut into tiles of 64 (one wavefront of lanes), super
// tiles of 16 tiles and mega tiles of 64 super tiles.  A wavefront owns one
// word (64 queries) of a tile: lane v holds that word of entity 64*tile+v, and
// for each query a ballot gives the mask of tile entities the query reached -
// its popcount is the tile's count, the population below a lane is the
// entity's rank inside the tile's run of the query's list.
//
//   count : per (query, tile) counts -> nested exclusive prefixes -> offsets
//   lists : one block per super tile compacts the (entity, hop) entries of each
//           query in LDS and writes them as whole 64-lane stores
//   pred  : the predecessor edge (smallest edge id whose subject sits one hop
//           closer and whose relation the query allows - the first active
//           triple of Eq. 5-7 in edge-id order) is found by walking the object
//           row of the entity in ascending edge id with a mask of still
//           unresolved queries, so every (query, entity) pair is written once.
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

// blocks are dealt round-robin to the 8 XCDs; give every XCD a contiguous run of
// tiles so that neighbouring tiles (which write neighbouring list entries) share
// an L2
__device__ __forceinline__ long long xcd_contiguous(long long block, long long nblocks) {
    long long per = (nblocks + 7) / 8;
    return (block & 7) * per + (block >> 3);
}

// ---------------------------------------------------------------- counts
// One block per super tile, one wavefront per word: tile_base[tile][q] = entities
// query q reached in the earlier tiles of the super tile, super_sum[st][q] = in
// the whole super tile.
template <int W>
__global__ void k_count(const unsigned long long *__restrict__ visited, long long ntiles, uint16_t *tile_base,
                        uint32_t *super_sum) {
    constexpr int Qp = 64 * W;
    __shared__ unsigned long long stage[64][W + 1];
    const long long st = blockIdx.x;
    const int wave = threadIdx.x >> 6;
    int run = 0;
    for (int i = 0; i < kSuperTiles; ++i) {
        long long tile = st * kSuperTiles + i;
        if (tile >= ntiles) break;
        unsigned long long x = stage_word<W>(stage, visited + (size_t)tile * 64 * W, wave);
        tile_base[(size_t)tile * Qp + threadIdx.x] = (uint16_t)run;
        int mine = 0;
        if (wave_any(x != 0)) {
            for (int qq = 0; qq < 64; ++qq) {
                unsigned long long m = __ballot((x >> qq) & 1ull);
                if (lane() == qq) mine = __popcll(m);
            }
        }
        run += mine;
    }
    super_sum[(size_t)st * Qp + threadIdx.x] = (uint32_t)run;
}

// exclusive prefix of `sum` over groups of `group` consecutive rows; total per group to `up`
__global__ void k_scan_level(long long nrows, int group, int Qp, uint32_t *sum_to_base, uint32_t *up) {
    long long g = blockIdx.x;
    for (int q = threadIdx.x; q < Qp; q += blockDim.x) {
        uint32_t run = 0;
        for (int t = 0; t < group; ++t) {
            long long row = g * group + t;
            if (row >= nrows) break;
            uint32_t x = sum_to_base[(size_t)row * Qp + q];
            sum_to_base[(size_t)row * Qp + q] = run;
            run += x;
        }
        up[(size_t)g * Qp + q] = run;
    }
}

// one block: prefix over mega tiles for every query, then the prefix over queries
__global__ void k_scan_top(long long nmega, int Q, int Qp, uint32_t *mega_base, long long *reached_off) {
    __shared__ long long total[1024];
    for (int q = threadIdx.x; q < Qp; q += blockDim.x) {
        long long run = 0;
        for (long long m = 0; m < nmega; ++m) {
            uint32_t x = mega_base[(size_t)m * Qp + q];
            mega_base[(size_t)m * Qp + q] = (uint32_t)run;
            run += x;
        }
        total[q] = q < Q ? run : 0;
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

// position of a super tile's first entry in the list of query q (relative to query q0's start)
__device__ __forceinline__ long long super_start(const FillArgs &a, long long st, int Qp, int q) {
    return a.reached_off[q] - a.reached_off[a.q0] + a.mega_base[(size_t)(st / kMegaSupers) * Qp + q] +
           a.super_base[(size_t)st * Qp + q];
}

// ---------------------------------------------------------------- entity / hop lists
// One block per super tile (1024 entities), one wavefront per word.  The wave
// keeps its word of all 16 tiles in registers (visited and the bit-sliced hop
// number), and for one query at a time compacts the reached entities into LDS,
// then streams them out with full-width stores.
template <int W, int NB>
__global__ void __launch_bounds__(64 * W) k_lists(FillArgs a) {
    constexpr int Qp = 64 * W;
    __shared__ unsigned long long stage[64][W + 1];
    __shared__ uint16_t s_ent[W][kSuperTiles * 64];
    __shared__ uint8_t s_hop[W][kSuperTiles * 64];
    const long long st = blockIdx.x;
    const int wave = threadIdx.x >> 6, v = lane();
    unsigned long long visw[kSuperTiles];
    unsigned long long hb[NB][kSuperTiles];
#pragma unroll
    for (int i = 0; i < kSuperTiles; ++i) {
        long long tile = st * kSuperTiles + i;
        visw[i] = 0;
#pragma unroll
        for (int b = 0; b < NB; ++b) hb[b][i] = 0;
        if (tile < a.ntiles) {  // block-uniform
            visw[i] = stage_word<W>(stage, a.visited + (size_t)tile * 64 * W, wave);
            for (int h = 1; h <= a.k; ++h) {  // hop number of each bit, bit-sliced over NB words
                unsigned long long x =
                    stage_word<W>(stage, a.levels + (size_t)h * a.plane + (size_t)tile * 64 * W, wave);
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    if ((h >> b) & 1) hb[b][i] |= x;
            }
        }
    }
    unsigned long long present = 0;
#pragma unroll
    for (int i = 0; i < kSuperTiles; ++i) present |= visw[i];
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) present |= shfl_xor64(present, m);
    present &= range_bits(a.q0, a.q1, wave);
    // lane qq keeps the list position where query 64*wave+qq continues in this super tile
    long long mybase = 0;
    if ((present >> v) & 1ull) mybase = super_start(a, st, Qp, wave * 64 + v);
    uint16_t *ent = s_ent[wave];
    uint8_t *hp = s_hop[wave];
    while (present) {
        const int qq = __ffsll((long long)present) - 1;
        present &= present - 1;
        int cnt = 0;
#pragma unroll
        for (int i = 0; i < kSuperTiles; ++i) {
            bool bit = (visw[i] >> qq) & 1ull;
            unsigned long long m = __ballot(bit);
            if (bit) {
                int pos = cnt + __popcll(m & ((1ull << v) - 1ull));
                int hv = 0;
#pragma unroll
                for (int b = 0; b < NB; ++b) hv |= (int)((hb[b][i] >> qq) & 1ull) << b;
                ent[pos] = (uint16_t)(i * 64 + v);
                hp[pos] = (uint8_t)hv;
            }
            cnt += __popcll(m);
        }
        __builtin_amdgcn_wave_barrier();
        const long long base = (long long)shfl64((unsigned long long)mybase, qq);
        const int e0 = (int)(st * (kSuperTiles * 64));
        for (int p = v; p < cnt; p += 64) {
            a.entity[base + p] = e0 + ent[p];
            if (a.hop) a.hop[base + p] = hp[p];
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// ---------------------------------------------------------------- predecessor edges
// Exclusive prefix-OR over the 64/W groups of a wavefront (word lw of each group).
template <int W>
__device__ __forceinline__ unsigned long long groups_before(unsigned long long x) {
    if constexpr (W >= 64) return 0ull;
    else {
        unsigned long long inc = x;
#pragma unroll
        for (int d = W; d < 64; d <<= 1) {
            unsigned long long y = shfl_up64(inc, d);
            if (lane() >= d) inc |= y;
        }
        unsigned long long ex = shfl_up64(inc, W);
        return lane() >= W ? ex : 0ull;
    }
}

template <int W>
__device__ __forceinline__ unsigned long long or_groups(unsigned long long acc) {
#pragma unroll
    for (int m = W; m < 64; m <<= 1) acc |= shfl_xor64(acc, m);
    return acc;
}

// Removes up to 64/W candidates from the wave-uniform mask; group g gets the
// g-th of them (lane position) or -1.
template <int W>
__device__ __forceinline__ int next_candidates(unsigned long long &rest) {
    constexpr int GPW = 64 / W;
    int g = lane() / W, mine = -1;
#pragma unroll
    for (int t = 0; t < GPW; ++t) {
        if (rest) {
            int p = __ffsll((long long)rest) - 1;
            rest &= rest - 1;
            if (t == g) mine = p;
        }
    }
    return mine;
}

// Ordered walk over the 64 in-edges [j0, j0+64) of an object row.  Every group
// holds the same `rem` (word lw of the still unresolved queries).  64/W
// candidate subjects are gathered at once; a group's line resolves the bits
// that no earlier candidate of the round has, so the result equals a strictly
// sequential walk in ascending edge id.  emit(hit, eid) runs on lanes whose word
// has newly resolved bits; returns the number of lines gathered.
template <int W, bool MASK, typename Emit>
__device__ __forceinline__ int pred_chunk(uint32_t j0, uint32_t hi, const FillArgs &a,
                                          const uint32_t *__restrict__ act_prev,
                                          const unsigned long long *__restrict__ prev,
                                          unsigned long long &rem, Emit emit) {
    const int lw = lane() & (W - 1);
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
        gathered += min(__popcll(cm), 64 / W);
        int p = next_candidates<W>(cm);
        int sc = __shfl(s, p < 0 ? 0 : p);
        unsigned long long ln = 0;
        if (p >= 0) {
            ln = prev[(size_t)sc * W + lw];
            if (MASK) ln &= a.allow[(size_t)a.in_rel[j0 + p] * W + lw];
        }
        unsigned long long hit = ln & rem & ~groups_before<W>(ln);
        rem &= ~or_groups<W>(ln);
        if (hit) emit(hit, a.in_eid[j0 + p]);
        if (!wave_any(rem != 0)) break;
    }
    return gathered;
}

// One block per tile of 64 entities.  Phase 1: per query, the mask of tile
// entities it reached (for ranks) and the list position of the tile's run;
// seeds get -1.  Phase 2: one wavefront per entity walks its object row.
template <int W, bool MASK>
__global__ void __launch_bounds__(64 * W) k_pred(FillArgs a) {
    constexpr int Qp = 64 * W;
    __shared__ unsigned long long stage[64][W + 1];
    __shared__ unsigned long long mT[Qp];
    __shared__ long long base[Qp];
    const long long tile_rel = xcd_contiguous(blockIdx.x, gridDim.x);
    if (tile_rel >= a.tile_count) return;
    const long long tile = a.tile_begin + tile_rel;
    const int t = threadIdx.x, wave = t >> 6, v = lane();
    {
        int q = t;
        long long b = 0;
        if (q >= a.q0 && q < a.q1)
            b = super_start(a, tile / kSuperTiles, Qp, q) + a.tile_base[(size_t)tile * Qp + q];
        base[q] = b;
    }
    unsigned long long visw = stage_word<W>(stage, a.visited + (size_t)tile * 64 * W, wave);
    unsigned long long seedw = stage_word<W>(stage, a.levels + (size_t)tile * 64 * W, wave);
    unsigned long long mine = 0;
    unsigned long long todo = range_bits(a.q0, a.q1, wave);
    if (!wave_any(visw != 0)) todo = 0;
    for (int qq = 0; qq < 64; ++qq) {
        if (!((todo >> qq) & 1ull)) continue;
        bool bit = (visw >> qq) & 1ull;
        unsigned long long m = __ballot(bit);
        if (v == qq) mine = m;
        if ((seedw >> qq) & 1ull) a.pred[base[wave * 64 + qq] + __popcll(m & ((1ull << v) - 1ull))] = -1;
    }
    mT[t] = mine;
    __syncthreads();

    const int nwaves = blockDim.x >> 6, lw = v & (W - 1);
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
        const unsigned long long below = (1ull << vi) - 1ull;
        for (int h = 1; h <= a.k; ++h) {
            unsigned long long rem = a.levels[(size_t)h * a.plane + (size_t)ev * W + lw] & range_bits(a.q0, a.q1, lw);
            if (!wave_any(rem != 0)) continue;
            if (hubrow) {  // the block-per-row kernel resolves these; give it the slots
                if (v < W)
                    for (unsigned long long m = rem; m; m &= m - 1) {
                        int q = v * 64 + (__ffsll((long long)m) - 1);
                        long long pos = base[q] + __popcll(mT[q] & below);
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
                        int q = lw * 64 + (__ffsll((long long)m) - 1);
                        a.pred[base[q] + __popcll(mT[q] & below)] = eid;
                    }
                });
                n_edges += min((uint32_t)64, hi - j0);
                if (!wave_any(rem != 0)) break;
            }
        }
    }
    if (a.stats_pred && v == 0) {
        if (n_rows) atomicAdd(&a.stats_pred[0], (unsigned long long)n_rows);
        if (n_edges) atomicAdd(&a.stats_pred[1], (unsigned long long)n_edges);
        if (n_lines) atomicAdd(&a.stats_pred[2], (unsigned long long)n_lines);
    }
}

// Hub object rows: one block per row.  The row is walked in steps of
// (waves x 64) edges; inside a step the waves work on disjoint edge ranges in
// parallel and merge with atomicMin, between steps the resolved bits are
// removed, so later steps never override earlier (smaller) edge ids.
template <int W, bool MASK>
__global__ void __launch_bounds__(1024) k_pred_hub(FillArgs a) {
    constexpr int Qp = 64 * W;
    __shared__ unsigned long long srem[16];
    const long long hidx = a.hub_begin + blockIdx.x;
    const int ev = a.hubs[hidx];
    const int t = threadIdx.x, wave = t >> 6, nw = blockDim.x >> 6, lw = lane() & (W - 1);
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
            unsigned long long rem = srem[lw];
            if (!wave_any(rem != 0)) break;  // same decision in every wave
            if (s0 == lo && wave == 0) ++n_rows;
            const unsigned long long before = rem;
            uint32_t j0 = s0 + 64u * wave;
            if (j0 < hi) {
                n_lines += pred_chunk<W, MASK>(j0, hi, a, act_prev, prev, rem, [&](unsigned long long hit, int eid) {
                    for (unsigned long long m = hit; m; m &= m - 1) {
                        int q = lw * 64 + (__ffsll((long long)m) - 1);
                        atomicMin(&a.pred[a.hub_slot[(size_t)hidx * Qp + q]], eid);
                    }
                });
                n_edges += min((uint32_t)64, hi - j0);
            }
            unsigned long long resolved = before & ~rem;
            __syncthreads();
            if (lane() < W && resolved) atomicAnd(&srem[lane()], ~resolved);
            __syncthreads();
        }
    }
    if (a.stats_hub && lane() == 0) {
        if (n_rows) atomicAdd(&a.stats_hub[0], (unsigned long long)n_rows);
        if (n_edges) atomicAdd(&a.stats_hub[1], (unsigned long long)n_edges);
        if (n_lines) atomicAdd(&a.stats_hub[2], (unsigned long long)n_lines);
    }
}

// ---------------------------------------------------------------- traversed
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
        for (int tt = 0; tt < kMegaSupers; ++tt) {
            long long tile = st * kMegaSupers + tt;
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
    const long long nmega = (nsuper + kMegaSupers - 1) / kMegaSupers;
    LKG_TRY(g->pool.alloc((void **)&r->tile_base, (size_t)ntiles * Qp * 2));
    LKG_TRY(g->pool.alloc((void **)&r->super_base, (size_t)nsuper * Qp * 4));
    LKG_TRY(g->pool.alloc((void **)&r->mega_base, (size_t)nmega * Qp * 4));
    LKG_TRY(g->pool.alloc((void **)&r->d_reached_off, (size_t)(Qp + 1) * 8));
    {
        ProfScope ps(g->prof, KK_COUNT, st);
        dim3 grid((unsigned)nsuper), block(Qp);
        switch (W) {
            case 1: k_count<1><<<grid, block, 0, st>>>(r->visited, ntiles, r->tile_base, r->super_base); break;
            case 4: k_count<4><<<grid, block, 0, st>>>(r->visited, ntiles, r->tile_base, r->super_base); break;
            default: k_count<16><<<grid, block, 0, st>>>(r->visited, ntiles, r->tile_base, r->super_base); break;
        }
        g->prof.acc[KK_COUNT].units[3] += g->prof.on ? r->Epad * W : 0;
    }
    {
        ProfScope ps(g->prof, KK_SCAN, st);
        k_scan_level<<<dim3((unsigned)nmega), dim3(std::min(Qp, 256)), 0, st>>>(nsuper, kMegaSupers, Qp,
                                                                              r->super_base, r->mega_base);
        k_scan_top<<<dim3(1), dim3(Qp), 0, st>>>(nmega, r->Q, Qp, r->mega_base, r->d_reached_off);
    }
    LKG_HIP(hipGetLastError());
    r->reached_off.assign((size_t)r->Q + 1, 0);
    LKG_HIP(hipMemcpyAsync(r->reached_off.data(), r->d_reached_off, (size_t)(r->Q + 1) * 8,
                           hipMemcpyDeviceToHost, st));
    LKG_HIP(hipStreamSynchronize(st));
    r->has_counts = true;
    return LOGOSKG_OK;
}

template <int W>
static void launch_lists_w(Profiler &prof, const FillArgs &a, hipStream_t st) {
    const long long nsuper = (a.ntiles + kSuperTiles - 1) / kSuperTiles;
    ProfScope ps(prof, KK_LISTS, st);
    int nb = 1;
    while ((1 << nb) <= a.k) ++nb;
    dim3 grid((unsigned)nsuper), block(64 * W);
    if (nb <= 2) k_lists<W, 2><<<grid, block, 0, st>>>(a);
    else if (nb <= 4) k_lists<W, 4><<<grid, block, 0, st>>>(a);
    else k_lists<W, 8><<<grid, block, 0, st>>>(a);
}

// predecessor kernels over the tiles [a.tile_begin, +a.tile_count) and `n_hubs_here` hub rows
// starting at a.hub_begin
template <int W>
static void launch_pred_w(Profiler &prof, const FillArgs &a, long long n_hubs_here, bool mask, hipStream_t st) {
    if (a.tile_count > 0) {
        ProfScope ps(prof, KK_PRED, st);
        dim3 grid((unsigned)((a.tile_count + 7) / 8 * 8)), block(64 * W);
        if (mask) k_pred<W, true><<<grid, block, 0, st>>>(a);
        else k_pred<W, false><<<grid, block, 0, st>>>(a);
    }
    if (n_hubs_here > 0) {
        ProfScope ps(prof, KK_PRED_HUB, st);
        if (mask) k_pred_hub<W, true><<<dim3((unsigned)n_hubs_here), dim3(1024), 0, st>>>(a);
        else k_pred_hub<W, false><<<dim3((unsigned)n_hubs_here), dim3(1024), 0, st>>>(a);
    }
}

void launch_lists(Profiler &prof, const FillArgs &a, int W, hipStream_t st) {
    switch (W) {
        case 1: launch_lists_w<1>(prof, a, st); break;
        case 4: launch_lists_w<4>(prof, a, st); break;
        default: launch_lists_w<16>(prof, a, st); break;
    }
}

void launch_pred(Profiler &prof, const FillArgs &a, int W, long long n_hubs_here, bool mask, hipStream_t st) {
    switch (W) {
        case 1: launch_pred_w<1>(prof, a, n_hubs_here, mask, st); break;
        case 4: launch_pred_w<4>(prof, a, n_hubs_here, mask, st); break;
        default: launch_pred_w<16>(prof, a, n_hubs_here, mask, st); break;
    }
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
    LKG_HIP(hipSetDevice(g->device));
    hipStream_t st = (hipStream_t)stream;
    const int W = r->W, Qp = 64 * W;
    if (pred && g->in_rows.n_hub > 0 && !r->hub_slot)
        LKG_TRY(g->pool.alloc((void **)&r->hub_slot, (size_t)g->in_rows.n_hub * Qp * 8));
    FillArgs a;
    a.E = g->E; a.Q = r->Q; a.k = r->k; a.q0 = q0; a.q1 = q1; a.hub_min = g->hub_min;
    a.ntiles = r->Epad / kTileEntities;
    a.tile_begin = 0; a.tile_count = a.ntiles; a.hub_begin = 0;
    a.plane = r->Epad * W; a.actw = r->Epad / 32;
    a.visited = r->visited; a.levels = r->levels; a.allow = r->allow;
    a.act = r->act; a.tile_base = r->tile_base; a.super_base = r->super_base; a.mega_base = r->mega_base;
    a.reached_off = r->d_reached_off;
    a.in_off = g->in_off; a.in_sub = g->in_sub; a.in_eid = g->in_eid; a.in_rel = g->in_rel;
    a.hubs = g->in_rows.hub; a.n_hubs = g->in_rows.n_hub;
    a.entity = entity; a.hop = hop; a.pred = pred; a.hub_slot = r->hub_slot;
    const bool counting = g->prof.counters;
    a.stats_pred = counting ? g->d_ctr + C_STATS + 4 * KK_PRED : nullptr;
    a.stats_hub = counting ? g->d_ctr + C_STATS + 4 * KK_PRED_HUB : nullptr;
    if (counting) LKG_HIP(hipMemsetAsync(g->d_ctr + C_STATS, 0, 4 * KK_NUM * sizeof(unsigned long long), st));
    launch_lists(g->prof, a, W, st);
    if (pred) {
        if (g->num_shards > 1) LKG_TRY(sharded_pred(g, &a, W, r->has_mask, st));
        else launch_pred(g->prof, a, W, a.n_hubs, r->has_mask, st);
    }
    LKG_HIP(hipGetLastError());
    if (g->prof.on) {
        g->prof.acc[KK_LISTS].units[3] += need;
        if (pred) g->prof.acc[KK_PRED].units[3] += need;
    }
    if (counting) {  // measurement mode only: wait for the counters
        LKG_HIP(hipMemcpyAsync(g->h_ctr, g->d_ctr, C_TOTAL * sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
        LKG_HIP(hipStreamSynchronize(st));
        for (int kind : {KK_PRED, KK_PRED_HUB})
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
    const long long nblocks = (ntiles + kMegaSupers - 1) / kMegaSupers;
    LKG_HIP(hipMemsetAsync(traversed, 0, (size_t)r->Q * r->k * 8, st));
    dim3 grid((unsigned)nblocks), block(64 * W);
    ProfScope ps(g->prof, KK_TRAVERSED, st);
    unsigned long long *tr = (unsigned long long *)traversed;
    const unsigned long long *lv = r->levels;
    switch (W) {
        case 1: k_traversed<1><<<grid, block, 0, st>>>(g->E, r->Q, r->k, r->Epad * W, ntiles, lv, g->out_off, tr); break;
        case 4: k_traversed<4><<<grid, block, 0, st>>>(g->E, r->Q, r->k, r->Epad * W, ntiles, lv, g->out_off, tr); break;
        default: k_traversed<16><<<grid, block, 0, st>>>(g->E, r->Q, r->k, r->Epad * W, ntiles, lv, g->out_off, tr); break;
    }
    LKG_HIP(hipGetLastError());
    return LOGOSKG_OK;
}
