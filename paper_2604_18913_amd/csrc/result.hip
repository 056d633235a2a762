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
//           (of the visited plane, or of one level plane for the per-level lists)
//   lists : one block per super tile compacts the (entity, hop) entries of each
//           query in LDS and writes them as whole 64-lane stores
//   pred  : the predecessor edge (smallest edge id whose subject sits one hop
//           closer and whose relation the query allows - the first active
//           triple of Eq. 5-7 in edge-id order) is found by walking the object
//           row of the entity with a mask of still unresolved queries, so every
//           (query, entity) pair is written once.  Object rows of up to 32
//           entries belong to the tile kernels that walk them in ascending
//           edge id (for 16-word planes and k <= 6 the pair k_pred_walk /
//           k_pred_emit, which writes the entity and hop lists as well;
//           k_pred otherwise); rows of 33 .. hub_min-1 entries belong to
//           k_pred_wave and longer ones to k_pred_row, whose lanes claim in
//           parallel and keep the minimum.  A level with a small frontier is
//           taken from the subject side for these longer rows (k_pred_push).
#include <algorithm>
#include <climits>
#include <cstdlib>
#include <type_traits>

#include "common.h"

namespace lkg {

// Tiles.  A tile is 64 entities.  Without a list (tile_ent == NULL) tile i holds the ids
// 64 i .. 64 i + 63; with the list of a result's active entities (those with a bit in any level,
// ascending, built by k_active_*) tile i holds entries 64 i .. 64 i + 63 of the list, so that the
// tiles carry no entity that no query reached (-1 pads the last tile).
__device__ __forceinline__ long long tile_entity(const int32_t *__restrict__ tile_ent, long long tile, int i,
                                                 int32_t E) {
    if (tile_ent) return tile_ent[tile * 64 + i];
    const long long e = tile * 64 + i;
    return e < E ? e : -1;
}

template <int W>
__device__ __forceinline__ unsigned long long stage_word(unsigned long long (*stage)[W + 1],
                                                         const unsigned long long *__restrict__ plane,
                                                         const int32_t *__restrict__ tile_ent, long long tile,
                                                         int32_t E, int wave) {
    // load of a tile's lines of one plane (W consecutive lanes per line), then lane v takes word
    // `wave` of the tile's entity v
    const int t = threadIdx.x;
    const long long e = tile_entity(tile_ent, tile, t / W, E);
    __syncthreads();
    stage[t / W][t % W] = e >= 0 ? plane[(size_t)e * W + t % W] : 0ull;
    __syncthreads();
    return stage[lane()][wave];
}

// ---------------------------------------------------------------- list of the active entities
// act holds one bitmap per level (one bit per entity with a non-zero line); their union marks the
// entities some query reached.  Chunks of 2,048 entities (64 bitmap words, one wavefront):
// k_active_count counts a chunk, k_active_scan turns the counts into exclusive offsets and the
// total, k_active_fill writes the ids (ascending) and every listed entity's position.
constexpr int kActChunkWords = 64;

__device__ __forceinline__ uint32_t active_word(const uint32_t *__restrict__ act, long long actw, int levels,
                                                long long word) {
    uint32_t u = 0;
    if (word < actw)
        for (int h = 0; h < levels; ++h) u |= act[(size_t)h * actw + word];
    return u;
}

__global__ void __launch_bounds__(256)
k_active_count(const uint32_t *__restrict__ act, long long actw, int levels, long long nchunks, uint32_t *chunk_cnt) {
    const long long chunk = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (chunk >= nchunks) return;
    const uint32_t u = active_word(act, actw, levels, chunk * kActChunkWords + lane());
    const long long c = wave_sum((long long)__popc(u));
    if (lane() == 0) chunk_cnt[chunk] = (uint32_t)c;
}

// one block: exclusive prefix over the chunk counts (in place), total to *n_active, and -1 in the
// 64 list entries behind the last id
__global__ void __launch_bounds__(1024)
k_active_scan(long long nchunks, uint32_t *chunk_cnt, unsigned long long *n_active, int32_t *tile_ent) {
    __shared__ unsigned long long part[2][1024];
    const int t = threadIdx.x;
    const long long per = (nchunks + 1023) / 1024, lo = (long long)t * per, hi = min(nchunks, lo + per);
    unsigned long long sum = 0;
    for (long long i = lo; i < hi; ++i) sum += chunk_cnt[i];
    int cur = 0;
    part[0][t] = sum;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {
        unsigned long long x = part[cur][t];
        if (t >= d) x += part[cur][t - d];
        part[cur ^ 1][t] = x;
        cur ^= 1;
        __syncthreads();
    }
    unsigned long long run = part[cur][t] - sum;
    for (long long i = lo; i < hi; ++i) {
        const uint32_t c = chunk_cnt[i];
        chunk_cnt[i] = (uint32_t)run;
        run += c;
    }
    const unsigned long long total = part[cur][1023];
    if (t == 0) *n_active = total;
    if (t < 64) tile_ent[total + t] = -1;
}

__global__ void __launch_bounds__(256)
k_active_fill(const uint32_t *__restrict__ act, long long actw, int levels, long long nchunks,
              const uint32_t *__restrict__ chunk_base, int32_t *tile_ent, int32_t *cpos) {
    const long long chunk = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (chunk >= nchunks) return;
    const long long word = chunk * kActChunkWords + lane();
    uint32_t u = active_word(act, actw, levels, word);
    int total;
    long long at = (long long)chunk_base[chunk] + wave_excl_scan(__popc(u), total);
    for (; u; u &= u - 1, ++at) {
        const int32_t e = (int32_t)(word * 32 + (__ffs((int)u) - 1));
        tile_ent[at] = e;
        cpos[e] = (int32_t)at;
    }
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
// With a list the number of tiles follows from *n_active (the grid covers the largest possible
// number of super tiles; those behind the list write zero sums).
template <int W>
__global__ void k_count(const unsigned long long *__restrict__ visited, long long ntiles, int32_t E,
                        const int32_t *__restrict__ tile_ent, const unsigned long long *__restrict__ n_active,
                        uint16_t *tile_base, uint32_t *super_sum) {
    constexpr int Qp = 64 * W;
    __shared__ unsigned long long stage[64][W + 1];
    const long long st = blockIdx.x;
    const int wave = threadIdx.x >> 6;
    if (tile_ent) ntiles = (long long)((*n_active + 63) / 64);
    int run = 0;
    for (int i = 0; i < kSuperTiles; ++i) {
        long long tile = st * kSuperTiles + i;
        if (tile >= ntiles) break;
        unsigned long long x = stage_word<W>(stage, visited, tile_ent, tile, E, wave);
        tile_base[(size_t)tile * Qp + threadIdx.x] = (uint16_t)run;
        int mine = 0;
        if (wave_any(x != 0)) mine = __popcll(transpose64(x));  // lane qq: entities of the tile query qq reached
        run += mine;
    }
    super_sum[(size_t)st * Qp + threadIdx.x] = (uint32_t)run;
}

// exclusive prefix of `sum` over groups of `group` consecutive rows; total per group to `up`.
// One thread per (group, query); the rows are read sixteen at a time before any is rewritten,
// so the loads of a batch are in flight together.
__global__ void k_scan_level(long long nrows, int group, int Qp, uint32_t *sum_to_base, uint32_t *up) {
    const long long g = blockIdx.x;
    const int q = blockIdx.y * blockDim.x + threadIdx.x;
    if (q >= Qp) return;
    uint32_t run = 0;
    for (int t0 = 0; t0 < group; t0 += 16) {
        uint32_t x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const long long row = g * group + t0 + i;
            x[i] = (t0 + i < group && row < nrows) ? sum_to_base[(size_t)row * Qp + q] : 0u;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const long long row = g * group + t0 + i;
            if (t0 + i < group && row < nrows) sum_to_base[(size_t)row * Qp + q] = run;
            run += x[i];
        }
    }
    up[(size_t)g * Qp + q] = run;
}

// one block of Qp threads: prefix over mega tiles for every query, then the prefix over queries
// (Hillis-Steele steps in LDS)
__global__ void k_scan_top(long long nmega, int Q, int Qp, uint32_t *mega_base, long long *reached_off) {
    __shared__ long long total[2][1024];
    const int q = threadIdx.x;
    long long run = 0;
    for (long long m = 0; m < nmega; ++m) {
        uint32_t x = mega_base[(size_t)m * Qp + q];
        mega_base[(size_t)m * Qp + q] = (uint32_t)run;
        run += x;
    }
    const long long mine = q < Q ? run : 0;
    int cur = 0;
    total[0][q] = mine;
    __syncthreads();
    for (int d = 1; d < Qp; d <<= 1) {  // inclusive prefix
        long long v = total[cur][q];
        if (q >= d) v += total[cur][q - d];
        total[cur ^ 1][q] = v;
        cur ^= 1;
        __syncthreads();
    }
    reached_off[q] = total[cur][q] - mine;  // exclusive
    if (q == Qp - 1) reached_off[Qp] = total[cur][q];
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
// NB = words of the bit-sliced hop number (0: entity ids only); TILES = tiles per block: a
// whole super tile, or half of one where the registers of a whole one would not leave room for
// two blocks per CU.
template <int W, int NB, int TILES>
__global__ void __launch_bounds__(64 * W) k_lists(FillArgs a) {
    constexpr int Qp = 64 * W, NBX = NB > 0 ? NB : 1;
    __shared__ unsigned long long stage[64][W + 1];
    __shared__ uint16_t s_ent[W][TILES * 64];
    __shared__ uint8_t s_hop[NB > 0 ? W : 1][TILES * 64];
    __shared__ int32_t blk_ent[TILES * 64];  // entity ids of the block's tiles
    const long long first_tile = (long long)blockIdx.x * TILES;
    for (int i = threadIdx.x; i < TILES * 64; i += 64 * W) {
        const long long tile = first_tile + i / 64;
        blk_ent[i] = tile < a.ntiles ? (int32_t)tile_entity(a.tile_ent, tile, i % 64, a.E) : -1;
    }
    const long long st = first_tile / kSuperTiles;
    const int wave = threadIdx.x >> 6, v = lane();
    unsigned long long visw[TILES];
    unsigned long long hb[NBX][TILES];
#pragma unroll
    for (int i = 0; i < TILES; ++i) {
        long long tile = first_tile + i;
        visw[i] = 0;
#pragma unroll
        for (int b = 0; b < NBX; ++b) hb[b][i] = 0;
        if (tile < a.ntiles) {  // block-uniform
            visw[i] = stage_word<W>(stage, a.visited, a.tile_ent, tile, a.E, wave);
            if constexpr (NB > 0)
                for (int h = 1; h <= a.k; ++h) {  // hop number of each bit, bit-sliced over NB words
                    unsigned long long x =
                        stage_word<W>(stage, a.levels + (size_t)h * a.plane, a.tile_ent, tile, a.E, wave);
#pragma unroll
                    for (int b = 0; b < NB; ++b)
                        if ((h >> b) & 1) hb[b][i] |= x;
                }
        }
    }
    unsigned long long present = 0;
#pragma unroll
    for (int i = 0; i < TILES; ++i) present |= visw[i];
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) present |= shfl_xor64(present, m);
    present &= range_bits(a.q0, a.q1, wave);
    // lane qq keeps the list position where query 64*wave+qq continues in this block's tiles
    long long mybase = 0;
    if ((present >> v) & 1ull) {
        mybase = super_start(a, st, Qp, wave * 64 + v);
        if (TILES < kSuperTiles) mybase += a.tile_base[(size_t)first_tile * Qp + wave * 64 + v];
    }
    uint16_t *ent = s_ent[wave];
    uint8_t *hp = s_hop[NB > 0 ? wave : 0];
    while (present) {
        const int qq = __ffsll((long long)present) - 1;
        present &= present - 1;
        int cnt = 0;
#pragma unroll
        for (int i = 0; i < TILES; ++i) {
            bool bit = (visw[i] >> qq) & 1ull;
            unsigned long long m = __ballot(bit);
            if (bit) {
                int pos = cnt + __popcll(m & ((1ull << v) - 1ull));
                ent[pos] = (uint16_t)(i * 64 + v);
                if constexpr (NB > 0) {
                    int hv = 0;
#pragma unroll
                    for (int b = 0; b < NB; ++b) hv |= (int)((hb[b][i] >> qq) & 1ull) << b;
                    hp[pos] = (uint8_t)hv;
                }
            }
            cnt += __popcll(m);
        }
        __builtin_amdgcn_wave_barrier();
        const long long base = (long long)shfl64((unsigned long long)mybase, qq);
        for (int p = v; p < cnt; p += 64) {
            a.entity[base + p] = blk_ent[ent[p]];
            if constexpr (NB > 0) a.hop[base + p] = hp[p];
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// ---------------------------------------------------------------- predecessor edges
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

// The 64 in-edges [j0, j0+64) of an object row for a caller that merges claims with a minimum over
// edge ids (the row kernels): every W-lane group keeps a mask `rem` of its own (word lw of the
// queries it has not resolved), takes every (64/W)-th candidate subject, gathers its line and
// claims whatever its mask still holds, with no exchange between the groups.  (An ordered walk -
// a candidate claims only what no earlier candidate of the round has, found with an exclusive
// prefix-OR across the groups - costs ten dependent LDS permutes per round, which is what these
// kernels then wait on.)  A query may be claimed by several groups; the smallest edge id wins.
// emit(hit, eid) runs on lanes whose word has newly claimed bits; returns the lines gathered.
template <int W, bool MASK, typename Emit>
__device__ __forceinline__ int pred_resolve_unordered(uint32_t j0, int s, bool cand, const FillArgs &a,
                                                      const unsigned long long *__restrict__ prev,
                                                      unsigned long long &rem, Emit emit) {
    const int lw = lane() & (W - 1);
    unsigned long long cm = __ballot(cand);
    int gathered = 0;
    constexpr int NR = 4;
    while (cm) {
        gathered += min(__popcll(cm), NR * (64 / W));
        int p[NR];
        unsigned long long l[NR];
#pragma unroll
        for (int x = 0; x < NR; ++x) p[x] = next_candidates<W>(cm);
#pragma unroll
        for (int x = 0; x < NR; ++x) {
            const int sx = __shfl(s, p[x] < 0 ? 0 : p[x]);
            l[x] = 0;
            if (p[x] >= 0) l[x] = prev[(size_t)sx * W + lw];
        }
        if (MASK) {
#pragma unroll
            for (int x = 0; x < NR; ++x)
                if (p[x] >= 0) l[x] &= a.allow[(size_t)a.in_rel[j0 + p[x]] * W + lw];
        }
#pragma unroll
        for (int x = 0; x < NR; ++x) {
            const unsigned long long hit = l[x] & rem;
            rem &= ~l[x];
            if (hit) emit(hit, a.in_eid[j0 + p[x]]);
        }
        if (!wave_any(rem != 0)) break;
    }
    return gathered;
}

// The same 64 in-edges when the fetched queries sit in one word `wq` of the 16-word lines: lane =
// entry, every lane gathers that one word of its own candidate, and a 64 x 64 bit transpose turns
// "entry -> queries it resolves" into "query -> entries that resolve it" (lane = query), whose lowest
// set bit is the entry with the smallest edge id (edge ids ascend inside a row).  One round of 64
// eight-byte gathers where the line-wide form needs sixteen rounds of four lines.  `rem` is
// wavefront-uniform; emit(q, eid) runs on lane q for the queries resolved here.
template <bool MASK, typename Emit>
__device__ __forceinline__ int pred_resolve_word(uint32_t j0, int s, bool cand, int wq, const FillArgs &a,
                                                 const unsigned long long *__restrict__ prev,
                                                 unsigned long long &rem, Emit emit) {
    unsigned long long l = 0;
    if (cand) {
        l = prev[(size_t)s * 16 + wq];
        if (MASK) l &= a.allow[(size_t)a.in_rel[j0 + lane()] * 16 + wq];
        l &= rem;
    }
    const int gathered = __popcll(__ballot(cand));
    if (wave_any(l != 0)) {
        const unsigned long long from = transpose64(l);  // lane q: the entries whose line holds query q
        if (from) emit(lane(), a.in_eid[j0 + (uint32_t)(__ffsll((long long)from) - 1)]);
        rem &= ~__ballot(from != 0);
    }
    return gathered;
}

// List positions of entity `ev` for every query: slot[q] = start of the tile's run in query q's
// list + rank of the entity inside the tile.  Called by a whole wavefront for the words
// w = w_first, w_first + w_step, ..
template <int W>
__device__ __forceinline__ void row_slots(const FillArgs &a, int ev, int w_first, int w_step, long long *slot) {
    constexpr int Qp = 64 * W;
    long long at = ev;  // place of the entity in the tiles
    if (a.cpos) {       // an entity no query reached is not listed: it needs no positions
        at = a.cpos[ev];
        if (at < 0 || at >= a.n_listed || a.tile_ent[at] != ev) return;
    }
    const long long tile = at >> 6;
    const int vi = (int)(at & 63), v = lane();
    const unsigned long long below = (1ull << vi) - 1ull;
    const long long ent_v = tile_entity(a.tile_ent, tile, v, a.E);
    for (int w = w_first; w < W; w += w_step) {  // lane v = entity v of the tile
        unsigned long long x = ent_v >= 0 ? a.visited[(size_t)ent_v * W + w] & range_bits(a.q0, a.q1, w) : 0ull;
        int rank = 0;
        if (shfl64(x, vi) != 0ull)  // only queries that reached this entity matter
            rank = __popcll(transpose64(x) & below);
        int q = w * 64 + v;
        long long b = 0;
        if (q >= a.q0 && q < a.q1)
            b = super_start(a, tile / kSuperTiles, Qp, q) + a.tile_base[(size_t)tile * Qp + q] + rank;
        slot[q] = b;
    }
}

// AND over the 64/W groups of a wavefront (word lw of each group).
template <int W>
__device__ __forceinline__ unsigned long long and_groups(unsigned long long x) {
#pragma unroll
    for (int m = W; m < 64; m <<= 1) x &= shfl_xor64(x, m);
    return x;
}

// Object rows of 33 .. hub_min-1 entries: one wavefront per row, four rows per block.  The W-lane
// groups of the wavefront claim independently (pred_resolve_unordered) and the smallest edge id per
// query is kept in a table of the wavefront in LDS; the groups' masks are merged once per 64
// entries, and after a level the table is written out (one contiguous store per 64 queries in the
// row-buffer mode) and reset.
// ONE (16-word lines, the fetched queries inside one word): every lane works on that word and
// takes an entry of its own (pred_resolve_word).
template <int W, bool MASK, bool STATS, bool BUF, bool ONE = false>
__global__ void __launch_bounds__(256) k_pred_wave(FillArgs a, long long first_row, long long n_rows_total) {
    static_assert(!ONE || (W == 16 && !STATS), "the one-word form is for 16-word lines");
    constexpr int Qp = 64 * W;
    __shared__ long long slots[BUF ? 1 : 4][BUF ? 1 : Qp];
    __shared__ int smin_all[4][Qp];
    const int wave = threadIdx.x >> 6, v = lane(), lw = ONE ? (a.q0 >> 6) : (v & (W - 1));
    const long long idx = (long long)blockIdx.x * 4 + wave;
    long long n_rows = 0, n_edges = 0, n_lines = 0;
    if (idx < n_rows_total) {  // wave-uniform
        const int ev = a.rows[first_row + idx];
        long long *slot = slots[BUF ? 0 : wave];
        int *smin = smin_all[wave];
        int32_t *out = BUF ? a.row_pred + (size_t)(first_row + idx) * Qp : a.pred;
        if (!BUF) row_slots<W>(a, ev, 0, 1, slot);
        for (int q = v; q < Qp; q += 64) smin[q] = INT_MAX;
        __builtin_amdgcn_wave_barrier();
        const uint32_t lo = a.in_off[ev], hi = a.in_off[ev + 1];
        for (int h = 1; h <= a.k; ++h) {
            const unsigned long long level = a.levels[(size_t)h * a.plane + (size_t)ev * W + lw] & range_bits(a.q0, a.q1, lw);
            unsigned long long rem = level;
            if (!wave_any(rem != 0) || ((a.push_levels >> h) & 1u)) continue;
            const uint32_t *act_prev = a.act + (size_t)(h - 1) * a.actw;
            const unsigned long long *prev = a.levels + (size_t)(h - 1) * a.plane;
            const bool dense = !STATS && ((a.dense_levels >> h) & 1u);  // the line of an entity outside the level is zero
            ++n_rows;
            for (uint32_t j0 = lo; j0 < hi; j0 += 64) {
                const uint32_t j = j0 + v;
                int s = 0;
                bool cand = false;
                if (j < hi) {
                    s = a.in_sub[j];
                    cand = dense || ((act_prev[s >> 5] >> (s & 31)) & 1u);
                }
                if constexpr (ONE) {
                    n_lines += pred_resolve_word<MASK>(j0, s, cand, lw, a, prev, rem,
                                                       [&](int q, int eid) { smin[lw * 64 + q] = eid; });
                } else {
                    n_lines += pred_resolve_unordered<W, MASK>(j0, s, cand, a, prev, rem, [&](unsigned long long hit, int eid) {
                        for (unsigned long long m = hit; m; m &= m - 1)
                            atomicMin(&smin[lw * 64 + (__ffsll((long long)m) - 1)], eid);
                    });
                    rem = and_groups<W>(rem);  // what any group has resolved is resolved
                }
                n_edges += min((uint32_t)64, hi - j0);
                if (!wave_any(rem != 0)) break;
            }
            __builtin_amdgcn_wave_barrier();
            for (int i = ONE ? lw : 0; i < (ONE ? lw + 1 : W); ++i) {  // queries 64 i .. 64 i + 63: word i of the level, held by lane i
                const unsigned long long word = ONE ? level : shfl64(level, i);
                const int q = 64 * i + v;
                if ((word >> v) & 1ull) {
                    out[BUF ? (long long)q : slot[q]] = smin[q];
                    smin[q] = INT_MAX;
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
    if (STATS && v == 0) {
        if (n_rows) atomicAdd(&a.stats_mid[0], (unsigned long long)n_rows);
        if (n_edges) atomicAdd(&a.stats_mid[1], (unsigned long long)n_edges);
        if (n_lines) atomicAdd(&a.stats_mid[2], (unsigned long long)n_lines);
    }
}

// One block per tile of 64 entities.  Phase 1: per query of the fetched range, the
// mask of tile entities it reached (for ranks) and the list position of the
// tile's run; seeds get -1.  Phase 2: every entity whose object row has at most
// 32 entries is walked by one W-lane group, two candidate lines in flight.
// Longer rows are left to k_pred_row.
template <int W, bool MASK, bool STATS>
__global__ void __launch_bounds__(64 * W) k_pred(FillArgs a) {
    constexpr int Qp = 64 * W;
    __shared__ unsigned long long stage[64][W + 1];
    __shared__ unsigned long long mT[Qp];
    __shared__ long long base[Qp];
    const long long tile_rel = xcd_contiguous(blockIdx.x, gridDim.x);
    if (tile_rel >= a.tile_count) return;
    const long long tile = a.tile_begin + tile_rel;
    const int t = threadIdx.x, wave = t >> 6, v = lane(), lw = t & (W - 1);
    {
        int q = t;
        long long b = 0;
        if (q >= a.q0 && q < a.q1)
            b = super_start(a, tile / kSuperTiles, Qp, q) + a.tile_base[(size_t)tile * Qp + q];
        base[q] = b;
    }
    const unsigned long long range_w = range_bits(a.q0, a.q1, wave);
    unsigned long long visw = stage_word<W>(stage, a.visited, a.tile_ent, tile, a.E, wave) & range_w;
    unsigned long long seedw = stage_word<W>(stage, a.levels, a.tile_ent, tile, a.E, wave) & range_w;
    unsigned long long mine = 0;
    if (wave_any(visw != 0)) mine = transpose64(visw);  // lane qq: mask of tile entities query qq reached
    mT[t] = mine;
    __syncthreads();
    auto slot = [&](int q, unsigned long long below) -> long long {
        return base[q] + __popcll(mT[q] & below);
    };
    {   // seeds have no predecessor
        const unsigned long long below_v = (1ull << v) - 1ull;
        for (unsigned long long m = seedw; m; m &= m - 1)
            a.pred[slot(wave * 64 + (__ffsll((long long)m) - 1), below_v)] = -1;
    }
    const int vi = t / W, g0 = v & ~(W - 1);
    const long long ev = tile_entity(a.tile_ent, tile, vi, a.E);
    uint32_t lo = 0, hi = 0;
    if (ev >= 0) {
        lo = a.in_off[ev];
        hi = a.in_off[ev + 1];
    }
    const bool longrow = hi - lo > (uint32_t)kTailMaxDegree;
    const unsigned long long below = (1ull << vi) - 1ull;
    long long n_rows = 0, n_edges = 0, n_lines = 0;
    if (hi > lo && !longrow)
        for (int h = 1; h <= a.k; ++h) {
            unsigned long long rem =
                a.levels[(size_t)h * a.plane + (size_t)ev * W + lw] & range_bits(a.q0, a.q1, lw);
            if (!group_any<W>(rem != 0)) continue;
            const uint32_t *act_prev = a.act + (size_t)(h - 1) * a.actw;
            const unsigned long long *prev = a.levels + (size_t)(h - 1) * a.plane;
            if (lw == 0) ++n_rows;
            for (uint32_t j0 = lo; j0 < hi; j0 += W) {
                uint32_t j = j0 + lw;
                int s = 0;
                bool cand = false;
                if (j < hi) {
                    s = a.in_sub[j];
                    cand = (act_prev[s >> 5] >> (s & 31)) & 1u;
                }
                unsigned gm = 0;
                if constexpr (W == 1) gm = cand ? 1u : 0u;
                else gm = (unsigned)((__ballot(cand) >> g0) & ((1ull << W) - 1ull));
                if (lw == 0) {
                    n_edges += min((uint32_t)W, hi - j0);
                    n_lines += __popc(gm);
                }
                while (gm) {  // two candidate lines in flight, resolved in edge order
                    int c0 = __ffs((int)gm) - 1;
                    gm &= gm - 1;
                    int c1 = -1;
                    if (gm) {
                        c1 = __ffs((int)gm) - 1;
                        gm &= gm - 1;
                    }
                    int s0 = __shfl(s, g0 + c0), s1 = __shfl(s, g0 + (c1 < 0 ? c0 : c1));
                    unsigned long long l0 = prev[(size_t)s0 * W + lw], l1 = 0;
                    if (c1 >= 0) l1 = prev[(size_t)s1 * W + lw];
                    if (MASK) {
                        l0 &= a.allow[(size_t)a.in_rel[j0 + c0] * W + lw];
                        if (c1 >= 0) l1 &= a.allow[(size_t)a.in_rel[j0 + c1] * W + lw];
                    }
                    unsigned long long hit0 = l0 & rem, hit1 = l1 & rem & ~l0;
                    rem &= ~(l0 | l1);
                    if (hit0) {
                        int eid = a.in_eid[j0 + c0];
                        for (unsigned long long m = hit0; m; m &= m - 1)
                            a.pred[slot(lw * 64 + (__ffsll((long long)m) - 1), below)] = eid;
                    }
                    if (hit1) {
                        int eid = a.in_eid[j0 + c1];
                        for (unsigned long long m = hit1; m; m &= m - 1)
                            a.pred[slot(lw * 64 + (__ffsll((long long)m) - 1), below)] = eid;
                    }
                    if (!group_any<W>(rem != 0)) break;
                }
                if (!group_any<W>(rem != 0)) break;
            }
        }
    if (STATS) {
        n_rows = wave_sum(n_rows);
        n_edges = wave_sum(n_edges);
        n_lines = wave_sum(n_lines);
        if (v == 0) {
            if (n_rows) atomicAdd(&a.stats_pred[0], (unsigned long long)n_rows);
            if (n_edges) atomicAdd(&a.stats_pred[1], (unsigned long long)n_edges);
            if (n_lines) atomicAdd(&a.stats_pred[2], (unsigned long long)n_lines);
        }
    }
}

// Predecessor pass for 16-word planes, bit-sliced, in two kernels.
//
// k_pred_walk: a 16-lane group per entity, lane lw owns word lw of the entity's lines.  The group
// walks the entity's object row (<= 32 entries) in edge-id order with a mask of unresolved
// queries per hop level; a candidate's line resolves the queries in (line & mask), all at once.
// What a (query, entity) pair needs later - its hop number and the position of its predecessor
// in the row - is kept bit-sliced: NB words H[b] hold bit b of (hop + 1) of each of the lane's 64
// queries (so H[0] | H[1] | .. is the visited word) and five words J[b] hold bit b of the row
// position.  A resolving line costs a fixed fifteen instructions for up to 64 pairs, whatever
// the number of set bits.  At the end the planes of a lane are turned into one code byte per
// query, (row position << 3) | (hop + 1), with eight 8 x 8 bit transposes, and the 64 bytes of
// every (entity, word) go to a buffer laid out [tile][word][entity][query], which a chunk of
// tiles fills and the second kernel empties while it is still in the caches.
//
// k_pred_emit: a block = one tile, its four wavefronts share the words of the fetched range; lane =
// entity, with the lane's 64 code bytes of the current word in registers.  A wavefront walks the
// queries of the word that reached the tile in a scalar loop; per query the lanes pick their code
// byte, a ballot ranks the reached ones inside the tile's piece of the query's run, and the lanes
// store (entity, hop, predecessor edge) at consecutive list positions: every lane issues the same
// few instructions and a store instruction covers one contiguous piece of a list.  The loop holds
// no load from memory (the edge ids of the tile's short rows are staged in LDS once per block), so
// nothing in it waits for its own stores.  Rows of more than 32 entries belong to the row
// kernels: such an entity's predecessors come from row_pred, which those kernels fill before
// this one starts (or, without that buffer, the row kernels write them to the lists themselves).
constexpr int kSlicedMaxK = 6;     // hop + 1 <= 7 fits three bits

__device__ __forceinline__ unsigned long long wave_or64(unsigned long long x) {
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) x |= shfl_xor64(x, m);
    return x;
}

// G = lanes per entity: 16 (lane = word of the line), 4 for a fetch whose queries sit in four
// aligned words or fewer (lane = word wb + lane % 4), which then walks four times as many entities
// per wavefront, or 1 for a fetch inside one word (lane = entity, word wb).
template <int NB, bool MASK, bool STATS, int G>
__global__ void __launch_bounds__(256)
k_pred_walk(FillArgs a, unsigned long long *__restrict__ codes, unsigned long long *__restrict__ visbuf,
            long long tile0, long long ntile, int w0, int nw, int wb) {
    constexpr int W = 16;
    constexpr int EPB = 256 / G;         // entities per block (a divisor of 64: one tile per block)
    constexpr unsigned GMASK = (1u << G) - 1u;
    constexpr int HMAX = (1 << NB) - 2;  // largest hop number the NB bits of (hop + 1) can hold
    const long long grp = xcd_contiguous(blockIdx.x, gridDim.x) * EPB + (threadIdx.x / G);  // entity slot of the chunk
    const long long tile_rel = grp >> 6;
    if (tile_rel >= ntile) return;  // wavefront-uniform: a wavefront's entities belong to one tile
    const int vi = (int)(grp & 63), lw = wb + (threadIdx.x & (G - 1)), v = lane(), g0 = v & ~(G - 1);
    const int gl = threadIdx.x & (G - 1);  // the lane's place in its group
    const long long ev = tile_entity(a.tile_ent, tile0 + tile_rel, vi, a.E);
    const unsigned long long range_w = range_bits(a.q0, a.q1, lw);
    unsigned long long visw = 0, lv0 = 0;
    uint32_t lo = 0, hi = 0;
    if (ev >= 0) {
        visw = a.visited[(size_t)ev * W + lw] & range_w;
        lv0 = a.levels[(size_t)ev * W + lw] & range_w;
        lo = a.in_off[ev];
        hi = a.in_off[ev + 1];
    }
    const uint32_t deg = hi - lo;
    const bool shortrow = deg > 0 && deg <= (uint32_t)kTailMaxDegree;
    unsigned long long H[NB], J[5];
    H[0] = lv0;  // hop 0: hop + 1 = 1
#pragma unroll
    for (int b = 1; b < NB; ++b) H[b] = 0;
#pragma unroll
    for (int b = 0; b < 5; ++b) J[b] = 0;
    long long n_rows = 0, n_edges = 0, n_lines = 0;
    if (group_any<G>((visw & ~lv0) != 0)) {  // some query of the range reached the entity by an edge
        // the level words of the first hops are requested together
        constexpr int PRE = HMAX < 3 ? HMAX : 3;
        unsigned long long pre[PRE];
#pragma unroll
        for (int h = 1; h <= PRE; ++h)
            pre[h - 1] = h <= a.k ? a.levels[(size_t)h * a.plane + (size_t)ev * W + lw] & range_w : 0ull;
#pragma unroll
        for (int h = 1; h <= HMAX; ++h) {
            if (h > a.k) break;
            unsigned long long rem;
            if (h <= PRE) rem = pre[h - 1];
            else rem = a.levels[(size_t)h * a.plane + (size_t)ev * W + lw] & range_w;
#pragma unroll
            for (int b = 0; b < NB; ++b)
                if (((h + 1) >> b) & 1) H[b] |= rem;
            if (!shortrow || !group_any<G>(rem != 0)) continue;
            const uint32_t *act_prev = a.act + (size_t)(h - 1) * a.actw;
            const unsigned long long *prev = a.levels + (size_t)(h - 1) * a.plane;
            const bool dense = !STATS && ((a.dense_levels >> h) & 1u);  // the line of an entity outside the level is zero
            if (STATS && gl == 0) ++n_rows;
            for (uint32_t j0 = lo; j0 < hi; j0 += G) {
                const uint32_t j = j0 + gl;
                int s = 0;
                bool cand = false;
                if (j < hi) {
                    s = a.in_sub[j];
                    cand = dense || ((act_prev[s >> 5] >> (s & 31)) & 1u);
                }
                unsigned gm = (unsigned)((__ballot(cand) >> g0) & GMASK);
                if (STATS && gl == 0) {
                    n_edges += min((uint32_t)G, hi - j0);
                    n_lines += __popc(gm);
                }
                while (gm) {  // two candidate lines in flight, resolved in edge order
                    const int d0 = __ffs((int)gm) - 1;
                    gm &= gm - 1;
                    int d1 = -1;
                    if (gm) {
                        d1 = __ffs((int)gm) - 1;
                        gm &= gm - 1;
                    }
                    const int s0 = __shfl(s, g0 + d0), s1 = __shfl(s, g0 + (d1 < 0 ? d0 : d1));
                    unsigned long long l0 = prev[(size_t)s0 * W + lw], l1 = 0;
                    if (d1 >= 0) l1 = prev[(size_t)s1 * W + lw];
                    if (MASK) {
                        l0 &= a.allow[(size_t)a.in_rel[j0 + d0] * W + lw];
                        if (d1 >= 0) l1 &= a.allow[(size_t)a.in_rel[j0 + d1] * W + lw];
                    }
                    const unsigned long long hit0 = l0 & rem, hit1 = l1 & rem & ~l0;
                    rem &= ~(l0 | l1);
                    const int p0 = (int)(j0 - lo) + d0, p1 = (int)(j0 - lo) + (d1 < 0 ? 0 : d1);
#pragma unroll
                    for (int b = 0; b < 5; ++b) {  // all-ones or zero from bit b of the position
                        const unsigned long long m0 = (unsigned long long)(long long)(-((p0 >> b) & 1));
                        const unsigned long long m1 = (unsigned long long)(long long)(-((p1 >> b) & 1));
                        J[b] |= (hit0 & m0) | (hit1 & m1);
                    }
                    if (!group_any<G>(rem != 0)) break;
                }
                if (!group_any<G>(rem != 0)) break;
            }
        }
    }
    if (lw >= w0 && lw < w0 + nw) {
        // From bit planes to one byte per query: plane b = bit b of the code, NB bits of (hop + 1)
        // below five bits of the row position.  Byte g of every plane forms an 8 x 8 bit matrix
        // (row = plane, column = query 8 g + j); its transpose holds the codes of those 8 queries.
        uint4 *out = reinterpret_cast<uint4 *>(codes) + (((size_t)tile_rel * nw + (lw - w0)) * 64 + vi) * 4;
        unsigned long long reached = 0;  // H[0] | H[1] | ..: the queries of the word that reached the entity
#pragma unroll
        for (int b = 0; b < NB; ++b) reached |= H[b];
        visbuf[((size_t)tile_rel * nw + (lw - w0)) * 64 + vi] = reached;
        unsigned long long P[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) P[b] = 0;
#pragma unroll
        for (int b = 0; b < NB; ++b) P[b] = H[b];
#pragma unroll
        for (int b = 0; b < 5; ++b) P[3 + b] = J[b];  // the position always starts at bit 3
        uint32_t d[16];
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            // byte b of x = byte g of plane b, picked with byte permutes (two planes per permute, then
            // the two pairs): six instructions instead of a shift, a mask and an or per plane and half
            uint32_t src[8];
#pragma unroll
            for (int b = 0; b < 8; ++b) src[b] = g < 4 ? (uint32_t)P[b] : (uint32_t)(P[b] >> 32);
            const uint32_t pick = 0x0c0c0000u | (uint32_t)((4 + (g & 3)) << 8) | (uint32_t)(g & 3);  // [b.byte, a.byte, 0, 0]
            const uint32_t t01 = __builtin_amdgcn_perm(src[1], src[0], pick), t23 = __builtin_amdgcn_perm(src[3], src[2], pick);
            const uint32_t t45 = __builtin_amdgcn_perm(src[5], src[4], pick), t67 = __builtin_amdgcn_perm(src[7], src[6], pick);
            const uint32_t xlo = __builtin_amdgcn_perm(t23, t01, 0x05040100u), xhi = __builtin_amdgcn_perm(t67, t45, 0x05040100u);
            unsigned long long x = ((unsigned long long)xhi << 32) | xlo;
            unsigned long long t;
            t = (x ^ (x >> 7)) & 0x00AA00AA00AA00AAull;
            x = x ^ t ^ (t << 7);
            t = (x ^ (x >> 14)) & 0x0000CCCC0000CCCCull;
            x = x ^ t ^ (t << 14);
            t = (x ^ (x >> 28)) & 0x00000000F0F0F0F0ull;
            x = x ^ t ^ (t << 28);
            d[2 * g] = (uint32_t)x;
            d[2 * g + 1] = (uint32_t)(x >> 32);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = make_uint4(d[4 * i], d[4 * i + 1], d[4 * i + 2], d[4 * i + 3]);
    }
    if (STATS) {
        n_rows = wave_sum(n_rows);
        n_edges = wave_sum(n_edges);
        n_lines = wave_sum(n_lines);
        if (v == 0) {
            if (n_rows) atomicAdd(&a.stats_pred[0], (unsigned long long)n_rows);
            if (n_edges) atomicAdd(&a.stats_pred[1], (unsigned long long)n_edges);
            if (n_lines) atomicAdd(&a.stats_pred[2], (unsigned long long)n_lines);
        }
    }
}

// A block = 16 consecutive tiles (one wavefront each) x every wsplit-th word of the fetched range.
// 8 wavefronts per SIMD = at most 64 vector registers.
constexpr int kEmitTiles = 16;
constexpr int kEmitEids = 9216;   // LDS: edge ids of the short rows of the block's 1,024 entities
constexpr int kEmitLines = 160;   // LDS: row_pred values (64 queries each) of the block's entities with longer rows
// (36 KB + 40 KB: two blocks per CU)

// STAGED: the edge ids of the block's short rows fit eid_tab; LINES: the block's row_pred entities
// fit rp_tab.  Otherwise the loop reads the edge ids from memory / a pass of its own moves the
// row_pred values with lanes = queries.
template <bool STAGED, bool LINES>
__device__ __forceinline__ void emit_word(const FillArgs &a, const uint32_t (&c)[16], unsigned long long live,
                                          uint32_t pos_lo, uint32_t pos_hi, int ent_id, bool longrow, bool by_query,
                                          const int *my_eids, const int32_t *my_row, const int *my_line) {
    const uint32_t live_lo = __builtin_amdgcn_readfirstlane((uint32_t)live);
    const uint32_t live_hi = __builtin_amdgcn_readfirstlane((uint32_t)(live >> 32));
    // unrolled over the sixteen code registers (four queries each): a query's byte is picked with
    // one bit-field extract
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        uint32_t rest = ((r < 8 ? live_lo : live_hi) >> (4 * (r & 7))) & 15u;
        while (rest) {  // scalar loop over the queries 4 r .. 4 r + 3 that reached the block's tiles
            const int j = __builtin_ctz(rest);
            rest &= rest - 1;
            const int qq = 4 * r + j;
            const uint32_t code = __builtin_amdgcn_ubfe(c[r], (unsigned)(8 * j), 8u);
            const uint32_t hc = code & 7u, jp = code >> 3;
            const bool bit = hc != 0u;
            const unsigned long long m = __ballot(bit);
            if (bit) {
                const unsigned rank =
                    __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                const unsigned long long base =
                    ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)pos_hi, qq) << 32) |
                    (uint32_t)__builtin_amdgcn_readlane((int)pos_lo, qq);
                int32_t *const pe = a.entity + base;
                pe[rank] = ent_id;
                if (a.hop) {
                    uint8_t *const ph8 = a.hop + base;
                    ph8[rank] = (uint8_t)(hc - 1u);
                }
                const bool seed = hc == 1u;
                if (!longrow || seed || (LINES && by_query)) {
                    int val = -1;
                    if (!seed) {
                        if constexpr (LINES) {
                            if constexpr (STAGED) val = by_query ? my_line[qq] : my_eids[jp];
                            else val = by_query ? my_line[qq] : my_row[jp];
                        } else {
                            if constexpr (STAGED) val = my_eids[jp];
                            else val = my_row[jp];
                        }
                    }
                    int32_t *const pp = a.pred + base;
                    pp[rank] = val;
                }
            }
            __builtin_amdgcn_s_barrier();  // the sixteen tiles write their pieces of a query together
        }
    }
}

__global__ void __launch_bounds__(kEmitTiles * 64) __attribute__((amdgpu_waves_per_eu(8, 8)))
k_pred_emit(FillArgs a, const unsigned long long *__restrict__ codes, const unsigned long long *__restrict__ visbuf,
            long long tile0, long long ntile, int w0, int nw, int wsplit, int eid_cap, int line_cap) {
    constexpr int Qp = 1024, TPB = kEmitTiles;
    __shared__ int eid_tab[kEmitEids];
    __shared__ int rp_tab[kEmitLines * 64];
    __shared__ unsigned long long s_live[2];
    __shared__ int s_wsum[2][TPB];
    const long long L = xcd_contiguous(blockIdx.x, gridDim.x);
    const long long nsup = (ntile + TPB - 1) / TPB;
    if (L >= nsup * wsplit) return;  // block-uniform
    const int part = (int)(L % wsplit);
    const int t = threadIdx.x, wave = t >> 6, v = lane();
    const long long tile_rel = (L / wsplit) * TPB + wave, tile = tile0 + tile_rel;
    const bool valid = tile_rel < ntile;  // wave-uniform
    if (t < 2) s_live[t] = 0ull;
    // ---- once per block: the tiles' entities (lane = entity)
    const long long ew = valid ? tile_entity(a.tile_ent, tile, v, a.E) : -1;
    uint32_t wlo = 0, whi = 0;
    if (ew >= 0) {
        wlo = a.in_off[ew];
        whi = a.in_off[ew + 1];
    }
    const uint32_t wdeg = whi - wlo;
    // where a lane's predecessors come from: the edge ids of its own short row (by row position),
    // its line of row_pred (by query), or nowhere (the block-per-row kernel writes them).  Seeds
    // get their -1 in the loop.
    const bool longrow = wdeg > (uint32_t)kTailMaxDegree;
    const bool by_query = longrow && a.row_pred;
    int li = 0;
    if (by_query) li = (int)(a.long_index[ew] - a.row_base);
    const int n_stage = longrow ? 0 : (int)wdeg;
    int wtot, ltot;
    int off = wave_excl_scan(n_stage, wtot);
    const unsigned long long bq_wave = __ballot(by_query);
    int slot = __popcll(bq_wave & ((1ull << v) - 1ull));
    ltot = __popcll(bq_wave);
    if (v == 0) {
        s_wsum[0][wave] = wtot;
        s_wsum[1][wave] = ltot;
    }
    __syncthreads();
    int total = 0, lines = 0, line0 = 0;
#pragma unroll
    for (int x = 0; x < TPB; ++x) {
        if (x < wave) {
            off += s_wsum[0][x];
            line0 += s_wsum[1][x];
        }
        total += s_wsum[0][x];
        lines += s_wsum[1][x];
    }
    slot += line0;
    const bool staged = total <= eid_cap, lined = lines <= line_cap;  // block-uniform
    if (staged)  // eight entries of the lane's row are requested before the first is stored
        for (int i0 = 0; i0 < n_stage; i0 += 8) {
            int e[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) e[x] = i0 + x < n_stage ? a.in_eid[wlo + i0 + x] : 0;
#pragma unroll
            for (int x = 0; x < 8; ++x)
                if (i0 + x < n_stage) eid_tab[off + i0 + x] = e[x];
        }
    const int ent_id = (int)ew;
    const int *const my_eids = eid_tab + (staged ? off : 0);
    const int32_t *const my_row = a.in_eid + wlo;
    const int *const my_line = rp_tab + (lined ? slot : 0) * 64;
    int turn = 0;
    for (int wi = part; wi < nw; wi += wsplit, turn ^= 1) {  // block-uniform trip count
        const int w = w0 + wi;
        // where query 64 w + v continues in this tile (lane = query here)
        long long pos = 0;
        const int ql = w * 64 + v;
        if (valid && ql >= a.q0 && ql < a.q1)
            pos = super_start(a, tile / kSuperTiles, Qp, ql) + a.tile_base[(size_t)tile * Qp + ql];
        // lane = entity: one code byte per query of the word, (row position << 3) | (hop + 1), zero where
        // the query did not reach the entity; vis = the queries that reached it
        uint32_t c[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) c[i] = 0;
        unsigned long long vis = 0;
        if (ew >= 0) {
            const size_t at = ((size_t)tile_rel * nw + wi) * 64 + v;
            const uint4 *in = reinterpret_cast<const uint4 *>(codes) + at * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint4 x = in[i];
                c[4 * i] = x.x; c[4 * i + 1] = x.y; c[4 * i + 2] = x.z; c[4 * i + 3] = x.w;
            }
            vis = visbuf[at];
        }
        // the row_pred values of this word: 64 queries x the wavefront's entities of that kind, eight
        // lines requested together (lanes = queries)
        if (lined) {
            unsigned long long bq = bq_wave;
            int s_at = line0;
            while (bq) {
                int val[8];
                int n = 0;
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    val[x] = 0;
                    if (bq) {
                        const int Lx = __builtin_ctzll(bq);
                        bq &= bq - 1;
                        val[x] = a.row_pred[(size_t)__builtin_amdgcn_readlane(li, Lx) * Qp + ql];
                        ++n;
                    }
                }
#pragma unroll
                for (int x = 0; x < 8; ++x)
                    if (x < n) rp_tab[(s_at + x) * 64 + v] = val[x];
                s_at += n;
            }
        }
        const unsigned long long live_wave = wave_or64(vis);
        if (v == 0 && live_wave) atomicOr(&s_live[turn], live_wave);
        __syncthreads();
        const unsigned long long live = s_live[turn];
        if (t == 0) s_live[turn ^ 1] = 0ull;  // for the next word (read again only after its barrier)
        uint32_t pos_lo = (uint32_t)(unsigned long long)pos, pos_hi = (uint32_t)((unsigned long long)pos >> 32);
        if (live != 0ull) {  // block-uniform
            if (!lined) {
                // Entities whose predecessors wait in row_pred, too many for rp_tab: lanes = queries.
                // Lane i knows where query i's run of this tile starts (pos) and, after a 64 x 64
                // transpose of the visited words, which of the tile's entities query i reached: the
                // rank of entity L in the run is the number of those below L.  Four lines are
                // requested before the first is stored.  Seeds (hop + 1 == 1) are left to the loop.
                unsigned long long bq = bq_wave;
                if (bq) {
                    const unsigned long long mT = transpose64(vis);
                    unsigned long long seed_w = 0;
#pragma unroll
                    for (int i = 0; i < 16; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            seed_w |= (unsigned long long)(((c[i] >> (8 * j)) & 7u) == 1u) << (4 * i + j);
                    const uint32_t seed_lo = (uint32_t)seed_w, seed_hi = (uint32_t)(seed_w >> 32);
                    const int32_t *const rp = a.row_pred + ql;
                    int32_t *const pp = a.pred + pos;
                    while (bq) {
                        int Lx[4], val[4];
                        bool on[4];
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            Lx[x] = -1;
                            on[x] = false;
                            val[x] = 0;
                            if (bq) {
                                Lx[x] = __builtin_ctzll(bq);
                                bq &= bq - 1;
                                const int liL = __builtin_amdgcn_readlane(li, Lx[x]);
                                const unsigned long long seedL =
                                    ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)seed_hi, Lx[x]) << 32) |
                                    (uint32_t)__builtin_amdgcn_readlane((int)seed_lo, Lx[x]);
                                on[x] = ((mT >> Lx[x]) & 1ull) && !((seedL >> v) & 1ull);
                                if (on[x]) val[x] = rp[(size_t)liL * Qp];
                            }
                        }
#pragma unroll
                        for (int x = 0; x < 4; ++x)
                            if (on[x]) pp[__popcll(mT & ((1ull << Lx[x]) - 1ull))] = val[x];
                    }
                }
            }
            // Everything requested from memory so far is consumed here, so that the loop holds stores
            // only: a wait on a load inside it would also wait for the loop's own stores.
            asm volatile("" : "+v"(pos_lo), "+v"(pos_hi));
            if (staged) {
                if (lined) emit_word<true, true>(a, c, live, pos_lo, pos_hi, ent_id, longrow, by_query, my_eids, my_row, my_line);
                else emit_word<true, false>(a, c, live, pos_lo, pos_hi, ent_id, longrow, by_query, my_eids, my_row, my_line);
            } else {
                if (lined) emit_word<false, true>(a, c, live, pos_lo, pos_hi, ent_id, longrow, by_query, my_eids, my_row, my_line);
                else emit_word<false, false>(a, c, live, pos_lo, pos_hi, ent_id, longrow, by_query, my_eids, my_row, my_line);
            }
        }
        __syncthreads();  // rp_tab is rewritten for the next word
    }
}

// Object rows of more than 32 entries: one block per row (4 waves; 16 for hub
// rows).  Phase 1 rebuilds the list positions of the row's entity (ranks inside
// its tile).  Phase 2 walks the row in steps of (waves x 4 x 64) entries: inside a
// step the waves take disjoint 64-entry chunks (interleaved, so that a row
// shorter than a step still occupies every wave) and keep, per query, the smallest
// edge id any of them found (LDS atomicMin); after the step the resolved queries
// are removed from the shared mask, so a later step (larger edge ids) never
// touches them.  Each predecessor is then written once.
// SEG (row-buffer mode only): a block per kGiantSegment entries of a giant row instead of one per
// row; the blocks of a row keep the smallest edge id per query in the row's line of the row buffer
// (atomicMin; the line starts at INT_MAX).  A block that walks a whole 140,000-entry row is a chain
// of dependent gathers that outlasts everything else in the launch; the segments of a row run side
// by side, at the price of the early exit between them (it saved a quarter of the entries).
// ONE: as in k_pred_wave.
template <int W, bool MASK, bool STATS, bool BUF, bool SEG = false, bool ONE = false>
__global__ void __launch_bounds__(1024) k_pred_row(FillArgs a, long long first_row) {
    static_assert(!SEG || BUF, "segments merge in the row buffer");
    static_assert(!ONE || (W == 16 && !STATS), "the one-word form is for 16-word lines");
    constexpr int Qp = 64 * W;
    constexpr int C = 4;  // 64-entry chunks per wavefront and step, loaded together
    __shared__ long long slot[BUF ? 1 : Qp];
    __shared__ int smin[Qp];
    __shared__ unsigned long long srem[16], slevel[16];
    long long row_i = blockIdx.x;
    uint32_t seg = 0;
    if (SEG) {  // the giant row this segment belongs to: last row whose first segment is <= blockIdx.x
        long long lo_r = 0, hi_r = a.n_giant_rows;
        while (hi_r - lo_r > 1) {
            const long long m = (lo_r + hi_r) >> 1;
            if (a.giant_seg_first[m] <= blockIdx.x) lo_r = m; else hi_r = m;
        }
        row_i = lo_r;
        seg = blockIdx.x - a.giant_seg_first[lo_r];
    }
    const int ev = a.rows[first_row + row_i];
    const int t = threadIdx.x, wave = t >> 6, nw = blockDim.x >> 6, v = lane(), lw = v & (W - 1);
    // gridDim.y > 1: one block per (row, hop level), so the levels of a long row run side by side
    const int h_first = gridDim.y > 1 ? (int)blockIdx.y + 1 : 1, h_last = gridDim.y > 1 ? h_first : a.k;
    if (gridDim.y > 1) {  // nothing of this level in the row's entity: leave before the list positions
        const unsigned long long x =
            lw < W ? a.levels[(size_t)h_first * a.plane + (size_t)ev * W + lw] & range_bits(a.q0, a.q1, lw) : 0ull;
        if (!wave_any(x != 0) || ((a.push_levels >> h_first) & 1u)) return;  // the same words in every wavefront
    }
    if (!BUF) row_slots<W>(a, ev, wave, nw, slot);
    int32_t *out = BUF ? a.row_pred + (size_t)(first_row + row_i) * Qp : a.pred;
    const uint32_t row_lo = a.in_off[ev], row_hi = a.in_off[ev + 1];
    const uint32_t lo = SEG ? row_lo + seg * (uint32_t)kGiantSegment : row_lo;
    const uint32_t hi = SEG ? min(row_hi, lo + (uint32_t)kGiantSegment) : row_hi;
    long long n_rows = 0, n_edges = 0, n_lines = 0;
    for (int h = h_first; h <= h_last; ++h) {
        __syncthreads();
        if (t < 16) {
            unsigned long long x =
                t < W ? a.levels[(size_t)h * a.plane + (size_t)ev * W + t] & range_bits(a.q0, a.q1, t) : 0ull;
            srem[t] = x;
            slevel[t] = x;
        }
        for (int q = t; q < Qp; q += blockDim.x) smin[q] = INT_MAX;
        __syncthreads();
        if (!wave_any(slevel[lw] != 0) || ((a.push_levels >> h) & 1u)) continue;  // block-uniform
        const uint32_t *act_prev = a.act + (size_t)(h - 1) * a.actw;
        const unsigned long long *prev = a.levels + (size_t)(h - 1) * a.plane;
        const bool dense = !STATS && ((a.dense_levels >> h) & 1u);  // the line of an entity outside the level is zero
        if (wave == 0) ++n_rows;
        // The first step is short (one chunk per wavefront): on a dense frontier the first
        // candidates of a row resolve most queries, and what is resolved after that step is not
        // claimed again by sixteen wavefronts in parallel.
        uint32_t span = 64u * nw;
        for (uint32_t s0 = lo; s0 < hi; s0 += span, span = 64u * C * nw) {
            const uint32_t step_hi = min(hi, s0 + span);
            const int lr = ONE ? (a.q0 >> 6) : lw;  // the word of the shared mask this lane works on
            unsigned long long rem = srem[lr];
            if (!wave_any(rem != 0)) break;  // same decision in every wave
            const unsigned long long before = rem;
            // chunk c of this wavefront is chunk c * nw + wave of the step: a row shorter than a
            // step still spreads over all wavefronts
            const uint32_t w0 = s0 + 64u * wave;
            int sj[C];
            bool cj[C];
#pragma unroll
            for (int c = 0; c < C; ++c) {  // all loads of the step first
                uint32_t j = w0 + 64u * nw * c + v;
                sj[c] = 0;
                cj[c] = false;
                if (j < step_hi) {
                    sj[c] = a.in_sub[j];
                    cj[c] = dense || ((act_prev[sj[c] >> 5] >> (sj[c] & 31)) & 1u);
                }
            }
#pragma unroll
            for (int c = 0; c < C; ++c) {
                uint32_t j0 = w0 + 64u * nw * c;
                if (j0 < step_hi && wave_any(rem != 0)) {
                    if constexpr (ONE) {
                        n_lines += pred_resolve_word<MASK>(j0, sj[c], cj[c], lr, a, prev, rem,
                                                           [&](int q, int eid) { atomicMin(&smin[lr * 64 + q], eid); });
                    } else {
                        n_lines += pred_resolve_unordered<W, MASK>(j0, sj[c], cj[c], a, prev, rem,
                                                                   [&](unsigned long long hit, int eid) {
                            for (unsigned long long m = hit; m; m &= m - 1)
                                atomicMin(&smin[lw * 64 + (__ffsll((long long)m) - 1)], eid);
                        });
                    }
                    n_edges += min((uint32_t)64, step_hi - j0);
                }
            }
            unsigned long long resolved = before & ~rem;  // by this group of lanes (ONE: by this wavefront)
            __syncthreads();
            if (resolved && (!ONE || v == 0)) atomicAnd(&srem[lr], ~resolved);
            __syncthreads();
        }
        __syncthreads();
        for (int q = t; q < Qp; q += blockDim.x)
            if ((slevel[q >> 6] >> (q & 63)) & 1ull) {
                if (SEG) {
                    if (smin[q] != INT_MAX) atomicMin(&out[q], smin[q]);
                } else {
                    out[BUF ? (long long)q : slot[q]] = smin[q];
                }
            }
    }
    if (STATS && v == 0) {
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

// The list of a result's active entities and their positions in it, built once per result.  The
// tiles of every count / list / predecessor kernel of a resident graph are cut from this list.
// A sharded graph keeps tiles of consecutive ids: its predecessor pass works on ranges of ids,
// the ranges its object-sorted triples are streamed in.
static logoskg_status ensure_active_list(logoskg_result *r, hipStream_t st) {
    logoskg_graph *g = r->g;
    if (r->tile_ent || g->num_shards > 1) return LOGOSKG_OK;
    const long long actw = r->Epad / 32, nchunks = (actw + kActChunkWords - 1) / kActChunkWords;
    LKG_TRY(g->pool.alloc((void **)&r->tile_ent, ((size_t)r->Epad + 64) * sizeof(int32_t), st));
    LKG_TRY(g->pool.alloc((void **)&r->cpos, (size_t)r->Epad * sizeof(int32_t), st));
    LKG_TRY(g->pool.alloc((void **)&r->act_chunk, ((size_t)nchunks + 2) * sizeof(uint32_t) + 8, st));
    r->d_nact = reinterpret_cast<unsigned long long *>(r->act_chunk + (nchunks + 1) / 2 * 2);
    r->n_active = -1;
    ProfScope ps(g->prof, KK_SCAN, st);
    const unsigned nb = (unsigned)((nchunks + 3) / 4);
    k_active_count<<<dim3(nb), dim3(256), 0, st>>>(r->act, actw, r->k + 1, nchunks, r->act_chunk);
    k_active_scan<<<dim3(1), dim3(1024), 0, st>>>(nchunks, r->act_chunk, r->d_nact, r->tile_ent);
    k_active_fill<<<dim3(nb), dim3(256), 0, st>>>(r->act, actw, r->k + 1, nchunks, r->act_chunk, r->tile_ent, r->cpos);
    LKG_HIP(hipGetLastError());
    return LOGOSKG_OK;
}

// Per-query counts of the set bits of one plane (visited, or a level) as three nested exclusive
// prefixes plus the offsets of the query-major lists; the tables are allocated on first use.
static logoskg_status count_plane(logoskg_result *r, const unsigned long long *plane_bits, uint16_t **tile_base,
                                  uint32_t **super_base, uint32_t **mega_base, long long **d_off,
                                  std::vector<int64_t> *off, hipStream_t st) {
    logoskg_graph *g = r->g;
    const int W = r->W, Qp = 64 * W;
    const long long ntiles = r->Epad / kTileEntities;
    const long long nsuper = (ntiles + kSuperTiles - 1) / kSuperTiles;
    const long long nmega = (nsuper + kMegaSupers - 1) / kMegaSupers;
    r->last_stream = st;
    if (!*tile_base) LKG_TRY(g->pool.alloc((void **)tile_base, (size_t)ntiles * Qp * 2, st));
    if (!*super_base) LKG_TRY(g->pool.alloc((void **)super_base, (size_t)nsuper * Qp * 4, st));
    if (!*mega_base) LKG_TRY(g->pool.alloc((void **)mega_base, (size_t)nmega * Qp * 4, st));
    if (!*d_off) LKG_TRY(g->pool.alloc((void **)d_off, (size_t)(Qp + 1) * 8, st));
    LKG_TRY(ensure_active_list(r, st));
    {
        ProfScope ps(g->prof, KK_COUNT, st);
        dim3 grid((unsigned)nsuper), block(Qp);
        switch (W) {
            case 1: k_count<1><<<grid, block, 0, st>>>(plane_bits, ntiles, g->E, r->tile_ent, r->d_nact, *tile_base, *super_base); break;
            case 4: k_count<4><<<grid, block, 0, st>>>(plane_bits, ntiles, g->E, r->tile_ent, r->d_nact, *tile_base, *super_base); break;
            default: k_count<16><<<grid, block, 0, st>>>(plane_bits, ntiles, g->E, r->tile_ent, r->d_nact, *tile_base, *super_base); break;
        }
    }
    {
        ProfScope ps(g->prof, KK_SCAN, st);
        const int threads = std::min(Qp, 256);
        k_scan_level<<<dim3((unsigned)nmega, (unsigned)(Qp / threads)), dim3(threads), 0, st>>>(
            nsuper, kMegaSupers, Qp, *super_base, *mega_base);
        k_scan_top<<<dim3(1), dim3(Qp), 0, st>>>(nmega, r->Q, Qp, *mega_base, *d_off);
    }
    LKG_HIP(hipGetLastError());
    off->assign((size_t)r->Q + 1, 0);
    LKG_HIP(hipMemcpyAsync(off->data(), *d_off, (size_t)(r->Q + 1) * 8, hipMemcpyDeviceToHost, st));
    unsigned long long *h_nact = g->h_ctr + C_TOTAL;  // one more pinned word behind the counters' mirror
    if (r->tile_ent && r->n_active < 0)
        LKG_HIP(hipMemcpyAsync(h_nact, r->d_nact, 8, hipMemcpyDeviceToHost, st));
    LKG_HIP(hipStreamSynchronize(st));
    if (r->tile_ent && r->n_active < 0) r->n_active = (long long)*h_nact;
    if (g->prof.on) g->prof.acc[KK_COUNT].units[3] += (r->tile_ent ? (r->n_active + 63) / 64 * 64 : r->Epad) * W;
    return LOGOSKG_OK;
}

logoskg_status count_reached(logoskg_result *r, hipStream_t st) {
    LKG_TRY(count_plane(r, r->visited, &r->tile_base, &r->super_base, &r->mega_base, &r->d_reached_off,
                        &r->reached_off, st));
    r->has_counts = true;
    return LOGOSKG_OK;
}

__global__ void k_long_index(const int32_t *__restrict__ rows, long long n, int32_t *index) {
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) index[rows[i]] = (int32_t)i;
}

// First predecessor fetch with 16-word planes: the entity -> long-row position map and the
// buffer the row kernels write to (one 1024-query line per long row of a launch).  A graph whose
// buffer would pass 8 GiB keeps the direct path.
logoskg_status prepare_row_pred(logoskg_graph *g, hipStream_t st) {
    if (g->row_pred_tried) return LOGOSKG_OK;
    g->row_pred_tried = true;
    // code bytes and visited words between the two kernels of the bit-sliced predecessor pass: room
    // for every tile of the graph and 16 words, but not more than 1.25 GiB
    g->plane_buf_bytes = std::min<size_t>((size_t)5 << 28, (size_t)(g->Epad / 64 + kEmitTiles) * 16 * 64 * (64 + 8));
    if (hipMalloc((void **)&g->plane_buf, g->plane_buf_bytes) != hipSuccess) {
        (void)hipGetLastError();
        g->plane_buf = nullptr;
        g->plane_buf_bytes = 0;
    }
    LKG_HIP(hipEventCreateWithFlags(&g->ev_rows, hipEventDisableTiming));

    const long long rows = g->num_shards > 1 ? max_chunk_rows(g) : (long long)g->in_rows.n_long;
    if (rows <= 0 || (size_t)rows * 4096 > ((size_t)8 << 30)) return LOGOSKG_OK;
    LKG_HIP(hipMalloc((void **)&g->long_index, (size_t)g->E * sizeof(int32_t)));
    if (hipMalloc((void **)&g->row_pred, (size_t)rows * 4096) != hipSuccess) {
        (void)hipGetLastError();
        g->row_pred = nullptr;
        return LOGOSKG_OK;
    }
    g->row_pred_rows = rows;
    LKG_HIP(hipMemsetAsync(g->long_index, 0xFF, (size_t)g->E * sizeof(int32_t), st));  // -1: not a long row
    k_long_index<<<dim3((unsigned)((g->in_rows.n_long + 255) / 256)), dim3(256), 0, st>>>(g->in_rows.longrows,
                                                                                         g->in_rows.n_long, g->long_index);
    LKG_HIP(hipGetLastError());
    return LOGOSKG_OK;
}

template <int W>
static void launch_lists_w(Profiler &prof, const FillArgs &a, hipStream_t st) {
    constexpr int TILES = W == 16 ? kSuperTiles / 2 : kSuperTiles;
    const long long nblocks = (a.ntiles + TILES - 1) / TILES;
    ProfScope ps(prof, KK_LISTS, st);
    int nb = 1;
    while ((1 << nb) <= a.k) ++nb;
    dim3 grid((unsigned)nblocks), block(64 * W);
    if (!a.hop) k_lists<W, 0, TILES><<<grid, block, 0, st>>>(a);
    else if (nb <= 2) k_lists<W, 2, TILES><<<grid, block, 0, st>>>(a);
    else if (nb <= 4) k_lists<W, 4, TILES><<<grid, block, 0, st>>>(a);
    else k_lists<W, 8, TILES><<<grid, block, 0, st>>>(a);
}

// True when the 16-word tile kernel can serve this launch (it then can also write the entity and
// hop lists, see FillArgs::fuse_lists).
// A level with a small frontier (at most a quarter of the triples leave it: the first level, whose
// frontier is the seeds) reaches a long object row for few queries: walking the row from
// its first entry until each of them has met a frontier subject reads most of the row.  Such a
// level is resolved from the subject side instead: the out-rows of the frontier entities are
// walked as in a push hop, and an edge (u -> o, id t) with o a long row offers t, for every query in
// level[h-1](u) & level[h](o) (& the relation's whitelist), to o's line of the row buffer with an
// atomicMin.  k_pred_push_init first sets the level's entries of the long rows to INT_MAX.
__global__ void __launch_bounds__(256) k_pred_push_init(FillArgs a, int h, long long n_rows) {
    const long long i = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n_rows) return;  // wavefront-uniform
    const int ev = a.rows[i];
    if (!((a.act[(size_t)h * a.actw + (ev >> 5)] >> (ev & 31)) & 1u)) return;
    const int w0 = a.q0 >> 6, w1 = (a.q1 - 1) >> 6;
    for (int w = w0; w <= w1; ++w) {
        const unsigned long long x = a.levels[(size_t)h * a.plane + (size_t)ev * 16 + w] & range_bits(a.q0, a.q1, w);
        if ((x >> lane()) & 1ull) a.row_pred[(size_t)i * 1024 + w * 64 + lane()] = INT_MAX;
    }
}

// One wavefront per short frontier row (SEG = false) or per 64-entry segment of a longer one; lane = out-edge.
template <bool MASK, bool SEG>
__global__ void __launch_bounds__(256)
k_pred_push(FillArgs a, int h, const int32_t *__restrict__ tail_rows, const RowSegment *__restrict__ segs,
            const unsigned long long *__restrict__ ctr, const uint32_t *__restrict__ out_off,
            const int32_t *__restrict__ out_obj, const uint16_t *__restrict__ out_rel,
            const int32_t *__restrict__ out_eid) {
    const long long item = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (item >= (long long)ctr[SEG ? C_NSEG : C_NTAIL]) return;  // wavefront-uniform
    int u;
    uint32_t lo, hi;
    if (SEG) {
        const RowSegment sg = segs[item];
        u = sg.row;
        lo = sg.begin;
        hi = min(lo + (uint32_t)kPushSegment, out_off[u + 1]);
    } else {
        u = tail_rows[item];
        lo = out_off[u];
        hi = out_off[u + 1];
    }
    const int w0 = a.q0 >> 6, w1 = (a.q1 - 1) >> 6, v = lane();
    unsigned long long mine = 0;  // lane w: word w of the subject's frontier line
    if (v >= w0 && v <= w1)
        mine = a.levels[(size_t)(h - 1) * a.plane + (size_t)u * 16 + v] & range_bits(a.q0, a.q1, v);
    if (!wave_any(mine != 0)) return;  // none of the fetched queries has this subject in its frontier
    const uint32_t j = lo + (uint32_t)v;  // a segment holds at most 64 entries, a short row 32
    int o = 0, li = -1, rl = 0, eid = 0;
    if (j < hi) {
        o = out_obj[j];
        li = a.long_index[o];  // -1: a short object row, which the row walk of the tiles resolves
        if (li >= 0) {
            eid = out_eid[j];
            if (MASK) rl = out_rel[j];
        }
    }
    for (int w = w0; w <= w1; ++w) {
        const unsigned long long lu = shfl64(mine, w);
        if (lu == 0ull || li < 0) continue;
        unsigned long long m = lu & a.levels[(size_t)h * a.plane + (size_t)o * 16 + w];
        if (MASK && m) m &= a.allow[(size_t)rl * 16 + w];
        for (; m; m &= m - 1)
            atomicMin(&a.row_pred[(size_t)li * 1024 + w * 64 + (__ffsll((long long)m) - 1)], eid);
    }
}

bool pred_uses_staged_kernel(const FillArgs &a, int W) {
    return W == 16 && a.k <= kSlicedMaxK && a.plane_buf != nullptr;
}

__global__ void k_fill_int(int32_t *p, long long n, int32_t value) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

template <int W>
constexpr long long Qp_of() { return 64 * W; }

template <int W, bool MASK, bool STATS>
static void launch_pred_wms(Profiler &prof, const FillArgs &a0, long long n_hub_rows, long long n_other_rows,
                            hipStream_t st_tiles, hipStream_t st_hub) {
    FillArgs a = a0;
    const bool mt = pred_uses_staged_kernel(a, W);
    if (!mt) {
        a.row_pred = nullptr;
        a.fuse_lists = 0;
    }
    if (!mt || W != 16 || STATS) a.push_levels = 0;
    // a fetch whose queries sit in one word of 16-word lines: the row kernels take an entry per lane
    const bool one = W == 16 && !STATS && a.q1 > a.q0 && (a.q0 >> 6) == ((a.q1 - 1) >> 6);
    // issued first: the tile kernel waits for it, and launched after the hub kernel it ran half as fast
    if (n_other_rows > 0) {  // with row_pred: must precede the tile kernel on its stream
        hipStream_t st = a.row_pred ? st_tiles : st_hub;
        ProfScope ps(prof, KK_PRED_MID, st);
        const dim3 gw((unsigned)((n_other_rows + 3) / 4));
        bool done = false;
        if constexpr (W == 16 && !STATS) {
            if (one) {
                if (a.row_pred) k_pred_wave<W, MASK, STATS, true, true><<<gw, dim3(256), 0, st>>>(a, n_hub_rows, n_other_rows);
                else k_pred_wave<W, MASK, STATS, false, true><<<gw, dim3(256), 0, st>>>(a, n_hub_rows, n_other_rows);
                done = true;
            }
        }
        if (done) {
        } else if (a.row_pred) k_pred_wave<W, MASK, STATS, true><<<gw, dim3(256), 0, st>>>(a, n_hub_rows, n_other_rows);
        else k_pred_wave<W, MASK, STATS, false><<<gw, dim3(256), 0, st>>>(a, n_hub_rows, n_other_rows);
    }
    if (n_hub_rows > 0) {  // writes the lists itself: independent of the other two kernels
        ProfScope ps(prof, KK_PRED_HUB, st_hub);
        // 16 wavefronts per row for the longest rows, 4 for the others: a row of a thousand entries
        // leaves most of a large block waiting at its barriers, and the smaller blocks disturb the
        // tile kernel less while both run
        const long long giants = a.n_giant_rows < 0 ? n_hub_rows : std::min(a.n_giant_rows, n_hub_rows);
        // and one block per hop level of a row: the levels are independent, and the longest row
        // sets the duration of the launch
        const unsigned levels = (unsigned)std::max(a.k, 1);
        auto rows = [&](auto one_c) {
            constexpr bool ONE = decltype(one_c)::value;
            if (a.row_pred) {  // into the row buffer, from which the list writer takes them
                if (giants > 0 && a.giant_seg_first && giants == a.n_giant_rows) {
                    k_fill_int<<<dim3((unsigned)((giants * Qp_of<W>() + 255) / 256)), dim3(256), 0, st_hub>>>(
                        a.row_pred, giants * Qp_of<W>(), INT_MAX);
                    k_pred_row<W, MASK, STATS, true, true, ONE><<<dim3((unsigned)a.n_giant_segs, levels), dim3(1024), 0, st_hub>>>(a, 0);
                } else if (giants > 0)
                    k_pred_row<W, MASK, STATS, true, false, ONE><<<dim3((unsigned)giants, levels), dim3(1024), 0, st_hub>>>(a, 0);
                if (n_hub_rows > giants)
                    k_pred_row<W, MASK, STATS, true, false, ONE><<<dim3((unsigned)(n_hub_rows - giants), levels), dim3(256), 0, st_hub>>>(
                        a, giants);
            } else {  // straight into the lists
                if (giants > 0)
                    k_pred_row<W, MASK, STATS, false, false, ONE><<<dim3((unsigned)giants, levels), dim3(1024), 0, st_hub>>>(a, 0);
                if (n_hub_rows > giants)
                    k_pred_row<W, MASK, STATS, false, false, ONE><<<dim3((unsigned)(n_hub_rows - giants), levels), dim3(256), 0, st_hub>>>(
                        a, giants);
            }
        };
        bool done = false;
        if constexpr (W == 16 && !STATS) {
            if (one) {
                rows(std::true_type{});
                done = true;
            }
        }
        if (!done) rows(std::false_type{});
    }
    if constexpr (W == 16 && !STATS) {
        if (a.push_levels) {  // the pushed levels of the long rows, from the subject side (behind the row kernels:
                              // the giant rows' lines are filled before those run)
            logoskg_graph *g = static_cast<logoskg_graph *>(a.host_graph);
            logoskg_result *r = static_cast<logoskg_result *>(a.host_result);
            const long long n_long = n_hub_rows + n_other_rows;
            for (int h = 1; h <= a.k && n_long > 0; ++h) {
                if (!((a.push_levels >> h) & 1u)) continue;
                // (timed with the row kernels whose work it takes over; profiler scopes do not nest)
                if (census_lists(g, r, h - 1, -1, st_hub, KK_PRED_HUB) != LOGOSKG_OK) break;  // (the caller reads the last error)
                ProfScope ps(prof, KK_PRED_HUB, st_hub);
                k_pred_push_init<<<dim3((unsigned)((n_long + 3) / 4)), dim3(256), 0, st_hub>>>(a, h, n_long);
                // the lists' lengths are on the device; the hop's own statistics bound them
                const long long rows = r->stats[(size_t)h - 1].active_rows;
                const long long max_seg = rows + r->stats[(size_t)h - 1].frontier_edges / kPushSegment;
                if (rows > 0) {
                    k_pred_push<MASK, false><<<dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st_hub>>>(
                        a, h, g->fr_tail, g->fr_seg, g->d_ctr, g->out_off, g->out_obj, g->out_rel, g->out_eid);
                    k_pred_push<MASK, true><<<dim3((unsigned)((max_seg + 3) / 4)), dim3(256), 0, st_hub>>>(
                        a, h, g->fr_tail, g->fr_seg, g->d_ctr, g->out_off, g->out_obj, g->out_rel, g->out_eid);
                }
            }
        }
    }
    // the list writer reads the row buffer: it starts behind the block-per-row kernel
    const bool rows_first = n_hub_rows > 0 && a.row_pred && mt && st_hub != st_tiles && a.ev_rows;
    if (rows_first) (void)hipEventRecord((hipEvent_t)a.ev_rows, st_hub);
    if (a.tile_count > 0 && mt) {
        // in chunks of tiles whose code bytes (64 per entity and word) and visited words fit the buffer
        const int w0 = a.q0 / 64, nw = (a.q1 - 1) / 64 - w0 + 1;
        const size_t per_tile = (size_t)nw * 64 * (64 + 8);
        long long chunk = (long long)(a.plane_buf_bytes / per_tile);
        chunk = std::max<long long>(kEmitTiles, chunk / kEmitTiles * kEmitTiles);
        for (long long c0 = 0; c0 < a.tile_count; c0 += chunk) {
            const long long n = std::min(chunk, a.tile_count - c0), t0 = a.tile_begin + c0;
            unsigned long long *visbuf = a.plane_buf + (size_t)n * nw * 64 * 8;  // behind the codes
            // each block of the second kernel takes every wsplit-th word: enough blocks to go
            // round the GPU a few times, as many words per block as that allows
            const long long nsup = (n + kEmitTiles - 1) / kEmitTiles;
            int wsplit = 1;
            while (wsplit < nw && nsup * wsplit < 8192) wsplit *= 2;
            wsplit = std::min(wsplit, nw);
            dim3 gw((unsigned)((n * 4 + 7) / 8 * 8));
            dim3 ge((unsigned)((nsup * wsplit + 7) / 8 * 8));
            {
                ProfScope ps(prof, KK_PRED_WALK, st_tiles);
                // a range inside four aligned words takes four lanes per entity (16 entities per wavefront)
                const int wb = w0 & ~3;
                if (nw == 1) {  // one word: a lane per entity (64 entities per wavefront)
                    dim3 g1((unsigned)(((n + 3) / 4 + 7) / 8 * 8));  // 256 entities per block
                    if (a.k <= 2) k_pred_walk<2, MASK, STATS, 1><<<g1, dim3(256), 0, st_tiles>>>(a, a.plane_buf, visbuf, t0, n, w0, nw, w0);
                    else k_pred_walk<3, MASK, STATS, 1><<<g1, dim3(256), 0, st_tiles>>>(a, a.plane_buf, visbuf, t0, n, w0, nw, w0);
                } else if (w0 + nw <= wb + 4) {
                    dim3 g4((unsigned)((n + 7) / 8 * 8));  // 64 entities per block
                    if (a.k <= 2) k_pred_walk<2, MASK, STATS, 4><<<g4, dim3(256), 0, st_tiles>>>(a, a.plane_buf, visbuf, t0, n, w0, nw, wb);
                    else k_pred_walk<3, MASK, STATS, 4><<<g4, dim3(256), 0, st_tiles>>>(a, a.plane_buf, visbuf, t0, n, w0, nw, wb);
                } else {
                    if (a.k <= 2) k_pred_walk<2, MASK, STATS, 16><<<gw, dim3(256), 0, st_tiles>>>(a, a.plane_buf, visbuf, t0, n, w0, nw, 0);
                    else k_pred_walk<3, MASK, STATS, 16><<<gw, dim3(256), 0, st_tiles>>>(a, a.plane_buf, visbuf, t0, n, w0, nw, 0);
                }
            }
            if (rows_first && c0 == 0) (void)hipStreamWaitEvent(st_tiles, (hipEvent_t)a.ev_rows, 0);
            ProfScope ps(prof, KK_PRED, st_tiles);
            k_pred_emit<<<ge, dim3(kEmitTiles * 64), 0, st_tiles>>>(a, a.plane_buf, visbuf, t0, n, w0, nw, wsplit,
                                                                   a.emit_eid_cap, a.emit_line_cap);
            if (prof.on) {  // entities x words whose code bytes pass from the first kernel to the second
                prof.acc[KK_PRED_WALK].units[3] += n * 64 * nw;
                prof.acc[KK_PRED].units[0] += n * 64 * nw;
            }
        }
    } else if (a.tile_count > 0) {
        ProfScope ps(prof, KK_PRED, st_tiles);
        dim3 grid((unsigned)((a.tile_count + 7) / 8 * 8)), block(64 * W);
        k_pred<W, MASK, STATS><<<grid, block, 0, st_tiles>>>(a);
    }
}

// predecessor kernels over the tiles [a.tile_begin, +a.tile_count) and the long rows a.rows[0 ..
// n_hub_rows + n_other_rows): the hub rows first (16 waves per row), then the others (one wave
// each).  The counting mode runs instantiations of its own, so that kernel statistics of the
// ordinary ones are not mixed with it.
template <int W>
static void launch_pred_w(Profiler &prof, const FillArgs &a, long long n_hub_rows, long long n_other_rows,
                          bool mask, hipStream_t st_tiles, hipStream_t st) {
    const bool stats = a.stats_pred != nullptr;
    if (mask) {
        if (stats) launch_pred_wms<W, true, true>(prof, a, n_hub_rows, n_other_rows, st_tiles, st);
        else launch_pred_wms<W, true, false>(prof, a, n_hub_rows, n_other_rows, st_tiles, st);
    } else {
        if (stats) launch_pred_wms<W, false, true>(prof, a, n_hub_rows, n_other_rows, st_tiles, st);
        else launch_pred_wms<W, false, false>(prof, a, n_hub_rows, n_other_rows, st_tiles, st);
    }
}

void launch_lists(Profiler &prof, const FillArgs &a, int W, hipStream_t st) {
    switch (W) {
        case 1: launch_lists_w<1>(prof, a, st); break;
        case 4: launch_lists_w<4>(prof, a, st); break;
        default: launch_lists_w<16>(prof, a, st); break;
    }
}

// The block-per-row kernel of the hub rows goes to st_hub and may overlap the rest; the kernel of
// the other long rows goes to st_tiles ahead of the tile kernel when its results pass through
// a.row_pred, to st_hub otherwise.
void launch_pred(Profiler &prof, const FillArgs &a, int W, long long n_hub_rows, long long n_other_rows, bool mask,
                 hipStream_t st_tiles, hipStream_t st_hub) {
    switch (W) {
        case 1: launch_pred_w<1>(prof, a, n_hub_rows, n_other_rows, mask, st_tiles, st_hub); break;
        case 4: launch_pred_w<4>(prof, a, n_hub_rows, n_other_rows, mask, st_tiles, st_hub); break;
        default: launch_pred_w<16>(prof, a, n_hub_rows, n_other_rows, mask, st_tiles, st_hub); break;
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
    if (r->walk_exact) {
        set_error("hop and predecessor are not defined for a LOGOSKG_WALK_EXACT result: use logoskg_result_level_fetch");
        return LOGOSKG_EINVAL;
    }
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
    r->last_stream = st;
    const int W = r->W;
    FillArgs a = {};
    a.E = g->E; a.Q = r->Q; a.k = r->k; a.q0 = q0; a.q1 = q1; a.hub_min = g->hub_min;
    a.tile_ent = r->tile_ent; a.cpos = r->cpos; a.n_listed = r->n_active;
    a.ntiles = r->tile_ent ? (r->n_active + 63) / 64 : r->Epad / kTileEntities;
    a.tile_begin = 0; a.tile_count = a.ntiles;
    a.plane = r->Epad * W; a.actw = r->Epad / 32;
    a.visited = r->visited; a.levels = r->levels; a.allow = r->allow;
    a.act = r->act; a.tile_base = r->tile_base; a.super_base = r->super_base; a.mega_base = r->mega_base;
    a.reached_off = r->d_reached_off;
    a.in_off = g->in_off; a.in_sub = g->in_sub; a.in_eid = g->in_eid; a.in_rel = g->in_rel;
    a.rows = g->in_rows.longrows;
    a.row_base = 0; a.long_index = nullptr; a.row_pred = nullptr; a.fuse_lists = 0;
    a.plane_buf = nullptr; a.plane_buf_bytes = 0; a.ev_rows = nullptr;
    // levels whose frontier (the level below) holds most of the triples: the same rule as the pull hops
    for (int h = 1; h <= r->k && h < 32; ++h)
        if ((long long)r->stats[(size_t)h - 1].frontier_edges * 100 >= g->T * (long long)kDensePullPercent)
            a.dense_levels |= 1u << h;
    a.n_giant_rows = g->num_shards > 1 ? -1 : g->in_rows.n_giant;
    a.giant_seg_first = g->num_shards > 1 ? nullptr : g->in_rows.giant_seg_first;
    a.n_giant_segs = g->num_shards > 1 ? 0 : g->in_rows.n_giant_segs;
    if (pred && W == 16) {
        LKG_TRY(prepare_row_pred(g, st));
        a.long_index = g->long_index;
        a.row_pred = g->row_pred;
        a.plane_buf = g->plane_buf;
        a.plane_buf_bytes = g->plane_buf_bytes;
        a.ev_rows = g->ev_rows;
        // (LOGOSKG_EMIT_CAPS="e,l" shrinks the two LDS tables of k_pred_emit so that tests reach its other paths)
        a.emit_eid_cap = kEmitEids;
        a.emit_line_cap = kEmitLines;
        if (const char *caps = getenv("LOGOSKG_EMIT_CAPS")) {
            int e = kEmitEids, l = kEmitLines;
            if (sscanf(caps, "%d,%d", &e, &l) == 2) {
                a.emit_eid_cap = std::max(0, std::min(e, kEmitEids));
                a.emit_line_cap = std::max(0, std::min(l, kEmitLines));
            }
        }
    }
    a.entity = entity; a.hop = hop; a.pred = pred;
    const bool counting = g->prof.counters;
    // levels whose frontier holds at most a quarter of the triples: their long rows are resolved from the
    // subject side (resident graphs, row buffer in use, minimum-hop search); needs the triple index of
    // every entry of SUB
    if (pred && W == 16 && g->num_shards <= 1 && !counting && !r->walk_exact && a.row_pred && a.long_index &&
        pred_uses_staged_kernel(a, W)) {
        uint32_t levels = 0;
        for (int h = 1; h <= r->k && h < 32; ++h)
            if (r->stats[(size_t)h - 1].active_rows > 0 &&
                (long long)r->stats[(size_t)h - 1].frontier_edges * kPredPushShare <= g->T)
                levels |= 1u << h;
        if (levels && ensure_out_eid(g, st) == LOGOSKG_OK) {
            a.push_levels = levels;
            a.host_graph = g;
            a.host_result = r;
        }
    }
    a.stats_pred = counting ? g->d_ctr + C_STATS + 4 * KK_PRED : nullptr;
    a.stats_hub = counting ? g->d_ctr + C_STATS + 4 * KK_PRED_HUB : nullptr;
    a.stats_mid = counting ? g->d_ctr + C_STATS + 4 * KK_PRED_MID : nullptr;
    if (counting) LKG_HIP(hipMemsetAsync(g->d_ctr + C_STATS, 0, 4 * KK_NUM * sizeof(unsigned long long), st));
    // The kernels of a fetch run in turn on the caller's stream.  The list kernel, the per-tile
    // predecessor kernel and the per-row predecessor kernels are independent, and with
    // LOGOSKG_OVERLAP_FETCH=1 a resident graph puts them on the helper streams and joins them on the
    // caller's; measured on every benchmark configuration that gains nothing (they are bound by
    // instruction issue and gather latency and share the same units) and costs small batches the
    // fork and join, so it is not the default.
    const char *overlap_env = getenv("LOGOSKG_OVERLAP_FETCH");
    const bool serial = !(overlap_env && overlap_env[0] == '1');
    // With predecessors on 16-word planes the tile kernel writes all three lists; otherwise the
    // list kernel runs beside the predecessor kernels.
    a.fuse_lists = pred && pred_uses_staged_kernel(a, W);
    const long long n_hub = g->in_rows.n_hub, n_mid = g->in_rows.n_long - g->in_rows.n_hub;
    // (nothing to fork for when the fused tile pass has no hub rows beside it)
    if (pred && g->num_shards <= 1 && !serial && (n_hub > 0 || !a.fuse_lists)) {
        LKG_HIP(hipEventRecord(g->ev_fork, st));
        for (int i = 0; i < 2; ++i) LKG_HIP(hipStreamWaitEvent(g->side[i], g->ev_fork, 0));
        if (a.fuse_lists) {
            launch_pred(g->prof, a, W, n_hub, n_mid, r->has_mask, st, g->side[0]);
        } else {
            launch_pred(g->prof, a, W, n_hub, n_mid, r->has_mask, g->side[0], g->side[1]);
            launch_lists(g->prof, a, W, st);
        }
        for (int i = 0; i < 2; ++i) {
            LKG_HIP(hipEventRecord(g->ev_join[i], g->side[i]));
            LKG_HIP(hipStreamWaitEvent(st, g->ev_join[i], 0));
        }
    } else {
        if (!a.fuse_lists) launch_lists(g->prof, a, W, st);
        if (pred) {
            if (g->num_shards > 1) LKG_TRY(sharded_pred(g, &a, W, r->has_mask, st));
            else launch_pred(g->prof, a, W, n_hub, n_mid, r->has_mask, st, st);
        }
    }
    LKG_HIP(hipGetLastError());
    if (g->prof.on) {
        if (!a.fuse_lists) g->prof.acc[KK_LISTS].units[3] += need;
        if (pred) g->prof.acc[KK_PRED].units[3] += need;
    }
    if (counting) {  // measurement mode only: wait for the counters
        LKG_HIP(hipMemcpyAsync(g->h_ctr, g->d_ctr, C_TOTAL * sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
        LKG_HIP(hipStreamSynchronize(st));
        for (int kind : {KK_PRED, KK_PRED_HUB, KK_PRED_MID})  // (the two-kernel tile pass counts in its first kernel)
            for (int u = 0; u < 3; ++u)
                g->prof.acc[kind == KK_PRED && a.fuse_lists ? KK_PRED_WALK : kind].units[u] +=
                    (long long)g->h_ctr[C_STATS + 4 * kind + u];
    }
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_result_level_offsets(logoskg_result *r, int32_t h, int64_t *level_off,
                                                       void *stream) {
    if (!r || !level_off) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    if (h < 0 || h > r->k) { set_error("level %d outside [0, %d]", h, r->k); return LOGOSKG_EINVAL; }
    LKG_HIP(hipSetDevice(r->g->device));
    r->level_counted = -1;
    LKG_TRY(count_plane(r, r->levels + (size_t)h * r->Epad * r->W, &r->lvl_tile_base, &r->lvl_super_base,
                        &r->lvl_mega_base, &r->d_level_off, &r->level_off, (hipStream_t)stream));
    r->level_counted = h;
    memcpy(level_off, r->level_off.data(), (size_t)(r->Q + 1) * sizeof(int64_t));
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_result_level_fetch(logoskg_result *r, int32_t h, int32_t q0, int32_t q1,
                                                     int64_t capacity, int32_t *entity, void *stream) {
    if (!r) { set_error("NULL result"); return LOGOSKG_EINVAL; }
    if (h < 0 || h > r->k || r->level_counted != h) {
        set_error("level %d was not counted: call logoskg_result_level_offsets for it first", h);
        return LOGOSKG_EINVAL;
    }
    if (q0 < 0 || q1 > r->Q || q0 > q1) { set_error("bad query range [%d, %d)", q0, q1); return LOGOSKG_EINVAL; }
    const int64_t need = r->level_off[(size_t)q1] - r->level_off[(size_t)q0];
    if (capacity < need) {
        set_error("capacity %lld < %lld entries", (long long)capacity, (long long)need);
        return LOGOSKG_ERANGE;
    }
    if (need == 0) return LOGOSKG_OK;
    if (!entity) { set_error("entity buffer is NULL"); return LOGOSKG_EINVAL; }
    logoskg_graph *g = r->g;
    LKG_HIP(hipSetDevice(g->device));
    r->last_stream = (hipStream_t)stream;
    const int W = r->W;
    FillArgs a = {};
    // the level plane plays the part of the visited plane; no hop numbers are asked for
    a.E = g->E; a.Q = r->Q; a.k = 0; a.q0 = q0; a.q1 = q1; a.hub_min = g->hub_min;
    a.tile_ent = r->tile_ent; a.cpos = r->cpos; a.n_listed = r->n_active;
    a.ntiles = r->tile_ent ? (r->n_active + 63) / 64 : r->Epad / kTileEntities;
    a.tile_begin = 0; a.tile_count = a.ntiles;
    a.plane = r->Epad * W; a.actw = r->Epad / 32;
    a.visited = r->levels + (size_t)h * r->Epad * W; a.levels = a.visited; a.allow = r->allow;
    a.act = r->act; a.tile_base = r->lvl_tile_base; a.super_base = r->lvl_super_base; a.mega_base = r->lvl_mega_base;
    a.reached_off = r->d_level_off;
    a.entity = entity;
    launch_lists(g->prof, a, W, (hipStream_t)stream);
    LKG_HIP(hipGetLastError());
    if (g->prof.on) g->prof.acc[KK_LISTS].units[3] += need;
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_result_traversed(logoskg_result *r, int64_t *traversed, void *stream) {
    if (!r || (r->k > 0 && !traversed)) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    if (r->k == 0) return LOGOSKG_OK;
    logoskg_graph *g = r->g;
    LKG_HIP(hipSetDevice(g->device));
    hipStream_t st = (hipStream_t)stream;
    r->last_stream = st;
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
