// logoskg_khop: batched k-hop expansion on one gfx950 GPU.
//
// State (paper Sec. 3.3): the query vectors q^(h) of up to 1024 queries are
// packed entity-major, W uint64 words per entity (bit j%64 of word j/64 =
// query j).  level[h] holds the bits that become set for the first time at hop
// h, visited = OR of all levels so far, act[h] has one bit per entity whose
// level[h] line is non-zero.
//
// One hop (Eq. 4, q.SUB.OBJ with the relation whitelist applied to the active
// triples of Eq. 5) is evaluated in one of two directions:
//   push: for every subject row in the frontier, OR its line into the lines of
//         its objects (atomicOr), skipping bits already visited;
//   pull: for every object row that still misses a query whose frontier is
//         alive, OR the lines of its subjects that are in the frontier, and
//         stop as soon as nothing is missing; no atomics on short rows, and
//         visited is updated in the same kernel.
// Both give the same level[h].  Rows of up to 32 entries are handled by a
// W-lane group each; longer rows are cut into fixed-size segments, one
// wavefront per segment, so a 100,000-entry hub spreads over many CUs.
//
// With LOGOSKG_WALK_EXACT the visited filter is dropped (Eq. 4 iterated as
// written): level[h] = image of level[h-1], an entity may be in several levels;
// visited still collects their union.
#include <algorithm>

#include "common.h"

namespace lkg {

// ---------------------------------------------------------------- seeds, mask table
__global__ void k_seed(int Q, long long num_seeds, const long long *__restrict__ seed_off,
                       const int32_t *__restrict__ seeds, int32_t E, int W,
                       unsigned long long *level0, unsigned long long *visited, uint32_t *act0,
                       unsigned long long *ctr) {
    int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= Q) return;
    long long a = seed_off[q], b = seed_off[q + 1];
    if (a < 0 || b < a || b > num_seeds || (q == 0 && a != 0) || (q == Q - 1 && b != num_seeds)) {
        atomicOr(&ctr[C_ERR], 1ull);
        return;
    }
    unsigned long long bit = 1ull << (q & 63);
    for (long long i = a; i < b; ++i) {
        int32_t e = seeds[i];
        if ((uint32_t)e >= (uint32_t)E) {
            atomicOr(&ctr[C_ERR], 2ull);
            continue;
        }
        size_t idx = (size_t)e * W + (q >> 6);
        atomicOr(&level0[idx], bit);
        atomicOr(&visited[idx], bit);
        atomicOr(&act0[e >> 5], 1u << (e & 31));
    }
}

// allow[r][w]: bit b set when query 64w+b may follow relation r (the vector REL.m
// of every query, transposed so that one triple's relation selects a whole line).
__global__ void k_allow(int Q, int R, int W, int rel_words, const unsigned long long *__restrict__ rel_mask,
                        unsigned long long *allow) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= R * W) return;
    int r = i / W, w = i % W;
    unsigned long long v = 0;
    for (int b = 0; b < 64; ++b) {
        int q = w * 64 + b;
        if (q < Q && ((rel_mask[(size_t)q * rel_words + (r >> 6)] >> (r & 63)) & 1ull)) v |= 1ull << b;
    }
    allow[i] = v;
}

// ---------------------------------------------------------------- frontier census
// Turns the active bitmap of a level into the work lists of a push hop (short
// subject rows; segments of the longer ones) and the counters the host needs
// to pick the direction.
//
// row_begin[e] is where the triples of subject e start in the edge arrays (equal
// to out_off for a resident graph; shard-grouped order for a sharded one).  With
// shard_of != NULL only the subjects of `shard` are listed (Algorithm 1, line 6:
// restriction of the frontier to one sub-graph).
__global__ void __launch_bounds__(256)
k_census(const uint32_t *__restrict__ act, int32_t E, const uint32_t *__restrict__ out_off,
         const uint32_t *__restrict__ row_begin, const uint8_t *__restrict__ shard_of, int shard, int write_lists,
         int32_t *list_tail, RowSegment *list_seg, unsigned long long *ctr) {
    // one thread per entity and step (coalesced offsets); mode 0 counts, mode 1 appends the
    // lists (C_NTAIL / C_NSEG are then the append cursors)
    __shared__ long long part[4][5];
    const long long stride = (long long)gridDim.x * blockDim.x;
    long long ct = 0, cs = 0, cr = 0, na = 0, deg_sum = 0;
    for (long long base = (long long)blockIdx.x * blockDim.x; base < E; base += stride) {  // block-uniform trip count
        const long long e = base + threadIdx.x;
        bool on = false;
        uint32_t d = 0;
        if (e < E) {
            on = (act[e >> 5] >> (e & 31)) & 1u;
            if (on && shard_of && shard_of[e] != (uint8_t)shard) on = false;
            if (on) d = out_off[e + 1] - out_off[e];
        }
        const bool tail = d > 0 && d <= (uint32_t)kTailMaxDegree;
        const int segs = d > (uint32_t)kTailMaxDegree ? (int)((d + kPushSegment - 1) / kPushSegment) : 0;
        if (!write_lists) {
            na += on;
            cr += d > 0;
            ct += tail;
            cs += segs;
            deg_sum += d;
            continue;
        }
        const unsigned long long tmask = __ballot(tail);
        int ts;
        const int ps = wave_excl_scan(segs, ts);
        unsigned long long bt = 0, bs = 0;
        if (lane() == 0) {
            if (tmask) bt = atomicAdd(&ctr[C_NTAIL], (unsigned long long)__popcll(tmask));
            if (ts) bs = atomicAdd(&ctr[C_NSEG], (unsigned long long)ts);
        }
        bt = shfl64(bt, 0);
        bs = shfl64(bs, 0);
        if (tail) list_tail[bt + __popcll(tmask & ((1ull << lane()) - 1ull))] = (int32_t)e;
        if (segs) {
            const uint32_t lo = row_begin[e];
            for (int i = 0; i < segs; ++i) list_seg[bs + ps + i] = RowSegment{(int32_t)e, lo + (uint32_t)i * kPushSegment};
        }
    }
    if (write_lists) return;
    ct = wave_sum(ct);
    cs = wave_sum(cs);
    cr = wave_sum(cr);
    na = wave_sum(na);
    deg_sum = wave_sum(deg_sum);
    const int wave = threadIdx.x >> 6;
    if (lane() == 0) {
        part[wave][0] = ct; part[wave][1] = cs; part[wave][2] = cr; part[wave][3] = deg_sum; part[wave][4] = na;
    }
    __syncthreads();
    if (threadIdx.x < 5) {
        long long x = part[0][threadIdx.x] + part[1][threadIdx.x] + part[2][threadIdx.x] + part[3][threadIdx.x];
        const int slot[5] = {C_NTAIL, C_NSEG, C_NROWS, C_FEDGES, C_NACTIVE};
        if (x) atomicAdd(&ctr[slot[threadIdx.x]], (unsigned long long)x);
    }
}

template <int W>
__device__ __forceinline__ unsigned long long or_across_groups(unsigned long long acc) {
#pragma unroll
    for (int m = W; m < 64; m <<= 1) acc |= shfl_xor64(acc, m);
    return acc;
}

// live[w] = OR of the frontier lines of every subject row that has a triple:
// the queries for which this hop can still reach something.  A pull row stops
// as soon as it has all of them.
template <int W>
__device__ __forceinline__ int take_candidates(unsigned long long &rest);

template <int W>
__global__ void __launch_bounds__(256)
k_live(const uint32_t *__restrict__ act, int32_t E, const uint32_t *__restrict__ out_off,
       const unsigned long long *__restrict__ prev, unsigned long long *live) {
    __shared__ unsigned long long sl[16];
    if (threadIdx.x < 16) sl[threadIdx.x] = 0;
    __syncthreads();
    // a wavefront tests 64 consecutive entities (coalesced), then its groups fetch the lines of
    // the frontier rows among them, two at a time
    const long long nwaves = (long long)gridDim.x * (blockDim.x >> 6);
    const int lw = threadIdx.x & (W - 1);
    unsigned long long acc = 0;
    for (long long base = ((long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * 64; base < E;
         base += nwaves * 64) {
        const long long e = base + lane();
        bool on = false;
        if (e < E) on = ((act[e >> 5] >> (e & 31)) & 1u) && out_off[e + 1] > out_off[e];
        unsigned long long m = __ballot(on);
        while (m) {
            const int p0 = take_candidates<W>(m), p1 = take_candidates<W>(m);
            unsigned long long l0 = 0, l1 = 0;
            if (p0 >= 0) l0 = prev[(size_t)(base + p0) * W + lw];
            if (p1 >= 0) l1 = prev[(size_t)(base + p1) * W + lw];
            acc |= l0 | l1;
        }
    }
    acc = or_across_groups<W>(acc);
    if (lane() < W && acc) atomicOr(&sl[lane()], acc);
    __syncthreads();
    if (threadIdx.x < W) {
        unsigned long long x = sl[threadIdx.x];
        if (x & ~live[threadIdx.x]) atomicOr(&live[threadIdx.x], x);
    }
}

// Every query counts as live: used instead of k_live where the frontier holds most of the
// graph's triples (then hardly any query has none, and a query wrongly taken as live only keeps
// a row from stopping early: its bit is in no frontier line).
__global__ void k_live_all(int Q, int W, unsigned long long *live) {
    if ((int)threadIdx.x < W) live[threadIdx.x] = query_bits(Q, (int)threadIdx.x);
}

// ---------------------------------------------------------------- push
__device__ __forceinline__ void mark_active(uint32_t *act, int e) {
    uint32_t bit = 1u << (e & 31);
    if (!(act[e >> 5] & bit)) atomicOr(&act[e >> 5], bit);
}

// `known` = the bits that need not be set again: the visited plane (minimum-hop search: an entity
// keeps its first level) or, for walk-exact levels, the level under construction itself.
// One W-lane group per short frontier row; its edges are walked one after another.
template <int W, bool MASK>
__global__ void __launch_bounds__(256)
k_push_tail(const int32_t *__restrict__ rows, const unsigned long long *__restrict__ ctr,
            const uint32_t *__restrict__ off, const uint32_t *__restrict__ row_begin,
            const int32_t *__restrict__ obj,
            const uint16_t *__restrict__ rel, const unsigned long long *__restrict__ allow,
            const unsigned long long *__restrict__ prev, const unsigned long long *known,
            unsigned long long *cur, uint32_t *act_cur) {
    long long gidx = ((long long)blockIdx.x * blockDim.x + threadIdx.x) / W;
    int lw = threadIdx.x & (W - 1);
    long long n = (long long)ctr[C_NTAIL];
    uint32_t lo = 0, hi = 0;
    unsigned long long line = 0;
    if (gidx < n) {
        int s = rows[gidx];
        lo = row_begin[s];
        hi = lo + (off[s + 1] - off[s]);
        line = prev[(size_t)s * W + lw];
    }
    for (uint32_t j = lo; j < hi; ++j) {
        int o = obj[j];
        unsigned long long m = line;
        if (MASK) m &= allow[(size_t)rel[j] * W + lw];
        if (m) m &= ~known[(size_t)o * W + lw];
        if (m) atomicOr(&cur[(size_t)o * W + lw], m);
        bool any = group_any<W>(m != 0);
        if (any && lw == 0) mark_active(act_cur, o);
    }
}

// 64 consecutive edges of one subject row, handled by a whole wavefront: every
// lane loads one edge, then the 64/W groups take the edges in turn.
template <int W, bool MASK>
__device__ __forceinline__ void push_chunk(uint32_t j0, uint32_t hi, unsigned long long line,
                                           const int32_t *__restrict__ obj, const uint16_t *__restrict__ rel,
                                           const unsigned long long *__restrict__ allow,
                                           const unsigned long long *known,
                                           unsigned long long *cur, uint32_t *act_cur) {
    constexpr int GPW = 64 / W;
    int lw = lane() & (W - 1), g = lane() / W;
    uint32_t j = j0 + lane();
    int o = -1, r = 0;
    if (j < hi) {
        o = obj[j];
        if (MASK) r = rel[j];
    }
    int n = (int)min((uint32_t)64, hi - j0);
    if constexpr (W == 1) {
        if (o >= 0) {
            unsigned long long m = line;
            if (MASK) m &= allow[r];
            if (m) m &= ~known[o];
            if (m) {
                atomicOr(&cur[o], m);
                mark_active(act_cur, o);
            }
        }
    } else {
        for (int i = 0; i < n; i += GPW) {
            int idx = i + g;
            int oc = __shfl(o, idx & 63);
            int rc = MASK ? __shfl(r, idx & 63) : 0;
            if (idx < n) {
                unsigned long long m = line;
                if (MASK) m &= allow[(size_t)rc * W + lw];
                if (m) m &= ~known[(size_t)oc * W + lw];
                if (m) atomicOr(&cur[(size_t)oc * W + lw], m);
                bool any = group_any<W>(m != 0);
                if (any && lw == 0) mark_active(act_cur, oc);
            }
        }
    }
}

// One wavefront per segment of a long frontier row.
template <int W, bool MASK>
__global__ void __launch_bounds__(256)
k_push_seg(const RowSegment *__restrict__ segs, const unsigned long long *__restrict__ ctr,
           const uint32_t *__restrict__ off, const uint32_t *__restrict__ row_begin,
           const int32_t *__restrict__ obj,
           const uint16_t *__restrict__ rel, const unsigned long long *__restrict__ allow,
           const unsigned long long *__restrict__ prev, const unsigned long long *known,
           unsigned long long *cur, uint32_t *act_cur) {
    long long item = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (item >= (long long)ctr[C_NSEG]) return;
    RowSegment sg = segs[item];
    int lw = lane() & (W - 1);
    unsigned long long line = prev[(size_t)sg.row * W + lw];
    uint32_t row_end = row_begin[sg.row] + (off[sg.row + 1] - off[sg.row]);
    uint32_t hi = min(sg.begin + (uint32_t)kPushSegment, row_end);
    for (uint32_t j0 = sg.begin; j0 < hi; j0 += 64)
        push_chunk<W, MASK>(j0, hi, line, obj, rel, allow, known, cur, act_cur);
}

// visited |= level[h] on the lines the push kernels touched.
// One wavefront per 64 entities: it reads their two words of the active bitmap once and touches
// only the lines of the active ones (after a push from a small frontier almost none), W lanes per
// line, so a dense level is still updated with contiguous accesses.
template <int W>
__global__ void __launch_bounds__(256)
k_update_visited(long long Epad, const uint32_t *__restrict__ act_cur, const unsigned long long *__restrict__ cur,
                 unsigned long long *visited) {
    const long long base = ((long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * 64;
    if (base >= Epad) return;  // Epad is a multiple of 64
    const unsigned long long m =
        ((unsigned long long)act_cur[base / 32 + 1] << 32) | (unsigned long long)act_cur[base / 32];
    if (m == 0) return;
    constexpr int GPW = 64 / W;
    const int g = lane() / W, lw = lane() & (W - 1);
#pragma unroll
    for (int i = 0; i < W; ++i) {
        const int e = i * GPW + g;
        if ((m >> e) & 1ull) {
            const size_t x = ((size_t)base + e) * W + lw;
            visited[x] |= cur[x];
        }
    }
}

// ---------------------------------------------------------------- pull
// From this share of the triples leaving the frontier the pull kernels gather every edge's line
// without asking for its frontier bit first.  A bit test is a scattered 4-byte load, i.e. a 64-byte
// sector through the L1 per edge, and these kernels are bound by what the L2s deliver; skipping the
// test costs the lines of the edges outside the frontier (zero lines: a level line is non-zero only
// where its active bit is set), which is less traffic as soon as half the edges are inside.
// Removes up to 64/W candidates from the (wave-uniform) mask and returns the
// lane position of the one that belongs to the caller's group, or -1.
template <int W>
__device__ __forceinline__ int take_candidates(unsigned long long &rest) {
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

// 64 consecutive in-edges of one object row, in three stages so that a caller can
// keep the loads of later chunks in flight: subject (and relation) ids, the
// frontier bit of every subject, then the gather of the frontier lines of the
// candidates (pull_gather).
struct PullEdges {
    int s, r;
};

template <bool MASK>
__device__ __forceinline__ PullEdges pull_load_edges(uint32_t j0, uint32_t hi, const int32_t *__restrict__ in_sub,
                                                     const uint16_t *__restrict__ in_rel) {
    PullEdges e{-1, 0};
    uint32_t j = j0 + lane();
    if (j < hi) {
        e.s = in_sub[j];
        if (MASK) e.r = in_rel[j];
    }
    return e;
}

__device__ __forceinline__ bool pull_test(const PullEdges &e, const uint32_t *__restrict__ act_prev) {
    return e.s >= 0 && ((act_prev[e.s >> 5] >> (e.s & 31)) & 1u);
}

// Gather stage.  The candidates' subject ids are compacted into a per-wavefront
// LDS queue (position = number of candidates in lower lanes); group g of round r
// then reads entry r * (groups per round) + g, so picking a candidate costs one
// LDS read instead of a search in the ballot mask and a cross-lane move.  A lane
// loads two plane words (16 bytes): W/2 lanes cover a line and one load
// instruction of a wavefront fetches 128/W lines, which halves the number of
// vector memory instructions against one word per lane.  Up to four rounds of
// loads are in flight; only the last, partly filled batch is predicated.
// a0 / a1 collect words 2*(lane % (W/2)) and 2*(lane % (W/2)) + 1 (W = 1: a0 only).
template <int W, bool MASK>
__device__ __forceinline__ int pull_gather(const PullEdges &e, bool cand, const unsigned long long *__restrict__ prev,
                                           const unsigned long long *__restrict__ allow, unsigned long long &a0,
                                           unsigned long long &a1, int *queue_s, uint16_t *queue_r) {
    const unsigned long long cm = __ballot(cand);
    const int ncand = __popcll(cm);
    if constexpr (W == 1) {
        if (cand) {
            unsigned long long ln = prev[e.s];
            if (MASK) ln &= allow[e.r];
            a0 |= ln;
        }
    } else {
        constexpr int LW = W / 2, GPW = 64 / LW;            // lanes per line, lines per load instruction
        constexpr int NR = GPW >= 32 ? 64 / GPW : 4, B = NR * GPW;  // rounds and candidates per batch
        const ulonglong2 *prev2 = reinterpret_cast<const ulonglong2 *>(prev);
        const ulonglong2 *allow2 = reinterpret_cast<const ulonglong2 *>(allow);
        if (ncand == 0) return 0;
        if (cand) {
            const int pos = __popcll(cm & ((1ull << lane()) - 1ull));
            queue_s[pos] = e.s;
            if (MASK) queue_r[pos] = (uint16_t)e.r;
        }
        __builtin_amdgcn_wave_barrier();
        const int lw = lane() & (LW - 1), g = lane() / LW;
        int base = 0;
        for (; base + B <= ncand; base += B) {  // full batches
            ulonglong2 l[NR];
#pragma unroll
            for (int x = 0; x < NR; ++x) {
                const int i = base + x * GPW + g;
                l[x] = prev2[(size_t)queue_s[i] * LW + lw];
                if (MASK) {
                    const ulonglong2 m = allow2[(size_t)queue_r[i] * LW + lw];
                    l[x].x &= m.x;
                    l[x].y &= m.y;
                }
            }
#pragma unroll
            for (int x = 0; x < NR; ++x) {
                a0 |= l[x].x;
                a1 |= l[x].y;
            }
        }
        if (base < ncand) {
            ulonglong2 l[NR];
#pragma unroll
            for (int x = 0; x < NR; ++x) {
                const int i = base + x * GPW + g;
                l[x] = make_ulonglong2(0, 0);
                if (i < ncand) {
                    l[x] = prev2[(size_t)queue_s[i] * LW + lw];
                    if (MASK) {
                        const ulonglong2 m = allow2[(size_t)queue_r[i] * LW + lw];
                        l[x].x &= m.x;
                        l[x].y &= m.y;
                    }
                }
            }
#pragma unroll
            for (int x = 0; x < NR; ++x) {
                a0 |= l[x].x;
                a1 |= l[x].y;
            }
        }
        __builtin_amdgcn_wave_barrier();  // the queue is rewritten by the next chunk
    }
    return ncand;
}

// Folds the accumulators of pull_gather into one word per lane (word lane % W),
// the union over the whole wavefront.
template <int W>
__device__ __forceinline__ unsigned long long fold_gathered(unsigned long long a0, unsigned long long a1) {
    if constexpr (W == 1) {
        return or_across_groups<1>(a0);
    } else {
        a0 = or_across_groups<W / 2>(a0);
        a1 = or_across_groups<W / 2>(a1);
        const int lw = lane() & (W - 1);
        const unsigned long long x = shfl64(a0, lw >> 1), y = shfl64(a1, lw >> 1);
        return (lw & 1) ? y : x;
    }
}

__device__ __forceinline__ void add_stats(unsigned long long *stats, long long rows, long long edges,
                                          long long lines) {
    // called by every lane of a wavefront with per-lane partial counts
    rows = wave_sum(rows);
    edges = wave_sum(edges);
    lines = wave_sum(lines);
    if (lane() == 0) {
        if (rows) atomicAdd(&stats[0], (unsigned long long)rows);
        if (edges) atomicAdd(&stats[1], (unsigned long long)edges);
        if (lines) atomicAdd(&stats[2], (unsigned long long)lines);
    }
}

template <int W>
__device__ __forceinline__ unsigned group_ballot(bool p) {
    if constexpr (W == 1) return p ? 1u : 0u;
    else {
        unsigned long long b = __ballot(p);
        return (unsigned)((b >> (lane() & ~(W - 1))) & ((1ull << W) - 1ull));
    }
}

// Short object rows (<= 32 entries): a W-lane group works on kTailRows rows at
// once.  A row is a chain of dependent loads (row record -> visited line and
// subject ids -> frontier bits -> frontier lines), and with all wavefront
// slots of a CU taken the kernel is bound by that latency, so the work list carries
// the row bounds (no look-up in the offsets) and every group keeps
// the chains of two rows in flight: each stage is issued for both rows before
// either result is used.  Per stage the group's lanes load W entries of a row,
// then gather the frontier lines of its candidates, two per row at a time.
// (three or four rows per group measured the same: the kernel then runs at the
// rate at which the memory system serves its scattered lines.)
constexpr int kTailRows = 2;
constexpr int kTailLines = 2;  // candidate lines of each row requested together

template <int W, bool MASK, bool STATS, bool DENSE>
__global__ void __launch_bounds__(256)
k_pull_tail(const ShortRow *__restrict__ rows, long long n, const int32_t *__restrict__ in_sub, const uint16_t *__restrict__ in_rel,
            const unsigned long long *__restrict__ allow, const uint32_t *__restrict__ act_prev,
            const unsigned long long *__restrict__ prev, const unsigned long long *__restrict__ live,
            unsigned long long *visited, unsigned long long *cur, uint32_t *act_cur,
            unsigned long long *stats, int walk_exact) {
    constexpr int NR = kTailRows;
    const long long group = ((long long)blockIdx.x * blockDim.x + threadIdx.x) / W;
    const int lw = threadIdx.x & (W - 1), g0 = lane() & ~(W - 1);
    uint32_t lo[NR], hi[NR], j0[NR];
    int v[NR];
    bool have[NR];
    unsigned long long vis[NR], need[NR], acc[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) {  // the row's id and bounds come in one record
        have[r] = group * NR + r < n;
        v[r] = 0;
        lo[r] = hi[r] = 0;
        if (have[r]) {
            const ShortRow row = rows[group * NR + r];
            v[r] = row.row;
            lo[r] = row.begin;
            hi[r] = row.end;
        }
    }
    int s_next[NR], rel_next[NR];  // subject (and relation) ids of the next W entries, loaded one stage ahead
#pragma unroll
    for (int r = 0; r < NR; ++r) {  // the visited line and the first entries are requested together
        vis[r] = need[r] = acc[r] = 0;
        s_next[r] = -1;
        rel_next[r] = 0;
        if (have[r]) {
            vis[r] = visited[(size_t)v[r] * W + lw];
            if (lo[r] + lw < hi[r]) {
                s_next[r] = in_sub[lo[r] + lw];
                if (MASK) rel_next[r] = in_rel[lo[r] + lw];
            }
        }
    }
    const unsigned long long live_w = live[lw];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        need[r] = (walk_exact ? ~0ull : ~vis[r]) & live_w;
        if (!have[r]) need[r] = 0;
        if (!group_any<W>(need[r] != 0)) hi[r] = lo[r];
        j0[r] = lo[r];
    }
    uint32_t row_end[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) row_end[r] = hi[r];
    long long n_edges = 0, n_lines = 0;
    auto any_open = [&]() {
        bool o = false;
#pragma unroll
        for (int r = 0; r < NR; ++r) o |= j0[r] < hi[r];
        return o;
    };
    while (any_open()) {
        int s[NR], rl[NR];
        bool cand[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const bool open = j0[r] < hi[r];
            s[r] = open ? s_next[r] : -1;
            rl[r] = rel_next[r];
            s_next[r] = -1;
            const uint32_t j = j0[r] + W + lw;
            if (open && j < hi[r]) {
                s_next[r] = in_sub[j];
                if (MASK) rel_next[r] = in_rel[j];
            }
        }
#pragma unroll
        for (int r = 0; r < NR; ++r)
            cand[r] = s[r] >= 0 && (DENSE || ((act_prev[s[r] >> 5] >> (s[r] & 31)) & 1u));
        unsigned gm[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            gm[r] = group_ballot<W>(cand[r]);
            if (j0[r] < hi[r]) n_edges += min((uint32_t)W, hi[r] - j0[r]);
            n_lines += __popc(gm[r]);
        }
        auto any_candidate = [&]() {
            unsigned o = 0;
#pragma unroll
            for (int r = 0; r < NR; ++r) o |= gm[r];
            return o != 0;
        };
        constexpr int NL = kTailLines;
        while (any_candidate()) {  // two candidate lines of each row in flight
            int c[NR][NL];
            unsigned long long l[NR][NL];
#pragma unroll
            for (int r = 0; r < NR; ++r)
#pragma unroll
                for (int x = 0; x < NL; ++x) {
                    c[r][x] = -1;
                    if (gm[r]) {
                        c[r][x] = __ffs((int)gm[r]) - 1;
                        gm[r] &= gm[r] - 1;
                    }
                }
#pragma unroll
            for (int r = 0; r < NR; ++r)
#pragma unroll
                for (int x = 0; x < NL; ++x) {
                    const int src = g0 + (c[r][x] < 0 ? 0 : c[r][x]);
                    const int sx = __shfl(s[r], src);
                    l[r][x] = 0;
                    if (c[r][x] >= 0) l[r][x] = prev[(size_t)sx * W + lw];
                    if (MASK) {
                        const int rx = __shfl(rl[r], src);
                        if (c[r][x] >= 0) l[r][x] &= allow[(size_t)rx * W + lw];
                    }
                }
#pragma unroll
            for (int r = 0; r < NR; ++r)
#pragma unroll
                for (int x = 0; x < NL; ++x) acc[r] |= l[r][x];
        }
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            if (j0[r] < hi[r]) {
                j0[r] += W;
                if (!group_any<W>((need[r] & ~acc[r]) != 0)) hi[r] = j0[r];  // nothing left to find in this row
            }
        }
    }
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const unsigned long long nw = acc[r] & need[r];
        if (row_end[r] > lo[r] && group_any<W>(nw != 0)) {
            cur[(size_t)v[r] * W + lw] = nw;
            visited[(size_t)v[r] * W + lw] = vis[r] | nw;
            if (lw == 0) atomicOr(&act_cur[v[r] >> 5], 1u << (v[r] & 31));
        }
    }
    if (STATS) {
        const bool lead = (lw == 0);
        long long n_rows = 0;
#pragma unroll
        for (int r = 0; r < NR; ++r) n_rows += (row_end[r] > lo[r]) ? 1 : 0;
        add_stats(stats, lead ? n_rows : 0, lead ? n_edges : 0, lead ? n_lines : 0);
    }
}

// One wavefront per segment (<= 1024 entries) of a longer object row.  A row
// with one segment is finished here; segments of a multi-segment row merge
// through atomicOr on level[h] and look at what the others have found so far
// to stop early; k_pull_finish then folds those rows into visited.
template <int W, bool MASK, bool STATS, bool DENSE>
__global__ void __launch_bounds__(256)
k_pull_seg(const PullSegment *__restrict__ segs, long long n,
           const int32_t *__restrict__ in_sub, const uint16_t *__restrict__ in_rel,
           const unsigned long long *__restrict__ allow, const uint32_t *__restrict__ act_prev,
           const unsigned long long *__restrict__ prev, const unsigned long long *__restrict__ live,
           unsigned long long *visited, unsigned long long *cur, uint32_t *act_cur,
           unsigned long long *stats, int walk_exact) {
    __shared__ int queue_s[4][64];
    __shared__ uint16_t queue_r[4][64];
    long long item = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const bool have = item < n;  // wave-uniform
    const int lw = lane() & (W - 1);
    int v = 0;
    uint32_t lo = 0, hi = 0;
    bool multi = false;
    unsigned long long vis = 0, need = 0, acc = 0;
    if (have) {
        const PullSegment sg = segs[item];  // carries its bounds: no look-up in the offsets before the first loads
        v = sg.row;
        lo = sg.begin;
        hi = sg.end;
        multi = sg.multi != 0;
        vis = visited[(size_t)v * W + lw];
        need = (walk_exact ? ~0ull : ~vis) & live[lw];
        if (multi) need &= ~__atomic_load_n(&cur[(size_t)v * W + lw], __ATOMIC_RELAXED);
    }
    const bool work = wave_any(need != 0);
    long long n_edges = 0, n_lines = 0;
    unsigned long long a0 = 0, a1 = 0;
    if (work) {
        // software pipeline: ids of chunk i+2 and frontier bits of chunk i+1 are requested
        // before the lines of chunk i are gathered
        PullEdges e0 = pull_load_edges<MASK>(lo, hi, in_sub, in_rel);
        PullEdges e1 = pull_load_edges<MASK>(lo + 64, hi, in_sub, in_rel);
        // DENSE: nearly every subject is in the frontier, so the one-bit test (a 64-byte sector per
        // edge) is skipped and every edge's line is gathered: the line of an entity outside the frontier is zero
        bool c0 = DENSE ? e0.s >= 0 : pull_test(e0, act_prev);
        int it = 0;
        for (uint32_t j0 = lo; j0 < hi; j0 += 64, ++it) {
            PullEdges e2 = pull_load_edges<MASK>(j0 + 128, hi, in_sub, in_rel);
            const bool c1 = DENSE ? e1.s >= 0 : pull_test(e1, act_prev);
            n_lines += pull_gather<W, MASK>(e0, c0, prev, allow, a0, a1, queue_s[threadIdx.x >> 6], queue_r[threadIdx.x >> 6]);
            n_edges += min((uint32_t)64, hi - j0);
            e0 = e1;
            c0 = c1;
            e1 = e2;
            if ((it & 3) == 3) {  // early exit is rare: test it every fourth chunk
                acc = fold_gathered<W>(a0, a1);
                if (multi) acc |= __atomic_load_n(&cur[(size_t)v * W + lw], __ATOMIC_RELAXED);
                if (!wave_any((need & ~acc) != 0)) break;
            }
        }
        acc |= fold_gathered<W>(a0, a1);
        unsigned long long nb = acc & need;
        if (wave_any(nb != 0)) {
            if (!multi) {
                if (lane() < W) {
                    cur[(size_t)v * W + lane()] = nb;
                    visited[(size_t)v * W + lane()] = vis | nb;
                }
                if (lane() == 0) atomicOr(&act_cur[v >> 5], 1u << (v & 31));
            } else if (lane() < W && nb) {
                atomicOr(&cur[(size_t)v * W + lane()], nb);
            }
        }
    }
    if (STATS) {
        bool lead = lane() == 0;
        add_stats(stats, (lead && work) ? 1 : 0, lead ? n_edges : 0, lead ? n_lines : 0);
    }
}

// Rows that were expanded by several segments: visited |= level[h], mark active.
template <int W>
__global__ void __launch_bounds__(256)
k_pull_finish(const int32_t *__restrict__ rows, long long n, unsigned long long *visited,
              const unsigned long long *__restrict__ cur, uint32_t *act_cur) {
    long long gidx = ((long long)blockIdx.x * blockDim.x + threadIdx.x) / W;
    const int lw = threadIdx.x & (W - 1);
    unsigned long long c = 0;
    int v = 0;
    if (gidx < n) {
        v = rows[gidx];
        c = cur[(size_t)v * W + lw];
    }
    if (group_any<W>(c != 0)) {
        visited[(size_t)v * W + lw] |= c;
        if (lw == 0) atomicOr(&act_cur[v >> 5], 1u << (v & 31));
    }
}

// ---------------------------------------------------------------- planes back to zero
// A finished result's planes are zero except in the lines of entities that have their bit in some
// level's active bitmap: when the result is released those lines (of the level and of visited) and
// the bitmaps are cleared, so that the next call that gets the block starts from zeros without a
// fill of all k + 2 planes.  One wavefront per 64 entities, W lanes per line.
template <int W>
__global__ void __launch_bounds__(256)
k_sparse_clear(long long Epad, int levels, uint32_t *act, long long actw, unsigned long long *visited,
               unsigned long long *level_planes, long long plane, unsigned long long *live) {
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < levels * 16; i += blockDim.x) live[i] = 0ull;
    const long long base = ((long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * 64;
    if (base >= Epad) return;  // Epad is a multiple of 64
    constexpr int GPW = 64 / W;
    const int g = lane() / W, lw = lane() & (W - 1);
    unsigned long long any = 0;
    for (int h = 0; h <= levels; ++h) {  // the levels, then visited with the union of their bits
        unsigned long long m = any;
        unsigned long long *dst = visited;
        if (h < levels) {
            uint32_t *a = act + (size_t)h * actw + base / 32;
            m = ((unsigned long long)a[1] << 32) | (unsigned long long)a[0];
            any |= m;
            dst = level_planes + (size_t)h * plane;
            if (m && lane() < 2) a[lane()] = 0u;
        }
        if (m == 0) continue;
#pragma unroll
        for (int i = 0; i < W; ++i) {
            const int e = i * GPW + g;
            if ((m >> e) & 1ull) dst[((size_t)base + e) * W + lw] = 0ull;
        }
    }
}

// ---------------------------------------------------------------- host side
static inline unsigned blocks_for(long long threads, int block) {
    return (unsigned)((threads + block - 1) / block);
}

template <int W, bool MASK>
static void launch_push(logoskg_graph *g, logoskg_result *r, int h, const unsigned long long *hc,
                        const int32_t *obj, const uint16_t *rel, bool update, const int32_t *list_tail,
                        const RowSegment *list_seg, const unsigned long long *ctr, hipStream_t st) {
    const size_t plane = (size_t)r->Epad * W;
    const unsigned long long *prev = r->levels + plane * (h - 1);
    unsigned long long *cur = r->levels + plane * h;
    uint32_t *act_cur = r->act + (size_t)(r->Epad / 32) * h;
    long long nt = (long long)hc[C_NTAIL], ns = (long long)hc[C_NSEG];
    const unsigned long long *known = r->walk_exact ? cur : r->visited;
    if (ns > 0) {
        ProfScope ps(g->prof, KK_PUSH_SEG, st);
        k_push_seg<W, MASK><<<dim3(blocks_for(ns, 4)), dim3(256), 0, st>>>(
            list_seg, ctr, g->out_off, g->row_begin, obj, rel, r->allow, prev, known, cur, act_cur);
        g->prof.acc[KK_PUSH_SEG].units[0] += g->prof.on ? ns : 0;
    }
    if (nt > 0) {
        ProfScope ps(g->prof, KK_PUSH_TAIL, st);
        k_push_tail<W, MASK><<<dim3(blocks_for(nt * W, 256)), dim3(256), 0, st>>>(
            list_tail, ctr, g->out_off, g->row_begin, obj, rel, r->allow, prev, known, cur, act_cur);
        g->prof.acc[KK_PUSH_TAIL].units[0] += g->prof.on ? nt : 0;
    }
    if (!update) return;
    ProfScope ps(g->prof, KK_UPDATE, st);
    k_update_visited<W><<<dim3(blocks_for(r->Epad / 64, 4)), dim3(256), 0, st>>>(r->Epad, act_cur, cur, r->visited);
}

// STATS: the counting mode runs instantiations of its own, so that kernel statistics of the
// ordinary ones are not mixed with it.
// When most triples leave the frontier the kernels gather every edge's line without asking for
// its frontier bit first (never in the counting mode: its statistics count frontier lines).
static inline bool dense_pull(const logoskg_graph *g, const unsigned long long *hc, bool want_stats) {
    return !want_stats && (long long)hc[C_FEDGES] * 100 >= g->T * (long long)kDensePullPercent;
}

// live[h-1]: the queries this hop can still reach something for (once per hop).
template <int W>
static void launch_live(logoskg_graph *g, logoskg_result *r, int h, bool dense, hipStream_t st) {
    const size_t plane = (size_t)r->Epad * W;
    ProfScope ps(g->prof, KK_LIVE, st);
    unsigned nb = std::min<unsigned>(2048u, std::max(1u, blocks_for(g->E, 256)));
    unsigned long long *live = r->live + (size_t)16 * (h - 1);
    if (dense) k_live_all<<<dim3(1), dim3(64), 0, st>>>(r->Q, W, live);
    else k_live<W><<<dim3(nb), dim3(256), 0, st>>>(r->act + (size_t)(r->Epad / 32) * (h - 1), g->E, g->out_off,
                                                   r->levels + plane * (h - 1), live);
}

// Pull over the object rows of the work lists `rc`, whose entries index in_sub / in_rel (the whole
// object-sorted CSR of a resident graph, or one object range of a sharded one in a cache slot).
template <int W, bool MASK, bool STATS>
static void launch_pull_rows(logoskg_graph *g, logoskg_result *r, int h, const RowClasses &rc, const int32_t *in_sub,
                             const uint16_t *in_rel, bool dense, hipStream_t st) {
    const size_t plane = (size_t)r->Epad * W;
    const unsigned long long *prev = r->levels + plane * (h - 1);
    unsigned long long *cur = r->levels + plane * h;
    const uint32_t *act_prev = r->act + (size_t)(r->Epad / 32) * (h - 1);
    uint32_t *act_cur = r->act + (size_t)(r->Epad / 32) * h;
    const unsigned long long *live = r->live + (size_t)16 * (h - 1);
    auto stats = [&](int kind) { return STATS ? g->d_ctr + C_STATS + 4 * kind : nullptr; };
    const int walk = r->walk_exact ? 1 : 0;
    if (rc.n_seg > 0) {
        ProfScope ps(g->prof, KK_PULL_SEG, st);
        const dim3 grid(blocks_for(rc.n_seg, 4)), block(256);
        if (dense)
            k_pull_seg<W, MASK, STATS, true><<<grid, block, 0, st>>>(rc.seg, rc.n_seg, in_sub, in_rel,
                                                                     r->allow, act_prev, prev, live, r->visited, cur,
                                                                     act_cur, stats(KK_PULL_SEG), walk);
        else
            k_pull_seg<W, MASK, STATS, false><<<grid, block, 0, st>>>(rc.seg, rc.n_seg, in_sub, in_rel,
                                                                      r->allow, act_prev, prev, live, r->visited, cur,
                                                                      act_cur, stats(KK_PULL_SEG), walk);
    }
    if (rc.n_tail > 0) {
        ProfScope ps(g->prof, KK_PULL_TAIL, st);
        const long long groups = (rc.n_tail + kTailRows - 1) / kTailRows;
        const dim3 grid(blocks_for(groups * W, 256)), block(256);
        if (dense)
            k_pull_tail<W, MASK, STATS, true><<<grid, block, 0, st>>>(rc.tail, rc.n_tail, in_sub, in_rel, r->allow,
                                                                      act_prev, prev, live, r->visited, cur, act_cur,
                                                                      stats(KK_PULL_TAIL), walk);
        else
            k_pull_tail<W, MASK, STATS, false><<<grid, block, 0, st>>>(rc.tail, rc.n_tail, in_sub, in_rel, r->allow,
                                                                       act_prev, prev, live, r->visited, cur, act_cur,
                                                                       stats(KK_PULL_TAIL), walk);
    }
    if (rc.n_multi > 0) {
        ProfScope ps(g->prof, KK_PULL_FINISH, st);
        k_pull_finish<W><<<dim3(blocks_for(rc.n_multi * W, 256)), dim3(256), 0, st>>>(rc.multi, rc.n_multi,
                                                                                      r->visited, cur, act_cur);
    }
}

template <int W>
static void pull_rows_w(logoskg_graph *g, logoskg_result *r, int h, const RowClasses &rc, const int32_t *in_sub,
                        const uint16_t *in_rel, bool dense, bool want_stats, hipStream_t st) {
    if (r->has_mask) {
        if (want_stats) launch_pull_rows<W, true, true>(g, r, h, rc, in_sub, in_rel, dense, st);
        else launch_pull_rows<W, true, false>(g, r, h, rc, in_sub, in_rel, dense, st);
    } else {
        if (want_stats) launch_pull_rows<W, false, true>(g, r, h, rc, in_sub, in_rel, dense, st);
        else launch_pull_rows<W, false, false>(g, r, h, rc, in_sub, in_rel, dense, st);
    }
}

// One object range of a pull hop (a sharded graph visits them one after the other; `first`: the
// live words of the hop are computed before the range).
void launch_pull_range(logoskg_graph *g, logoskg_result *r, int h, const RowClasses &rc, const int32_t *in_sub,
                       const uint16_t *in_rel, const unsigned long long *hc, bool want_stats, bool first,
                       hipStream_t st) {
    const bool dense = dense_pull(g, hc, want_stats);
    switch (r->W) {
        case 1:
            if (first) launch_live<1>(g, r, h, dense, st);
            pull_rows_w<1>(g, r, h, rc, in_sub, in_rel, dense, want_stats, st);
            break;
        case 4:
            if (first) launch_live<4>(g, r, h, dense, st);
            pull_rows_w<4>(g, r, h, rc, in_sub, in_rel, dense, want_stats, st);
            break;
        default:
            if (first) launch_live<16>(g, r, h, dense, st);
            pull_rows_w<16>(g, r, h, rc, in_sub, in_rel, dense, want_stats, st);
            break;
    }
}

template <int W>
static void run_hop(logoskg_graph *g, logoskg_result *r, int h, bool pull, bool want_stats,
                    const unsigned long long *hc, hipStream_t st) {
    if (pull) {
        launch_pull_range(g, r, h, g->in_rows, g->in_sub, g->in_rel, hc, want_stats, true, st);
    } else {
        if (r->has_mask) launch_push<W, true>(g, r, h, hc, g->out_obj, g->out_rel, true, g->fr_tail, g->fr_seg, g->d_ctr, st);
        else launch_push<W, false>(g, r, h, hc, g->out_obj, g->out_rel, true, g->fr_tail, g->fr_seg, g->d_ctr, st);
    }
}

// Push of prepared work lists (short rows, segments; ctr[0], ctr[1] = their lengths on the
// device), reading the edge arrays through the given base pointers (a shard slot, shifted so
// that grouped edge indices apply).
void launch_push_lists(logoskg_graph *g, logoskg_result *r, int h, const unsigned long long *hc,
                       const int32_t *obj, const uint16_t *rel, bool update, const int32_t *list_tail,
                       const RowSegment *list_seg, const unsigned long long *ctr, hipStream_t st) {
    switch (r->W) {
        case 1:
            if (r->has_mask) launch_push<1, true>(g, r, h, hc, obj, rel, update, list_tail, list_seg, ctr, st);
            else launch_push<1, false>(g, r, h, hc, obj, rel, update, list_tail, list_seg, ctr, st);
            break;
        case 4:
            if (r->has_mask) launch_push<4, true>(g, r, h, hc, obj, rel, update, list_tail, list_seg, ctr, st);
            else launch_push<4, false>(g, r, h, hc, obj, rel, update, list_tail, list_seg, ctr, st);
            break;
        default:
            if (r->has_mask) launch_push<16, true>(g, r, h, hc, obj, rel, update, list_tail, list_seg, ctr, st);
            else launch_push<16, false>(g, r, h, hc, obj, rel, update, list_tail, list_seg, ctr, st);
            break;
    }
}

void launch_resident_hop(logoskg_graph *g, logoskg_result *r, int h, bool pull, bool want_stats,
                         const unsigned long long *hc, hipStream_t st) {
    switch (r->W) {
        case 1: run_hop<1>(g, r, h, pull, want_stats, hc, st); break;
        case 4: run_hop<4>(g, r, h, pull, want_stats, hc, st); break;
        default: run_hop<16>(g, r, h, pull, want_stats, hc, st); break;
    }
}

// Census of level h's active bitmap (all subjects, or those of one shard): counts the rows,
// edges and list entries into g->h_ctr (stream synchronised); with write_lists a second pass
// appends the push work lists.
static void launch_census(logoskg_graph *g, logoskg_result *r, int h, int shard, bool lists, hipStream_t st,
                          int prof_kind = KK_CENSUS) {
    const long long nwords = r->Epad / 32;
    ProfScope ps(g->prof, prof_kind, st);
    const unsigned nb = std::min<unsigned>(1024u, std::max(1u, blocks_for(g->E, 256)));
    k_census<<<dim3(nb), dim3(256), 0, st>>>(r->act + (size_t)nwords * h, g->E, g->out_off, g->row_begin,
                                             shard >= 0 ? g->shard_of_dev : nullptr, shard, lists ? 1 : 0,
                                             g->fr_tail, g->fr_seg, g->d_ctr);
}

logoskg_status census_lists(logoskg_graph *g, logoskg_result *r, int h, int shard, hipStream_t st, int prof_kind) {
    LKG_HIP(hipMemsetAsync(g->d_ctr, 0, 2 * sizeof(unsigned long long), st));  // C_NTAIL, C_NSEG: append cursors
    launch_census(g, r, h, shard, true, st, prof_kind);
    LKG_HIP(hipGetLastError());
    return LOGOSKG_OK;
}

logoskg_status census(logoskg_graph *g, logoskg_result *r, int h, int shard, bool write_lists, hipStream_t st) {
    LKG_HIP(hipMemsetAsync(g->d_ctr, 0, 5 * sizeof(unsigned long long), st));
    launch_census(g, r, h, shard, false, st);
    LKG_HIP(hipGetLastError());
    LKG_HIP(hipMemcpyAsync(g->h_ctr, g->d_ctr, C_TOTAL * sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
    if (write_lists) LKG_TRY(census_lists(g, r, h, shard, st));
    LKG_HIP(hipStreamSynchronize(st));
    return LOGOSKG_OK;
}

logoskg_status count_reached(logoskg_result *r, hipStream_t st);  // result.hip

}  // namespace lkg

using namespace lkg;

extern "C" void logoskg_result_free(logoskg_result *r) {
    if (!r) return;
    logoskg_graph *g = r->g;
    (void)hipSetDevice(g->device);
    drop_walk_tables(r);
    // levels follows visited and live follows act in one allocation each
    void *ptrs[] = {r->visited, r->act, r->allow, r->tile_base,
                    r->super_base, r->mega_base, r->d_reached_off, r->lvl_tile_base, r->lvl_super_base,
                    r->lvl_mega_base, r->d_level_off, r->trip_ent, r->trip_off,
                    r->trip_chunk_entry, r->trip_chunk_first, r->tile_ent, r->cpos, r->act_chunk};
    constexpr int n = (int)(sizeof(ptrs) / sizeof(ptrs[0]));
    bool zeroed[n] = {};
    const hipStream_t st = r->last_stream;
    if (r->complete && r->visited && r->act) {  // hand the planes and the bitmaps back as zeros
        ProfScope ps(g->prof, KK_CLEAR, st);
        const long long plane = r->Epad * r->W, actw = r->Epad / 32;
        const dim3 grid(blocks_for(r->Epad / 64, 4)), block(256);
        switch (r->W) {
            case 1: k_sparse_clear<1><<<grid, block, 0, st>>>(r->Epad, r->k + 1, r->act, actw, r->visited, r->levels, plane, r->live); break;
            case 4: k_sparse_clear<4><<<grid, block, 0, st>>>(r->Epad, r->k + 1, r->act, actw, r->visited, r->levels, plane, r->live); break;
            default: k_sparse_clear<16><<<grid, block, 0, st>>>(r->Epad, r->k + 1, r->act, actw, r->visited, r->levels, plane, r->live); break;
        }
        if (hipGetLastError() == hipSuccess) zeroed[0] = zeroed[1] = true;
        if (g->prof.on && r->n_active > 0) g->prof.acc[KK_CLEAR].units[3] += 2 * r->n_active * r->W;
    }
    // the blocks may still be in use by work on the stream of the result's last call
    g->pool.release_after(ptrs, zeroed, n, st);
    delete r;
}

extern "C" logoskg_status logoskg_khop(logoskg_graph *g, const logoskg_query_batch *b, logoskg_result **out) {
    if (!g || !b || !out) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    *out = nullptr;
    if (b->struct_size != sizeof(logoskg_query_batch)) {
        set_error("logoskg_query_batch.struct_size is %u, expected %zu", b->struct_size, sizeof(*b));
        return LOGOSKG_EINVAL;
    }
    if (b->num_queries < 1 || b->num_queries > LOGOSKG_MAX_QUERIES || b->k < 0 || b->k > LOGOSKG_MAX_K ||
        b->num_seeds < 0 || !b->seed_off || (b->num_seeds > 0 && !b->seeds)) {
        set_error("bad query batch: Q=%d k=%d num_seeds=%lld", b->num_queries, b->k, (long long)b->num_seeds);
        return LOGOSKG_EINVAL;
    }
    uint32_t dir = b->flags & LOGOSKG_DIR_MASK;
    const bool walk_exact = (b->flags & LOGOSKG_WALK_EXACT) != 0;
    if (dir == 3u) { set_error("bad direction flags"); return LOGOSKG_EINVAL; }
    LKG_HIP(hipSetDevice(g->device));
    hipStream_t st = (hipStream_t)b->stream;

    logoskg_result *r = new (std::nothrow) logoskg_result();
    if (!r) { set_error("out of host memory"); return LOGOSKG_ENOMEM; }
    r->g = g;
    r->Q = b->num_queries;
    r->k = b->k;
    r->W = words_for_queries(r->Q);
    r->Epad = g->Epad;
    r->has_mask = b->rel_mask != nullptr;
    r->walk_exact = walk_exact;
    r->stats.assign((size_t)r->k, logoskg_hop_stats{});
    const int W = r->W, k = r->k;
    const size_t plane = (size_t)r->Epad * W;
    const size_t actw = (size_t)r->Epad / 32;
    logoskg_status s;
    auto fail = [&](logoskg_status e) { logoskg_result_free(r); return e; };
    // visited and the level planes are one allocation, the active bitmaps and the live words
    // another: each is cleared by one fill
    const size_t act_bytes = actw * 4 * (size_t)(k + 1), live_bytes = (size_t)16 * 8 * (size_t)(k + 1);
    r->last_stream = st;
    bool planes_zero = false, act_zero = false;  // a block released by an earlier result comes back cleared
    if ((s = g->pool.alloc((void **)&r->visited, plane * 8 * (size_t)(k + 2), st, &planes_zero)) != LOGOSKG_OK) return fail(s);
    r->levels = r->visited + plane;
    if ((s = g->pool.alloc((void **)&r->act, act_bytes + live_bytes, st, &act_zero)) != LOGOSKG_OK) return fail(s);
    r->live = reinterpret_cast<unsigned long long *>(reinterpret_cast<char *>(r->act) + act_bytes);
    if (r->has_mask && (s = g->pool.alloc((void **)&r->allow, (size_t)g->R * W * 8, st)) != LOGOSKG_OK) return fail(s);

#define KH(call)                                  \
    do {                                          \
        logoskg_status s2_ = [&]() -> logoskg_status { LKG_HIP(call); return LOGOSKG_OK; }(); \
        if (s2_ != LOGOSKG_OK) return fail(s2_);  \
    } while (0)

    {
        ProfScope ps(g->prof, KK_CLEAR, st);
        if (!planes_zero) {
            KH(hipMemsetAsync(r->visited, 0, plane * 8 * (size_t)(k + 2), st));
            g->prof.acc[KK_CLEAR].units[3] += g->prof.on ? (long long)(plane * (size_t)(k + 2)) : 0;
        }
        if (!act_zero) KH(hipMemsetAsync(r->act, 0, act_bytes + live_bytes, st));
        KH(hipMemsetAsync(g->d_ctr, 0, C_TOTAL * sizeof(unsigned long long), st));
    }
    g->prof.begin(KK_SEED, st);
    if (r->has_mask) {
        int n = g->R * W;
        k_allow<<<dim3((n + 255) / 256), dim3(256), 0, st>>>(r->Q, g->R, W, (g->R + 63) / 64,
                                                             (const unsigned long long *)b->rel_mask,
                                                             (unsigned long long *)r->allow);
    }
    k_seed<<<dim3((r->Q + 255) / 256), dim3(256), 0, st>>>(r->Q, (long long)b->num_seeds,
                                                           (const long long *)b->seed_off, b->seeds, g->E, W,
                                                           (unsigned long long *)r->levels,
                                                           (unsigned long long *)r->visited, r->act, g->d_ctr);
    g->prof.end(st);
    KH(hipGetLastError());
    const bool want_stats = g->prof.counters;
    if ((s = census(g, r, 0, -1, false, st)) != LOGOSKG_OK) return fail(s);
    if (g->h_ctr[C_ERR]) {
        set_error("seed_off / seeds are inconsistent or out of range (device check, code %llu)", g->h_ctr[C_ERR]);
        return fail(LOGOSKG_EINVAL);
    }
    for (int h = 1; h <= k; ++h) {
        logoskg_hop_stats &hs = r->stats[h - 1];
        long long rows = (long long)g->h_ctr[C_NROWS];
        long long fedges = (long long)g->h_ctr[C_FEDGES];
        if (rows == 0) break;  // nothing can be reached any more: the remaining levels stay empty
        hs.active_rows = rows;
        hs.frontier_edges = fedges;
        const bool pull = dir == LOGOSKG_DIR_PULL || (dir == LOGOSKG_DIR_AUTO && fedges * 12 > g->T);
        hs.direction = pull ? LOGOSKG_DIR_PULL : LOGOSKG_DIR_PUSH;
        unsigned long long hc[C_TOTAL];
        memcpy(hc, g->h_ctr, sizeof(hc));
        if (want_stats)
            KH(hipMemsetAsync(g->d_ctr + C_STATS, 0, 4 * KK_NUM * sizeof(unsigned long long), st));
        if (g->num_shards > 1) {
            // Alg. 1: the hop visits sub-graphs one after the other through the cache -- the
            // subject shards that hold a frontier row (push) or every object range (pull)
            if ((s = run_sharded_hop(g, r, h, pull, want_stats, hc, st, &hs)) != LOGOSKG_OK) return fail(s);
            KH(hipGetLastError());
        } else {
            hs.shards_touched = 1;
            if (!pull && (s = census_lists(g, r, h - 1, -1, st)) != LOGOSKG_OK) return fail(s);
            launch_resident_hop(g, r, h, pull, want_stats, hc, st);
            KH(hipGetLastError());
        }
        if ((s = census(g, r, h, -1, false, st)) != LOGOSKG_OK) return fail(s);
        hs.entities_reached = (long long)g->h_ctr[C_NACTIVE];
        if (hs.direction == LOGOSKG_DIR_PULL) {
            for (int kind : {KK_PULL_TAIL, KK_PULL_SEG}) {
                const unsigned long long *c = g->h_ctr + C_STATS + 4 * kind;
                hs.rows_scanned += (long long)c[0];
                hs.edges_scanned += (long long)c[1];
                hs.lines_gathered += (long long)c[2];
                for (int u = 0; u < 3; ++u) g->prof.acc[kind].units[u] += (long long)c[u];
                // distinct frontier lines this kernel can have gathered
                g->prof.acc[kind].units[3] += std::min<long long>((long long)c[2], (long long)hs.active_rows);
            }
        } else {
            hs.edges_scanned = fedges;
            hs.lines_gathered = fedges;
        }
    }
    if (!(b->flags & LOGOSKG_NO_COUNTS)) {
        if ((s = count_reached(r, st)) != LOGOSKG_OK) return fail(s);
    }
#undef KH
    r->complete = true;
    *out = r;
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_result_get_info(const logoskg_result *r, logoskg_result_info *o) {
    if (!r || !o) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    o->num_queries = r->Q;
    o->k = r->k;
    o->words_per_entity = r->W;
    o->num_levels = r->k + 1;
    o->padded_entities = r->Epad;
    o->visited = (const uint64_t *)r->visited;
    o->levels = (const uint64_t *)r->levels;
    o->total_reached = r->has_counts ? r->reached_off.back() : -1;
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_result_hop_stats(const logoskg_result *r, logoskg_hop_stats *o) {
    if (!r || (r->k > 0 && !o)) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    for (int i = 0; i < r->k; ++i) o[i] = r->stats[(size_t)i];
    return LOGOSKG_OK;
}

// ---------------------------------------------------------------- measurement aid
// The line gathers of a dense pull hop and nothing else: for every entry of the object-sorted CSR,
// in order, the 128-byte line of its subject is loaded with the access shape of k_pull_seg (one
// wavefront per 1,024 entries, eight lanes per line, eight lines per load instruction, four rounds
// in flight, the ids of the next 64 entries requested ahead) and ORed into sixteen words.  No row
// bounds, no visited or level lines, no writes: what this takes is what the memory system needs
// for the gathers of such a hop on this graph.
namespace lkg {
__global__ void __launch_bounds__(256)
k_probe_gather(const int32_t *__restrict__ in_sub, long long T, const ulonglong2 *__restrict__ lines,
               unsigned long long *out) {
    const long long lo = ((long long)blockIdx.x * 4 + (threadIdx.x >> 6)) * kPullSegment;
    if (lo >= T) return;  // wavefront-uniform
    const long long hi = min(T, lo + (long long)kPullSegment);
    const int l8 = lane() & 7, grp = lane() >> 3;
    unsigned long long a0 = 0, a1 = 0;
    int s_next = lo + lane() < hi ? in_sub[lo + lane()] : 0;
    for (long long j0 = lo; j0 < hi; j0 += 64) {
        const int s = s_next;
        const long long jn = j0 + 64 + lane();
        s_next = jn < hi ? in_sub[jn] : 0;
        const int n = (int)min(64ll, hi - j0);
        for (int base = 0; base < n; base += 32) {
            ulonglong2 l[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int i = base + 8 * x + grp;
                const int sx = __shfl(s, i & 63);
                l[x] = make_ulonglong2(0, 0);
                if (i < n) l[x] = lines[(size_t)sx * 8 + l8];
            }
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                a0 |= l[x].x;
                a1 |= l[x].y;
            }
        }
    }
#pragma unroll
    for (int m = 8; m < 64; m <<= 1) {
        a0 |= shfl_xor64(a0, m);
        a1 |= shfl_xor64(a1, m);
    }
    if (lane() < 8) {
        if (a0) atomicOr(&out[2 * lane()], a0);
        if (a1) atomicOr(&out[2 * lane() + 1], a1);
    }
}
}  // namespace lkg

extern "C" logoskg_status logoskg_probe_gather(const logoskg_graph *g, const uint64_t *lines, uint64_t *out16,
                                               void *stream) {
    if (!g || !lines || !out16) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    if (g->num_shards > 1 || !g->in_sub) {
        set_error("the gather probe needs a resident graph");
        return LOGOSKG_EINVAL;
    }
    LKG_HIP(hipSetDevice(g->device));
    hipStream_t st = static_cast<hipStream_t>(stream);
    LKG_HIP(hipMemsetAsync(out16, 0, 16 * sizeof(uint64_t), st));
    const long long nseg = (g->T + kPullSegment - 1) / kPullSegment;
    if (nseg > 0)
        k_probe_gather<<<dim3((unsigned)((nseg + 3) / 4)), dim3(256), 0, st>>>(
            g->in_sub, g->T, reinterpret_cast<const ulonglong2 *>(lines), reinterpret_cast<unsigned long long *>(out16));
    LKG_HIP(hipGetLastError());
    return LOGOSKG_OK;
}
