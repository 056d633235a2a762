// logoskg_paths: shortest-path listing from the level planes (paper Sec. 3.3,
// "Path reconstruction", Eq. 5-7).  A triple t is on a shortest path of query q
// to its object when its subject sits exactly one hop closer to the seeds and
// q allows its relation; chaining such triples backward from the target always
// ends at a seed, so a depth-first walk over the object rows (edge ids
// ascending) lists the paths in (t_d, t_{d-1}, .., t_1) order and can stop at
// max_paths.
//
// logoskg_walks lists walks of a given number of triples on a result of the
// plain iteration (no visited set) with the same kernel: there level h holds
// the ends of the walks of h triples, so the backward walk from level d of the
// target through levels d-1 .. 0 meets exactly the walks of d allowed triples
// from a seed (Sec. 3.3: complete paths, extended hop by hop).
#include <algorithm>
#include <mutex>

#include "common.h"

namespace lkg {

// One wavefront per (query, target) pair.  The depth-first state is the same in every lane: all
// lanes compute it, write it to the pair's three stacks (same address, same value) and read it
// back, so a lane only ever reads what it has written itself.  An object row is scanned 64
// entries at a time: every lane tests one entry (subject one level closer for the query, relation
// allowed) and a ballot gives the admissible entries in ascending position = ascending edge id,
// so a row of a hundred thousand entries is not a single lane's loop.
__global__ void __launch_bounds__(256)
k_paths(long long n_pairs, int Q, int k, int W, int32_t E, long long plane,
        const unsigned long long *__restrict__ levels, const unsigned long long *__restrict__ allow,
        const uint32_t *__restrict__ in_off, const int32_t *__restrict__ in_sub,
        const uint16_t *__restrict__ in_rel, const int32_t *__restrict__ in_eid,
        const int32_t *__restrict__ query_idx, const int32_t *__restrict__ target,
        const int32_t *__restrict__ length, int max_paths, int32_t *path_count, int32_t *path_edges,
        int32_t *stk_vertex, uint32_t *stk_pos, int32_t *stk_edge) {
    const long long i = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (i >= n_pairs) return;  // wave-uniform
    const int v_lane = lane();
    int32_t *out = path_edges + (size_t)i * max_paths * k;
    for (long long x = v_lane; x < (long long)max_paths * k; x += 64) out[x] = -1;
    const int q = query_idx[i], v = target[i];
    if ((uint32_t)q >= (uint32_t)Q || (uint32_t)v >= (uint32_t)E) {
        if (v_lane == 0) path_count[i] = 0;
        return;
    }
    const int w = q >> 6;
    const unsigned long long bit = 1ull << (q & 63);
    int d = -1;
    if (length) {  // walks of exactly that many triples: the target has to sit in that level
        const int want = length[i];
        if (want >= 0 && want <= k && (levels[(size_t)want * plane + (size_t)v * W + w] & bit)) d = want;
    } else {       // shortest paths: the first level that holds the target
        for (int h = 0; h <= k; ++h)
            if (levels[(size_t)h * plane + (size_t)v * W + w] & bit) { d = h; break; }
    }
    if (d <= 0) {  // not reached: no path; a seed: one empty path
        if (v_lane == 0) path_count[i] = d == 0 ? 1 : 0;
        return;
    }
    // explicit stack, entry l (1..d) = the vertex at hop l of the partial path, the next
    // in-edge position to try for it, and the edge chosen into it
    int32_t *sv = stk_vertex + (size_t)i * k - 1;
    uint32_t *sp = stk_pos + (size_t)i * k - 1;
    int32_t *se = stk_edge + (size_t)i * k - 1;
    int found = 0, l = d;
    sv[d] = v;
    sp[d] = in_off[v];
    while (l <= d && found < max_paths) {
        const int x = sv[l];
        uint32_t j = sp[l];
        const uint32_t hi = in_off[x + 1];
        bool descended = false;
        const unsigned long long *lv = levels + (size_t)(l - 1) * plane;
        while (j < hi && found < max_paths) {
            const uint32_t jj = j + (uint32_t)v_lane;
            int s = 0, eid = 0;
            bool ok = false;
            if (jj < hi) {
                s = in_sub[jj];
                ok = (lv[(size_t)s * W + w] & bit) != 0ull;
                if (ok && allow) ok = (allow[(size_t)in_rel[jj] * W + w] & bit) != 0ull;
                if (ok) eid = in_eid[jj];
            }
            unsigned long long m = __ballot(ok);
            if (m == 0ull) {
                j += 64;
                continue;
            }
            if (l == 1) {  // every admissible entry of the chunk ends a path, in this order
                while (m && found < max_paths) {
                    const int f = __builtin_ctzll(m);
                    m &= m - 1;
                    int32_t *row = out + (size_t)found * k;
                    for (int a = 2 + v_lane; a <= d; a += 64) row[a - 1] = se[a];
                    const int ef = __shfl(eid, f);
                    if (v_lane == 0) row[0] = ef;
                    ++found;
                }
                j += 64;
            } else {  // take the first one and go down; the rest of the row is tried after coming back
                const int f = __builtin_ctzll(m);
                se[l] = __shfl(eid, f);
                sp[l] = j + (uint32_t)f + 1u;
                const int sf = __shfl(s, f);
                sv[l - 1] = sf;
                sp[l - 1] = in_off[sf];
                --l;
                descended = true;
                break;
            }
        }
        if (!descended) ++l;  // this vertex's row is exhausted: back to the vertex after it
    }
    if (v_lane == 0) path_count[i] = found;
}

}  // namespace lkg

using namespace lkg;

// Launches the listing kernel with the three depth-first stacks (vertex, next row position,
// chosen edge; n_pairs * max(k, 1) int32 each) laid out one after another in `ws`.
static logoskg_status launch_paths(logoskg_graph *g, const logoskg_result *r, const int32_t *query_idx,
                                   const int32_t *target, const int32_t *length, int64_t n_pairs, int32_t max_paths,
                                   int32_t *path_count, int32_t *path_edges, void *ws, hipStream_t st) {
    const int k = r->k;
    r->last_stream = st;
    const size_t per = (size_t)n_pairs * (size_t)std::max(k, 1) * 4;
    int32_t *sv = (int32_t *)ws;
    uint32_t *sp = (uint32_t *)((char *)ws + per);
    int32_t *se = (int32_t *)((char *)ws + 2 * per);
    // a sharded graph keeps its object-sorted triples in pinned host memory: the kernel reads the
    // rows it walks from there
    const int32_t *in_sub = g->in_sub, *in_eid = g->in_eid;
    const uint16_t *in_rel = g->in_rel;
    if (g->num_shards > 1 && !shard_in_arrays(g, &in_sub, &in_rel, &in_eid)) {
        set_error("the object-sorted triples of the sharded graph are not available");
        return LOGOSKG_EINTERNAL;
    }
    ProfScope ps(g->prof, KK_PATHS, st);
    k_paths<<<dim3((unsigned)((n_pairs + 3) / 4)), dim3(256), 0, st>>>(
        n_pairs, r->Q, k, r->W, g->E, r->Epad * r->W, (const unsigned long long *)r->levels,
        r->has_mask ? (const unsigned long long *)r->allow : nullptr, g->in_off, in_sub, in_rel, in_eid,
        query_idx, target, length, max_paths, path_count, path_edges, sv, sp, se);
    LKG_HIP(hipGetLastError());
    return LOGOSKG_OK;
}

static logoskg_status check_path_args(logoskg_graph *g, const logoskg_result *r, const int32_t *query_idx,
                                      const int32_t *target, int64_t n_pairs, int32_t max_paths,
                                      const int32_t *path_count, const int32_t *path_edges) {
    if (n_pairs < 0 || max_paths < 1 || max_paths > LOGOSKG_MAX_PATHS) {
        set_error("bad n_pairs / max_paths");
        return LOGOSKG_EINVAL;
    }
    if (n_pairs > 0 && (!query_idx || !target || !path_count || (r->k > 0 && !path_edges))) {
        set_error("NULL argument");
        return LOGOSKG_EINVAL;
    }
    return LOGOSKG_OK;
}

static logoskg_status list_paths(logoskg_graph *g, const logoskg_result *r, const int32_t *query_idx,
                                 const int32_t *target, const int32_t *length, int64_t n_pairs, int32_t max_paths,
                                 int32_t *path_count, int32_t *path_edges, void *stream) {
    LKG_TRY(check_path_args(g, r, query_idx, target, n_pairs, max_paths, path_count, path_edges));
    if (n_pairs == 0) return LOGOSKG_OK;
    LKG_HIP(hipSetDevice(g->device));
    hipStream_t st = (hipStream_t)stream;
    void *ws = nullptr;
    LKG_TRY(g->pool.alloc(&ws, (size_t)n_pairs * (size_t)std::max(r->k, 1) * 4 * 3));
    logoskg_status s = launch_paths(g, r, query_idx, target, length, n_pairs, max_paths, path_count, path_edges, ws, st);
    hipError_t e2 = hipStreamSynchronize(st);  // the workspace goes back to the pool below
    g->pool.release(ws);
    LKG_TRY(s);
    LKG_HIP(e2);
    return LOGOSKG_OK;
}

// ---------------------------------------------------------------- listing without any allocation
// The depth-first stacks of logoskg_paths_static live in this array instead of a block from the
// graph's pool.  Every GPU the library runs on holds its own copy until the process ends; in host
// code the array's name is only a handle for hipGetSymbolAddress, the address that kernels and
// copies use is looked up once per device and kept in static_stack_ptr.
static __device__ __align__(256) unsigned char static_stacks[LOGOSKG_STATIC_PATH_SLOTS * 4 * 3];

constexpr int kMaxDevices = 64;
static void *static_stack_ptr[kMaxDevices];
static std::mutex static_stack_lock;

// Address of the calling device's copy of static_stacks (`device` must be current).
static logoskg_status static_stack_address(int device, void **out) {
    if (device < 0 || device >= kMaxDevices) {
        set_error("device ordinal %d is outside [0, %d)", device, kMaxDevices);
        return LOGOSKG_EINVAL;
    }
    std::lock_guard<std::mutex> lock(static_stack_lock);
    if (!static_stack_ptr[device]) {
        void *p = nullptr;
        LKG_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(static_stacks)));
        if (!p) { set_error("hipGetSymbolAddress returned a null address"); return LOGOSKG_EDEVICE; }
        static_stack_ptr[device] = p;
    }
    *out = static_stack_ptr[device];
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_paths_static(logoskg_graph *g, const logoskg_result *r, const int32_t *query_idx,
                                               const int32_t *target, int64_t n_pairs, int32_t max_paths,
                                               int32_t *path_count, int32_t *path_edges, void *stream) {
    if (!g || !r || r->g != g) { set_error("graph / result mismatch"); return LOGOSKG_EINVAL; }
    if (r->walk_exact) {
        set_error("shortest paths are not defined for a LOGOSKG_WALK_EXACT result");
        return LOGOSKG_EINVAL;
    }
    LKG_TRY(check_path_args(g, r, query_idx, target, n_pairs, max_paths, path_count, path_edges));
    const long long slots = (long long)n_pairs * std::max(r->k, 1);
    if (slots > (long long)LOGOSKG_STATIC_PATH_SLOTS) {
        set_error("logoskg_paths_static: n_pairs * max(k, 1) = %lld exceeds LOGOSKG_STATIC_PATH_SLOTS = %lld; "
                  "split the pair list or use logoskg_paths", slots, (long long)LOGOSKG_STATIC_PATH_SLOTS);
        return LOGOSKG_ERANGE;
    }
    if (n_pairs == 0) return LOGOSKG_OK;
    LKG_HIP(hipSetDevice(g->device));
    void *ws = nullptr;
    LKG_TRY(static_stack_address(g->device, &ws));
    // every stack entry is written before it is read, so nothing has to be cleared between calls
    return launch_paths(g, r, query_idx, target, nullptr, n_pairs, max_paths, path_count, path_edges, ws,
                        (hipStream_t)stream);
}

extern "C" logoskg_status logoskg_paths(logoskg_graph *g, const logoskg_result *r, const int32_t *query_idx,
                                        const int32_t *target, int64_t n_pairs, int32_t max_paths,
                                        int32_t *path_count, int32_t *path_edges, void *stream) {
    if (!g || !r || r->g != g) { set_error("graph / result mismatch"); return LOGOSKG_EINVAL; }
    if (r->walk_exact) {
        set_error("shortest paths are not defined for a LOGOSKG_WALK_EXACT result: use logoskg_walks");
        return LOGOSKG_EINVAL;
    }
    return list_paths(g, r, query_idx, target, nullptr, n_pairs, max_paths, path_count, path_edges, stream);
}

extern "C" logoskg_status logoskg_walks(logoskg_graph *g, const logoskg_result *r, const int32_t *query_idx,
                                        const int32_t *target, const int32_t *length, int64_t n_pairs,
                                        int32_t max_paths, int32_t *path_count, int32_t *path_edges, void *stream) {
    if (!g || !r || r->g != g) { set_error("graph / result mismatch"); return LOGOSKG_EINVAL; }
    if (!r->walk_exact) {
        set_error("walks of a given length need a LOGOSKG_WALK_EXACT result (levels = ends of the walks of h triples)");
        return LOGOSKG_EINVAL;
    }
    if (n_pairs > 0 && !length) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    return list_paths(g, r, query_idx, target, length, n_pairs, max_paths, path_count, path_edges, stream);
}
