// logoskg_build: triple list -> device CSR forms of the SUB and OBJ incidence
// matrices (paper Sec. 3.2, Eq. 1-3) plus degree classes.  A resident graph is
// sorted on the GPU (build_device.hip); the host counting sorts below serve
// sharded graphs, whose edge arrays stay in host memory, and the host_build
// option.
#include <algorithm>
#include <numeric>

#include "common.h"

namespace lkg {

static thread_local std::string g_err;

void set_error(const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_err = buf;
}

const char *get_error() { return g_err.c_str(); }

logoskg_status DevPool::alloc(void **out, size_t bytes, hipStream_t st, bool have_stream, bool *zeroed) {
    if (zeroed) *zeroed = false;
    if (bytes == 0) bytes = 256;
    bytes = (bytes + 255) & ~size_t(255);
    auto it = free_.lower_bound(bytes);
    if (it != free_.end() && it->first <= bytes * 2) {
        Block b = it->second;
        live_[b.p] = it->first;
        free_.erase(it);
        if (b.after) {  // released behind work that may still run
            hipError_t e = hipSuccess;
            if (!have_stream) e = hipEventSynchronize(b.after->ev);
            else if (b.after->stream != st) e = hipStreamWaitEvent(st, b.after->ev, 0);
            if (e != hipSuccess) {
                set_error("waiting for a released block failed: %s", hipGetErrorString(e));
                return LOGOSKG_EDEVICE;
            }
        }
        if (zeroed) *zeroed = b.zeroed;
        *out = b.p;
        return LOGOSKG_OK;
    }
    void *p = nullptr;
    if (!raw_alloc(&p, bytes)) {
        trim();  // give cached blocks back and retry once
        if (!raw_alloc(&p, bytes)) {
            set_error("device allocation of %zu bytes failed%s", bytes, alloc_fn_ ? " (caller's allocator)" : "");
            return LOGOSKG_ENOMEM;
        }
    }
    held_ += bytes;
    live_[p] = bytes;
    *out = p;
    return LOGOSKG_OK;
}

bool DevPool::raw_alloc(void **p, size_t bytes) {
    if (alloc_fn_) {
        *p = alloc_fn_(bytes, ctx_);
        return *p != nullptr;
    }
    if (hipMalloc(p, bytes) == hipSuccess) return true;
    (void)hipGetLastError();
    *p = nullptr;
    return false;
}

void DevPool::raw_free(void *p) {
    if (free_fn_) free_fn_(p, ctx_);
    else (void)hipFree(p);
}

void DevPool::release(void *p) {
    if (!p) return;
    auto it = live_.find(p);
    if (it == live_.end()) return;
    free_.emplace(it->second, Block{p, nullptr, false});
    live_.erase(it);
}

// The blocks become reusable behind the work issued on `st` so far: one event for all of them
// (it goes back to the spare list when the last of these blocks has been handed out again).
void DevPool::release_after(void *const *ptrs, const bool *zeroed, int n, hipStream_t st) {
    hipEvent_t ev = nullptr;
    if (!spare_events_.empty()) {
        ev = spare_events_.back();
        spare_events_.pop_back();
    } else if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) {
        (void)hipGetLastError();
        ev = nullptr;
    }
    std::shared_ptr<After> after;
    if (ev && hipEventRecord(ev, st) == hipSuccess) {
        after = std::shared_ptr<After>(new After{ev, st}, [this](After *a) {
            spare_events_.push_back(a->ev);
            delete a;
        });
    } else {  // no event: wait here, then the blocks are free without conditions
        (void)hipGetLastError();
        (void)hipStreamSynchronize(st);
        if (ev) spare_events_.push_back(ev);
    }
    for (int i = 0; i < n; ++i) {
        if (!ptrs[i]) continue;
        auto it = live_.find(ptrs[i]);
        if (it == live_.end()) continue;
        free_.emplace(it->second, Block{ptrs[i], after, zeroed ? zeroed[i] : false});
        live_.erase(it);
    }
}

void DevPool::trim() {
    for (auto &kv : free_) {
        if (kv.second.after) (void)hipEventSynchronize(kv.second.after->ev);
        raw_free(kv.second.p);
        held_ -= kv.first;
    }
    free_.clear();
}

DevPool::~DevPool() {
    free_.clear();  // returns the events of pending releases to the spare list
    for (hipEvent_t e : spare_events_) (void)hipEventDestroy(e);
    spare_events_.clear();
}

const char *const kKernelNames[KK_NUM] = {
    "clear_planes", "seed_scatter", "frontier_census", "live_queries", "push_tail", "push_seg",
    "update_visited", "pull_tail", "pull_seg", "pull_finish", "count_tiles", "scan_counts",
    "lists", "pred", "pred_rows", "pred_mid_rows", "traversed", "paths", "shard_copy", "active_triples",
    "pred_walk"};

void Profiler::begin(int kind, hipStream_t st) {
    if (!on) return;
    hipEvent_t a = nullptr;
    if (!spare.empty()) { a = spare.back(); spare.pop_back(); }
    else if (hipEventCreate(&a) != hipSuccess) return;
    (void)hipEventRecord(a, st);
    cur_a = a;
    cur_kind = kind;
}

void Profiler::end(hipStream_t st) {
    if (!on || !cur_a) return;
    hipEvent_t b = nullptr;
    if (!spare.empty()) { b = spare.back(); spare.pop_back(); }
    else if (hipEventCreate(&b) != hipSuccess) { spare.push_back(cur_a); cur_a = nullptr; return; }
    (void)hipEventRecord(b, st);
    recs.push_back({cur_kind, cur_a, b});
    cur_a = nullptr;
}

void Profiler::drain() {
    for (auto &r : recs) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
            acc[r.kind].launches++;
            acc[r.kind].total_ms += ms;
            if (ms > acc[r.kind].max_ms) acc[r.kind].max_ms = ms;
        }
        spare.push_back(r.a);
        spare.push_back(r.b);
    }
    recs.clear();
}

void Profiler::release() {
    drain();
    for (hipEvent_t e : spare) (void)hipEventDestroy(e);
    spare.clear();
}

// The helper streams (two for the fetch's side work, one for shard copies) are made once per
// device and shared by every graph on it; they live until the process ends.  Work of different
// graphs on one helper stream is only serialised: every dependency goes through events.
hipStream_t helper_stream(int device, int which) {
    static std::mutex mu;
    static std::map<int, std::array<hipStream_t, 3>> table;
    std::lock_guard<std::mutex> lock(mu);
    auto &row = table[device];  // value-initialised to null handles
    if (!row[which] && hipStreamCreateWithFlags(&row[which], hipStreamNonBlocking) != hipSuccess) {
        (void)hipGetLastError();
        row[which] = nullptr;
    }
    return row[which];
}

template <typename T>
static logoskg_status upload(T **dst, const std::vector<T> &src, size_t *acct) {
    size_t bytes = std::max<size_t>(src.size(), 1) * sizeof(T);
    LKG_HIP(hipMalloc((void **)dst, bytes));
    if (!src.empty()) LKG_HIP(hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice));
    *acct += bytes;
    return LOGOSKG_OK;
}

// Object rows with >= 1 entry: short rows, segments of the longer ones (longest
// rows first), rows with several segments, and the hub rows.
static void classify_rows(const std::vector<uint32_t> &off, int32_t E, int hub_min,
                          std::vector<ShortRow> &tail, std::vector<PullSegment> &seg,
                          std::vector<int32_t> &multi, std::vector<int32_t> &longer, int64_t *n_hub) {
    std::vector<std::vector<int32_t>> bucket(kTailMaxDegree + 1);
    *n_hub = 0;
    for (int32_t v = 0; v < E; ++v) {
        uint32_t d = off[v + 1] - off[v];
        if (d == 0) continue;
        if (d >= (uint32_t)hub_min) ++*n_hub;
        if (d > (uint32_t)kTailMaxDegree) longer.push_back(v);
        else bucket[d].push_back(v);
    }
    for (int d = kTailMaxDegree; d >= 1; --d)
        for (int32_t v : bucket[d]) tail.push_back({v, off[v], off[v + 1]});
    std::stable_sort(longer.begin(), longer.end(), [&](int32_t a, int32_t b) {
        return off[a + 1] - off[a] > off[b + 1] - off[b];
    });
    for (int32_t v : longer) {
        const bool several = off[v + 1] - off[v] > (uint32_t)kPullSegment;
        if (several) multi.push_back(v);
        for (uint32_t j = off[v]; j < off[v + 1]; j += kPullSegment)
            seg.push_back({v, j, std::min(j + (uint32_t)kPullSegment, off[v + 1]), several ? 1u : 0u});
    }
}

}  // namespace lkg

using namespace lkg;

extern "C" logoskg_status logoskg_build(const int32_t *subj, const int32_t *rel, const int32_t *obj,
                                        int64_t T, int32_t E, int32_t R,
                                        const logoskg_build_opts *opts, logoskg_graph **out) {
    if (!out) { set_error("out is NULL"); return LOGOSKG_EINVAL; }
    *out = nullptr;
    if (T < 0 || T >= (int64_t(1) << 31) || E <= 0 || R <= 0 || R > 65536) {
        set_error("sizes out of range: T=%lld E=%d R=%d", (long long)T, E, R);
        return LOGOSKG_EINVAL;
    }
    if (T > 0 && (!subj || !rel || !obj)) { set_error("triple arrays are NULL"); return LOGOSKG_EINVAL; }
    logoskg_build_opts o;
    memset(&o, 0, sizeof(o));
    if (opts) {
        if (opts->struct_size < 8 || opts->struct_size > sizeof(o)) {
            set_error("logoskg_build_opts.struct_size is %u", opts->struct_size);
            return LOGOSKG_EINVAL;
        }
        memcpy(&o, opts, opts->struct_size);
    }
    if (o.num_shards < 0 || o.num_shards > 127 || o.hub_min_degree < 0 || o.max_resident_shards < 0) {
        set_error("bad build options");
        return LOGOSKG_EINVAL;
    }
    if ((o.dev_alloc == nullptr) != (o.dev_free == nullptr)) {
        set_error("dev_alloc and dev_free must be given together");
        return LOGOSKG_EINVAL;
    }
    if (o.shard_dir && o.shard_dir[0] && o.num_shards <= 1) {
        set_error("shard_dir needs num_shards > 1");
        return LOGOSKG_EINVAL;
    }
    const bool device_build = o.num_shards <= 1 && !o.host_build;
    const bool device_sorts = !o.host_build;  // then the ids are checked on the device
    for (int64_t t = 0; !device_sorts && t < T; ++t) {
        if ((uint32_t)subj[t] >= (uint32_t)E || (uint32_t)obj[t] >= (uint32_t)E ||
            (uint32_t)rel[t] >= (uint32_t)R) {
            set_error("triple %lld = (%d, %d, %d) is out of range", (long long)t, subj[t], rel[t], obj[t]);
            return LOGOSKG_EINVAL;
        }
    }
    int ndev = 0;
    LKG_HIP(hipGetDeviceCount(&ndev));
    if (o.device < 0 || o.device >= ndev) { set_error("device %d not present", o.device); return LOGOSKG_EINVAL; }
    LKG_HIP(hipSetDevice(o.device));

    logoskg_graph *g = new (std::nothrow) logoskg_graph();
    if (!g) { set_error("out of host memory"); return LOGOSKG_ENOMEM; }
    g->device = o.device;
    g->E = E;
    g->R = R;
    g->T = T;
    g->Epad = ((int64_t)E + 63) / 64 * 64;
    g->hub_min = o.hub_min_degree > 0 ? std::max(o.hub_min_degree, kTailMaxDegree + 1) : kDefaultHubMin;
    g->num_shards = o.num_shards > 1 ? o.num_shards : 1;
    if (o.dev_alloc) g->pool.set_allocator(o.dev_alloc, o.dev_free, o.alloc_ctx);

    logoskg_status st = LOGOSKG_OK;
    auto fail = [&](logoskg_status s) { logoskg_graph_free(g); return s; };
    try {
        // row classes of the object-sorted CSR (pull and predecessor work lists)
        auto object_row_classes = [&](const std::vector<uint32_t> &ioff) -> logoskg_status {
            std::vector<int32_t> multi, longer;
            std::vector<ShortRow> tail;
            std::vector<PullSegment> seg;
            classify_rows(ioff, E, g->hub_min, tail, seg, multi, longer, &g->in_rows.n_hub);
            g->in_rows.n_giant = 0;
            for (int32_t v : longer)  // longest first
                if (ioff[(size_t)v + 1] - ioff[v] >= (uint32_t)std::max(kGiantRowMin, g->hub_min)) g->in_rows.n_giant++;
                else break;
            {   // segments of the giant rows, for the predecessor pass
                std::vector<uint32_t> first((size_t)g->in_rows.n_giant + 1, 0);
                for (int64_t i = 0; i < g->in_rows.n_giant; ++i) {
                    const int32_t v = longer[(size_t)i];
                    first[(size_t)i + 1] = first[(size_t)i] + (ioff[(size_t)v + 1] - ioff[v] + kGiantSegment - 1) / kGiantSegment;
                }
                g->in_rows.n_giant_segs = first.back();
                LKG_TRY(upload(&g->in_rows.giant_seg_first, first, &g->static_bytes));
            }
            g->in_rows.n_tail = (int64_t)tail.size();
            g->in_rows.n_seg = (int64_t)seg.size();
            g->in_rows.n_multi = (int64_t)multi.size();
            g->in_rows.n_long = (int64_t)longer.size();
            LKG_TRY(upload(&g->in_rows.tail, tail, &g->static_bytes));
            LKG_TRY(upload(&g->in_rows.seg, seg, &g->static_bytes));
            LKG_TRY(upload(&g->in_rows.multi, multi, &g->static_bytes));
            LKG_TRY(upload(&g->in_rows.longrows, longer, &g->static_bytes));
            return LOGOSKG_OK;
        };
        auto subject_row_counts = [&](const std::vector<uint32_t> &ooff) {
            for (int32_t e = 0; e < E; ++e) {
                uint32_t d = ooff[(size_t)e + 1] - ooff[e];
                if (d > 0) g->n_out_rows++;
                if (d >= (uint32_t)g->hub_min) g->n_out_hubs++;
            }
        };
        if (device_build) {
            std::vector<uint32_t> ooff, ioff;
            if ((st = build_csr_on_device(g, subj, rel, obj, &ooff, &ioff)) != LOGOSKG_OK) return fail(st);
            g->row_begin = g->out_off;
            subject_row_counts(ooff);
            if ((st = object_row_classes(ioff)) != LOGOSKG_OK) return fail(st);
        } else if (device_sorts) {
            // a sharded graph whose two sorts run on the device; the sorted arrays go to pinned host memory
            TripleSorter *sorter = nullptr;
            if ((st = sorter_create(g, subj, rel, obj, &sorter)) != LOGOSKG_OK) return fail(st);
            std::unique_ptr<TripleSorter, void (*)(TripleSorter *)> guard(sorter, sorter_destroy);
            std::vector<uint32_t> ooff;
            if ((st = sorter_offsets(sorter, false, &ooff)) != LOGOSKG_OK) return fail(st);
            subject_row_counts(ooff);
            if ((st = upload(&g->out_off, ooff, &g->static_bytes)) != LOGOSKG_OK) return fail(st);
            if ((st = build_shards(g, subj, rel, obj, &o, ooff, sorter)) != LOGOSKG_OK) return fail(st);
        } else {
        // out-degrees are needed by both the resident and the sharded form
        std::vector<uint32_t> ooff((size_t)E + 1, 0);
        for (int64_t t = 0; t < T; ++t) ooff[(size_t)subj[t] + 1]++;
        for (int32_t e = 0; e < E; ++e) ooff[(size_t)e + 1] += ooff[e];
        subject_row_counts(ooff);
        if ((st = upload(&g->out_off, ooff, &g->static_bytes)) != LOGOSKG_OK) return fail(st);

        if (g->num_shards > 1) {
            if ((st = build_shards(g, subj, rel, obj, &o, ooff, nullptr)) != LOGOSKG_OK) return fail(st);
        } else {
            g->row_begin = g->out_off;
            {   // SUB: stable counting sort by subject
                std::vector<int32_t> oobj((size_t)T);
                std::vector<uint16_t> orel((size_t)T);
                std::vector<uint32_t> cur(ooff.begin(), ooff.end() - 1);
                for (int64_t t = 0; t < T; ++t) {
                    uint32_t p = cur[subj[t]]++;
                    oobj[p] = obj[t];
                    orel[p] = (uint16_t)rel[t];
                }
                if ((st = upload(&g->out_obj, oobj, &g->static_bytes)) != LOGOSKG_OK) return fail(st);
                if ((st = upload(&g->out_rel, orel, &g->static_bytes)) != LOGOSKG_OK) return fail(st);
            }
            {   // OBJ: stable counting sort by object, edge ids ascend inside a row
                std::vector<uint32_t> ioff((size_t)E + 1, 0);
                for (int64_t t = 0; t < T; ++t) ioff[(size_t)obj[t] + 1]++;
                for (int32_t e = 0; e < E; ++e) ioff[(size_t)e + 1] += ioff[e];
                std::vector<int32_t> isub((size_t)T), ieid((size_t)T);
                std::vector<uint16_t> irel((size_t)T);
                std::vector<uint32_t> cur(ioff.begin(), ioff.end() - 1);
                for (int64_t t = 0; t < T; ++t) {
                    uint32_t p = cur[obj[t]]++;
                    isub[p] = subj[t];
                    irel[p] = (uint16_t)rel[t];
                    ieid[p] = (int32_t)t;
                }
                if ((st = upload(&g->in_off, ioff, &g->static_bytes)) != LOGOSKG_OK) return fail(st);
                if ((st = upload(&g->in_sub, isub, &g->static_bytes)) != LOGOSKG_OK) return fail(st);
                if ((st = upload(&g->in_rel, irel, &g->static_bytes)) != LOGOSKG_OK) return fail(st);
                if ((st = upload(&g->in_eid, ieid, &g->static_bytes)) != LOGOSKG_OK) return fail(st);
                if ((st = object_row_classes(ioff)) != LOGOSKG_OK) return fail(st);
            }
        }
        }
    } catch (const std::bad_alloc &) {
        set_error("out of host memory while sorting %lld triples", (long long)T);
        return fail(LOGOSKG_ENOMEM);
    }

    auto dev_alloc = [&](void **p, size_t bytes) -> logoskg_status {
        LKG_HIP(hipMalloc(p, bytes));
        g->static_bytes += bytes;
        return LOGOSKG_OK;
    };
    g->fr_seg_cap = (int64_t)E + T / kPushSegment + 64;  // every long row adds < deg/segment + 1 items
    if ((st = dev_alloc((void **)&g->fr_tail, (size_t)E * sizeof(int32_t))) != LOGOSKG_OK) return fail(st);
    if ((st = dev_alloc((void **)&g->fr_seg, (size_t)g->fr_seg_cap * sizeof(RowSegment))) != LOGOSKG_OK) return fail(st);
    if ((st = dev_alloc((void **)&g->d_ctr, C_TOTAL * sizeof(unsigned long long))) != LOGOSKG_OK) return fail(st);
    if (hipHostMalloc((void **)&g->h_ctr, (C_TOTAL + 1) * sizeof(unsigned long long), hipHostMallocDefault) != hipSuccess) {
        set_error("hipHostMalloc failed");
        return fail(LOGOSKG_ENOMEM);
    }
    for (int i = 0; i < 2; ++i) {
        if (!(g->side[i] = helper_stream(g->device, i)) ||
            hipEventCreateWithFlags(&g->ev_join[i], hipEventDisableTiming) != hipSuccess) {
            set_error("could not create the helper streams");
            return fail(LOGOSKG_EDEVICE);
        }
    }
    if (hipEventCreateWithFlags(&g->ev_fork, hipEventDisableTiming) != hipSuccess) {
        set_error("could not create events");
        return fail(LOGOSKG_EDEVICE);
    }
    *out = g;
    return LOGOSKG_OK;
}

extern "C" void logoskg_graph_free(logoskg_graph *g) {
    if (!g) return;
    (void)hipSetDevice(g->device);
    // nothing of this graph may still be queued when its events, streams and buffers go away
    // (a caller's stream can hold a wait on one of the events below)
    (void)hipDeviceSynchronize();
    free_shards(g);
    g->prof.release();
    for (int i = 0; i < 2; ++i) {
        if (g->side[i]) (void)hipStreamSynchronize(g->side[i]);
        if (g->ev_join[i]) (void)hipEventDestroy(g->ev_join[i]);
    }
    if (g->ev_fork) (void)hipEventDestroy(g->ev_fork);
    if (g->ev_rows) (void)hipEventDestroy(g->ev_rows);

    void *ptrs[] = {g->out_off, g->out_obj, g->out_rel, g->in_off, g->in_sub, g->in_rel, g->in_eid,
                    g->in_rows.tail, g->in_rows.seg, g->in_rows.multi, g->in_rows.longrows, g->in_rows.giant_seg_first, g->fr_tail,
                    g->fr_seg, g->d_ctr, g->long_index, g->row_pred, g->out_eid, g->plane_buf};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    if (g->h_ctr) (void)hipHostFree(g->h_ctr);
    g->pool.trim();
    delete g;
}

extern "C" const char *logoskg_last_error(void) { return lkg::get_error(); }
extern "C" const char *logoskg_version(void) { return "logoskg-gfx950 0.1"; }

extern "C" logoskg_status logoskg_profile_enable(logoskg_graph *g, int32_t enable) {
    if (!g) { set_error("NULL graph"); return LOGOSKG_EINVAL; }
    g->prof.drain();
    g->prof.on = enable != 0;
    g->prof.counters = enable >= 2;
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_profile_read(logoskg_graph *g, logoskg_kernel_profile *out, int32_t capacity,
                                               int32_t *n_out) {
    if (!g || (capacity > 0 && !out)) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    (void)hipSetDevice(g->device);
    g->prof.drain();
    if (n_out) *n_out = KK_NUM;
    for (int i = 0; i < KK_NUM && i < capacity; ++i) {
        memset(&out[i], 0, sizeof(out[i]));
        strncpy(out[i].name, kKernelNames[i], sizeof(out[i].name) - 1);
        const Profiler::Acc &a = g->prof.acc[i];
        out[i].launches = a.launches;
        out[i].total_ms = a.total_ms;
        out[i].max_ms = a.max_ms;
        out[i].rows = a.units[0];
        out[i].edges = a.units[1];
        out[i].lines = a.units[2];
        out[i].items = a.units[3];
    }
    for (int i = 0; i < KK_NUM; ++i) g->prof.acc[i] = Profiler::Acc();
    return LOGOSKG_OK;
}
