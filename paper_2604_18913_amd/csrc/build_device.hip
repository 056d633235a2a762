// Device-side part of logoskg_build: the two stable sorts of the triple list
// (by subject for SUB, by object for OBJ, Sec. 3.2, Eq. 1-3) run on the GPU, for
// a resident graph (the sorted arrays stay in HBM) and for a sharded one (the
// sorted arrays go to pinned host memory, the subject order grouped by shard).  A least-significant-digit radix sort of (key, triple index)
// pairs is stable, so triple indices ascend inside a row exactly as in the host
// counting sort; the row offsets come from a histogram and a prefix sum.  The
// sort and the scan are rocPRIM's device-wide primitives; everything else is a
// handful of streaming kernels.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>

#include "common.h"

namespace lkg {

namespace {

constexpr int kBlock = 256;

inline unsigned grid_for(int64_t n) { return (unsigned)std::max<int64_t>(1, (n + kBlock - 1) / kBlock); }

// index of the first triple with an id out of range (INT64_MAX-like sentinel = none)
__global__ void k_check_triples(const int32_t *__restrict__ subj, const int32_t *__restrict__ rel,
                                const int32_t *__restrict__ obj, long long T, int32_t E, int32_t R,
                                unsigned long long *first_bad) {
    long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    if ((uint32_t)subj[t] >= (uint32_t)E || (uint32_t)obj[t] >= (uint32_t)E || (uint32_t)rel[t] >= (uint32_t)R)
        atomicMin(first_bad, (unsigned long long)t);
}

__global__ void k_iota(uint32_t *v, long long n) {
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) v[i] = (uint32_t)i;
}

// cnt[key + 1] += 1: after an inclusive prefix sum cnt[e] is the first place of row e
__global__ void k_degrees(const int32_t *__restrict__ key, long long T, uint32_t *cnt) {
    long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < T) atomicAdd(&cnt[key[t] + 1], 1u);
}

__global__ void k_gather_sub_rows(const uint32_t *__restrict__ eid, long long T, const int32_t *__restrict__ obj,
                                  const int32_t *__restrict__ rel, int32_t *out_obj, uint16_t *out_rel) {
    long long p = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= T) return;
    const uint32_t t = eid[p];
    out_obj[p] = obj[t];
    out_rel[p] = (uint16_t)rel[t];
}

__global__ void k_gather_obj_rows(const uint32_t *__restrict__ eid, long long T, const int32_t *__restrict__ subj,
                                  const int32_t *__restrict__ rel, int32_t *in_sub, uint16_t *in_rel,
                                  int32_t *in_eid) {
    long long p = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= T) return;
    const uint32_t t = eid[p];
    in_sub[p] = subj[t];
    in_rel[p] = (uint16_t)rel[t];
    in_eid[p] = (int32_t)t;
}

// subject_of[t] = subject of triple t, from the object-sorted arrays (which keep the triple index)
__global__ void k_subject_of_triple(const int32_t *__restrict__ in_sub, const int32_t *__restrict__ in_eid,
                                    long long T, uint32_t *subject_of) {
    long long p = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < T) subject_of[in_eid[p]] = (uint32_t)in_sub[p];
}

struct Scratch {  // device temporaries, freed on every way out
    std::vector<void *> ptrs;
    ~Scratch() {
        for (void *p : ptrs)
            if (p) (void)hipFree(p);
    }
    template <typename T>
    logoskg_status get(T **p, size_t n) {
        LKG_HIP(hipMalloc((void **)p, std::max<size_t>(n, 1) * sizeof(T)));
        ptrs.push_back(*p);
        return LOGOSKG_OK;
    }
};

// sorted_eid = triple indices in (key, index) order; off = row offsets of that order
logoskg_status sort_by(const int32_t *d_key, int64_t T, int32_t E, unsigned key_bits, uint32_t *d_iota,
                       uint32_t *d_keys_out, uint32_t *d_sorted_eid, uint32_t *d_off, void *d_tmp, size_t tmp_bytes) {
    LKG_HIP(hipMemsetAsync(d_off, 0, ((size_t)E + 1) * sizeof(uint32_t), nullptr));
    if (T > 0) {
        k_degrees<<<dim3(grid_for(T)), dim3(kBlock)>>>(d_key, T, d_off);
        size_t need = tmp_bytes;
        LKG_HIP(rocprim::radix_sort_pairs(d_tmp, need, reinterpret_cast<const uint32_t *>(d_key), d_keys_out, d_iota,
                                          d_sorted_eid, (size_t)T, 0u, key_bits));
    }
    size_t need = tmp_bytes;
    LKG_HIP(rocprim::inclusive_scan(d_tmp, need, d_off, d_off, (size_t)E + 1, rocprim::plus<uint32_t>()));
    LKG_HIP(hipGetLastError());
    return LOGOSKG_OK;
}

}  // namespace

// Fills g->out_off/out_obj/out_rel and g->in_off/in_sub/in_rel/in_eid from host triple arrays;
// returns the two offset arrays to the host as well (row classes are built there).
logoskg_status build_csr_on_device(logoskg_graph *g, const int32_t *subj, const int32_t *rel, const int32_t *obj,
                                   std::vector<uint32_t> *ooff, std::vector<uint32_t> *ioff) {
    const int64_t T = g->T;
    const int32_t E = g->E;
    Scratch tmp;
    int32_t *d_subj = nullptr, *d_rel = nullptr, *d_obj = nullptr;
    uint32_t *d_iota = nullptr, *d_keys = nullptr, *d_eid = nullptr;
    unsigned long long *d_bad = nullptr;
    LKG_TRY(tmp.get(&d_subj, (size_t)T));
    LKG_TRY(tmp.get(&d_rel, (size_t)T));
    LKG_TRY(tmp.get(&d_obj, (size_t)T));
    LKG_TRY(tmp.get(&d_iota, (size_t)T));
    LKG_TRY(tmp.get(&d_keys, (size_t)T));
    LKG_TRY(tmp.get(&d_eid, (size_t)T));
    LKG_TRY(tmp.get(&d_bad, 1));
    if (T > 0) {
        LKG_HIP(hipMemcpy(d_subj, subj, (size_t)T * 4, hipMemcpyHostToDevice));
        LKG_HIP(hipMemcpy(d_rel, rel, (size_t)T * 4, hipMemcpyHostToDevice));
        LKG_HIP(hipMemcpy(d_obj, obj, (size_t)T * 4, hipMemcpyHostToDevice));
    }
    const unsigned long long none = ~0ull;
    LKG_HIP(hipMemcpy(d_bad, &none, sizeof(none), hipMemcpyHostToDevice));
    if (T > 0) {
        k_check_triples<<<dim3(grid_for(T)), dim3(kBlock)>>>(d_subj, d_rel, d_obj, T, E, g->R, d_bad);
        k_iota<<<dim3(grid_for(T)), dim3(kBlock)>>>(d_iota, T);
    }
    unsigned long long bad = none;
    LKG_HIP(hipMemcpy(&bad, d_bad, sizeof(bad), hipMemcpyDeviceToHost));
    if (bad != none) {
        set_error("triple %llu = (%d, %d, %d) is out of range", bad, subj[bad], rel[bad], obj[bad]);
        return LOGOSKG_EINVAL;
    }
    unsigned key_bits = 1;
    while (key_bits < 32 && (1ull << key_bits) < (unsigned long long)E) ++key_bits;
    // one temporary buffer that serves the sort and the scan
    size_t sort_bytes = 0, scan_bytes = 0;
    LKG_HIP(rocprim::radix_sort_pairs(nullptr, sort_bytes, reinterpret_cast<const uint32_t *>(d_subj), d_keys, d_iota,
                                      d_eid, (size_t)std::max<int64_t>(T, 1), 0u, key_bits));
    LKG_HIP(rocprim::inclusive_scan(nullptr, scan_bytes, (uint32_t *)nullptr, (uint32_t *)nullptr, (size_t)E + 1,
                                    rocprim::plus<uint32_t>()));
    const size_t tmp_bytes = std::max(sort_bytes, scan_bytes);
    char *d_tmp = nullptr;
    LKG_TRY(tmp.get(&d_tmp, tmp_bytes));

    auto keep = [&](void **p, size_t bytes) -> logoskg_status {
        LKG_HIP(hipMalloc(p, std::max<size_t>(bytes, 4)));
        g->static_bytes += std::max<size_t>(bytes, 4);
        return LOGOSKG_OK;
    };
    // SUB: rows by subject
    LKG_TRY(keep((void **)&g->out_off, ((size_t)E + 1) * 4));
    LKG_TRY(keep((void **)&g->out_obj, (size_t)T * 4));
    LKG_TRY(keep((void **)&g->out_rel, (size_t)T * 2));
    LKG_TRY(sort_by(d_subj, T, E, key_bits, d_iota, d_keys, d_eid, g->out_off, d_tmp, tmp_bytes));
    if (T > 0) k_gather_sub_rows<<<dim3(grid_for(T)), dim3(kBlock)>>>(d_eid, T, d_obj, d_rel, g->out_obj, g->out_rel);
    // OBJ: rows by object, triple indices kept as edge ids
    LKG_TRY(keep((void **)&g->in_off, ((size_t)E + 1) * 4));
    LKG_TRY(keep((void **)&g->in_sub, (size_t)T * 4));
    LKG_TRY(keep((void **)&g->in_rel, (size_t)T * 2));
    LKG_TRY(keep((void **)&g->in_eid, (size_t)T * 4));
    LKG_TRY(sort_by(d_obj, T, E, key_bits, d_iota, d_keys, d_eid, g->in_off, d_tmp, tmp_bytes));
    if (T > 0)
        k_gather_obj_rows<<<dim3(grid_for(T)), dim3(kBlock)>>>(d_eid, T, d_subj, d_rel, g->in_sub, g->in_rel, g->in_eid);
    LKG_HIP(hipGetLastError());
    ooff->resize((size_t)E + 1);
    ioff->resize((size_t)E + 1);
    LKG_HIP(hipMemcpy(ooff->data(), g->out_off, ((size_t)E + 1) * 4, hipMemcpyDeviceToHost));
    LKG_HIP(hipMemcpy(ioff->data(), g->in_off, ((size_t)E + 1) * 4, hipMemcpyDeviceToHost));
    LKG_HIP(hipDeviceSynchronize());
    return LOGOSKG_OK;
}

// ---------------------------------------------------------------- sharded graphs
// The triple list on the device with the scratch of the sorts, alive during logoskg_build only.
struct TripleSorter {
    int64_t T = 0;
    int32_t E = 0;
    unsigned key_bits = 1;
    Scratch tmp;
    int32_t *d_subj = nullptr, *d_rel = nullptr, *d_obj = nullptr;
    uint32_t *d_iota = nullptr, *d_keys = nullptr, *d_eid = nullptr, *d_off = nullptr, *d_key_in = nullptr;
    int32_t *d_a = nullptr, *d_b = nullptr;  // gathered 4-byte columns
    uint16_t *d_r = nullptr;                 // gathered relation ids
    char *d_tmp = nullptr;
    size_t tmp_bytes = 0;
};

__global__ void k_row_keys(const int32_t *subj, long long T, const uint32_t *__restrict__ row_begin,
                           uint32_t *key) {
    long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < T) key[t] = row_begin[subj[t]];
}

logoskg_status sorter_create(logoskg_graph *g, const int32_t *subj, const int32_t *rel, const int32_t *obj,
                             TripleSorter **out) {
    *out = nullptr;
    std::unique_ptr<TripleSorter> s(new (std::nothrow) TripleSorter());
    if (!s) { set_error("out of host memory"); return LOGOSKG_ENOMEM; }
    const int64_t T = g->T;
    s->T = T;
    s->E = g->E;
    unsigned long long *d_bad = nullptr;
    LKG_TRY(s->tmp.get(&s->d_subj, (size_t)T));
    LKG_TRY(s->tmp.get(&s->d_rel, (size_t)T));
    LKG_TRY(s->tmp.get(&s->d_obj, (size_t)T));
    LKG_TRY(s->tmp.get(&s->d_iota, (size_t)T));
    LKG_TRY(s->tmp.get(&s->d_keys, (size_t)T));
    LKG_TRY(s->tmp.get(&s->d_eid, (size_t)T));
    LKG_TRY(s->tmp.get(&s->d_key_in, (size_t)T));
    LKG_TRY(s->tmp.get(&s->d_a, (size_t)T));
    LKG_TRY(s->tmp.get(&s->d_b, (size_t)T));
    LKG_TRY(s->tmp.get(&s->d_r, (size_t)T));
    LKG_TRY(s->tmp.get(&s->d_off, (size_t)g->E + 1));
    LKG_TRY(s->tmp.get(&d_bad, 1));
    if (T > 0) {
        LKG_HIP(hipMemcpy(s->d_subj, subj, (size_t)T * 4, hipMemcpyHostToDevice));
        LKG_HIP(hipMemcpy(s->d_rel, rel, (size_t)T * 4, hipMemcpyHostToDevice));
        LKG_HIP(hipMemcpy(s->d_obj, obj, (size_t)T * 4, hipMemcpyHostToDevice));
    }
    const unsigned long long none = ~0ull;
    LKG_HIP(hipMemcpy(d_bad, &none, sizeof(none), hipMemcpyHostToDevice));
    if (T > 0) {
        k_check_triples<<<dim3(grid_for(T)), dim3(kBlock)>>>(s->d_subj, s->d_rel, s->d_obj, T, g->E, g->R, d_bad);
        k_iota<<<dim3(grid_for(T)), dim3(kBlock)>>>(s->d_iota, T);
    }
    unsigned long long bad = none;
    LKG_HIP(hipMemcpy(&bad, d_bad, sizeof(bad), hipMemcpyDeviceToHost));
    if (bad != none) {
        set_error("triple %llu = (%d, %d, %d) is out of range", bad, subj[bad], rel[bad], obj[bad]);
        return LOGOSKG_EINVAL;
    }
    while (s->key_bits < 32 && (1ull << s->key_bits) < (unsigned long long)g->E) ++s->key_bits;
    size_t sort_bytes = 0, scan_bytes = 0;
    LKG_HIP(rocprim::radix_sort_pairs(nullptr, sort_bytes, s->d_key_in, s->d_keys, s->d_iota, s->d_eid,
                                      (size_t)std::max<int64_t>(T, 1), 0u, 32u));
    LKG_HIP(rocprim::inclusive_scan(nullptr, scan_bytes, (uint32_t *)nullptr, (uint32_t *)nullptr, (size_t)g->E + 1,
                                    rocprim::plus<uint32_t>()));
    s->tmp_bytes = std::max(sort_bytes, scan_bytes);
    LKG_TRY(s->tmp.get(&s->d_tmp, s->tmp_bytes));
    *out = s.release();
    return LOGOSKG_OK;
}

void sorter_destroy(TripleSorter *s) { delete s; }

// Row offsets of SUB (by_object = false) or OBJ on the host: off[e] = triples of smaller keys.
logoskg_status sorter_offsets(TripleSorter *s, bool by_object, std::vector<uint32_t> *off) {
    const int32_t *key = by_object ? s->d_obj : s->d_subj;
    LKG_HIP(hipMemsetAsync(s->d_off, 0, ((size_t)s->E + 1) * sizeof(uint32_t), nullptr));
    if (s->T > 0) k_degrees<<<dim3(grid_for(s->T)), dim3(kBlock)>>>(key, s->T, s->d_off);
    size_t need = s->tmp_bytes;
    LKG_HIP(rocprim::inclusive_scan(s->d_tmp, need, s->d_off, s->d_off, (size_t)s->E + 1, rocprim::plus<uint32_t>()));
    off->resize((size_t)s->E + 1);
    LKG_HIP(hipMemcpy(off->data(), s->d_off, ((size_t)s->E + 1) * 4, hipMemcpyDeviceToHost));
    return LOGOSKG_OK;
}

// Objects and relation ids in the shard-grouped subject order: triples sorted (stably, so triple
// indices ascend inside a subject) by the place where their subject's run begins.
logoskg_status sorter_subject_order(TripleSorter *s, const uint32_t *d_row_begin, int32_t *h_obj, uint16_t *h_rel) {
    const int64_t T = s->T;
    if (T == 0) return LOGOSKG_OK;
    k_row_keys<<<dim3(grid_for(T)), dim3(kBlock)>>>(s->d_subj, T, d_row_begin, s->d_key_in);
    size_t need = s->tmp_bytes;
    LKG_HIP(rocprim::radix_sort_pairs(s->d_tmp, need, s->d_key_in, s->d_keys, s->d_iota, s->d_eid, (size_t)T, 0u, 32u));
    k_gather_sub_rows<<<dim3(grid_for(T)), dim3(kBlock)>>>(s->d_eid, T, s->d_obj, s->d_rel, s->d_a, s->d_r);
    LKG_HIP(hipGetLastError());
    LKG_HIP(hipMemcpy(h_obj, s->d_a, (size_t)T * 4, hipMemcpyDeviceToHost));
    LKG_HIP(hipMemcpy(h_rel, s->d_r, (size_t)T * 2, hipMemcpyDeviceToHost));
    return LOGOSKG_OK;
}

// Subjects, relation ids and triple indices in object order (rows of OBJ, indices ascending inside a row).
logoskg_status sorter_object_order(TripleSorter *s, int32_t *h_sub, uint16_t *h_rel, int32_t *h_eid) {
    const int64_t T = s->T;
    if (T == 0) return LOGOSKG_OK;
    size_t need = s->tmp_bytes;
    LKG_HIP(rocprim::radix_sort_pairs(s->d_tmp, need, reinterpret_cast<const uint32_t *>(s->d_obj), s->d_keys, s->d_iota,
                                      s->d_eid, (size_t)T, 0u, s->key_bits));
    k_gather_obj_rows<<<dim3(grid_for(T)), dim3(kBlock)>>>(s->d_eid, T, s->d_subj, s->d_rel, s->d_a, s->d_r, s->d_b);
    LKG_HIP(hipGetLastError());
    LKG_HIP(hipMemcpy(h_sub, s->d_a, (size_t)T * 4, hipMemcpyDeviceToHost));
    LKG_HIP(hipMemcpy(h_rel, s->d_r, (size_t)T * 2, hipMemcpyDeviceToHost));
    LKG_HIP(hipMemcpy(h_eid, s->d_b, (size_t)T * 4, hipMemcpyDeviceToHost));
    return LOGOSKG_OK;
}

// g->out_eid[p] = index of the triple behind entry p of the subject-sorted CSR (SUB's rows, Eq. 1).
// The build keeps triple indices only with the object-sorted arrays; this repeats the stable sort
// by subject on (subject, triple index) pairs, so the order is the one of out_obj / out_rel.
logoskg_status ensure_out_eid(logoskg_graph *g, hipStream_t st) {
    if (g->out_eid) return LOGOSKG_OK;
    // a sharded graph keeps the object-sorted triples in pinned host memory (read in place here) and
    // its rows of SUB in the shard-grouped order: the sort key is the place where a subject's run begins
    const int32_t *in_sub = g->in_sub, *in_eid = g->in_eid;
    const uint16_t *in_rel = g->in_rel;
    const bool sharded = g->num_shards > 1;
    if (sharded && !shard_in_arrays(g, &in_sub, &in_rel, &in_eid)) {
        set_error("the object-sorted triples of the sharded graph are not available");
        return LOGOSKG_EINTERNAL;
    }
    const int64_t T = g->T;
    Scratch tmp;
    uint32_t *d_subject = nullptr, *d_iota = nullptr, *d_keys = nullptr;
    LKG_TRY(tmp.get(&d_subject, (size_t)T));
    LKG_TRY(tmp.get(&d_iota, (size_t)T));
    LKG_TRY(tmp.get(&d_keys, (size_t)T));
    int32_t *eid = nullptr;
    LKG_HIP(hipMalloc((void **)&eid, std::max<size_t>((size_t)T, 1) * 4));
    auto fail = [&](logoskg_status s) { (void)hipFree(eid); return s; };
    if (T > 0) {
        unsigned key_bits = 1;
        while (key_bits < 32 && (1ull << key_bits) < (unsigned long long)g->E) ++key_bits;
        if (sharded) key_bits = 32;
        k_subject_of_triple<<<dim3(grid_for(T)), dim3(kBlock), 0, st>>>(in_sub, in_eid, T, d_subject);
        if (sharded)
            k_row_keys<<<dim3(grid_for(T)), dim3(kBlock), 0, st>>>(reinterpret_cast<const int32_t *>(d_subject), T,
                                                                   g->row_begin, d_subject);
        k_iota<<<dim3(grid_for(T)), dim3(kBlock), 0, st>>>(d_iota, T);
        size_t bytes = 0;
        hipError_t e = rocprim::radix_sort_pairs(nullptr, bytes, d_subject, d_keys, d_iota, (uint32_t *)eid, (size_t)T,
                                                 0u, key_bits, st);
        char *d_tmp = nullptr;
        if (e == hipSuccess && tmp.get(&d_tmp, bytes) != LOGOSKG_OK) return fail(LOGOSKG_ENOMEM);
        if (e == hipSuccess)
            e = rocprim::radix_sort_pairs(d_tmp, bytes, d_subject, d_keys, d_iota, (uint32_t *)eid, (size_t)T, 0u,
                                          key_bits, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);  // the temporaries are freed on return
        if (e != hipSuccess) {
            set_error("sort of the triple indices failed: %s", hipGetErrorString(e));
            return fail(LOGOSKG_EDEVICE);
        }
    }
    g->out_eid = eid;
    g->static_bytes += std::max<size_t>((size_t)T, 1) * 4;
    return LOGOSKG_OK;
}

}  // namespace lkg
