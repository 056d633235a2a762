// Sharded graphs (paper Sec. 3.4, Algorithm 1): placeholder until the shard
// cache is built; logoskg_build rejects num_shards > 1 through build_shards.
#include "common.h"

namespace lkg {

logoskg_status build_shards(logoskg_graph *, const int32_t *, const int32_t *, const int32_t *,
                            const logoskg_build_opts *) {
    set_error("sharded graphs are not available in this build");
    return LOGOSKG_EINVAL;
}

void free_shards(logoskg_graph *) {}

logoskg_status run_sharded_hop(logoskg_graph *, logoskg_result *, int, hipStream_t, logoskg_hop_stats *) {
    set_error("sharded graphs are not available in this build");
    return LOGOSKG_EINTERNAL;
}

}  // namespace lkg

using namespace lkg;

extern "C" logoskg_status logoskg_graph_get_info(const logoskg_graph *g, logoskg_graph_info *o) {
    if (!g || !o) { set_error("NULL argument"); return LOGOSKG_EINVAL; }
    memset(o, 0, sizeof(*o));
    o->num_triples = g->T;
    o->num_entities = g->E;
    o->num_relations = g->R;
    o->num_shards = g->num_shards;
    o->hub_min_degree = g->hub_min;
    o->num_out_rows = g->n_out_rows;
    o->num_out_hubs = g->n_out_hubs;
    o->num_in_rows = g->in_rows.n_tail + g->in_rows.n_long;
    o->num_in_hubs = g->in_rows.n_hub;
    o->device_bytes = (int64_t)(g->static_bytes + g->pool.bytes_held());
    o->pinned_host_bytes = (int64_t)g->pinned_bytes;
    return LOGOSKG_OK;
}

extern "C" logoskg_status logoskg_graph_partition(const logoskg_graph *g, int32_t *shard_of_entity,
                                                  int64_t *triples_per_shard) {
    if (!g) { set_error("NULL graph"); return LOGOSKG_EINVAL; }
    if (g->num_shards <= 1) {
        if (shard_of_entity) {
            std::vector<uint32_t> off((size_t)g->E + 1);
            LKG_HIP(hipMemcpy(off.data(), g->out_off, off.size() * 4, hipMemcpyDeviceToHost));
            for (int32_t e = 0; e < g->E; ++e) shard_of_entity[e] = off[(size_t)e + 1] > off[e] ? 0 : -1;
        }
        if (triples_per_shard) triples_per_shard[0] = g->T;
        return LOGOSKG_OK;
    }
    if (shard_of_entity) memcpy(shard_of_entity, g->shard_of.data(), (size_t)g->E * sizeof(int32_t));
    if (triples_per_shard)
        memcpy(triples_per_shard, g->shard_triples.data(), (size_t)g->num_shards * sizeof(int64_t));
    return LOGOSKG_OK;
}
