// Internal layout of fc_graph, shared by the host-side ingest (fc_host.cpp) and the
// device side (fc_device.hip).  Not part of the public ABI.
#pragma once
#include <cstdint>
#include <vector>

#include "fc_maxflow.h"

struct fc_graph {
    // ---- host side (always valid)
    int32_t n = 0;                 // |V| (super-source excluded)
    int32_t N = 0;                 // |V_c|
    int64_t m0 = 0;                // topology arcs after merging parallels
    std::vector<int32_t> row_ptr;  // [n+1] residual CSR offsets
    std::vector<int32_t> other;    // [2*m0] other endpoint of the residual arc
    std::vector<int32_t> pair;     // [2*m0] merged topology arc the record belongs to
    std::vector<int32_t> bw;       // [2*m0] bandwidth b_e of that topology arc
    std::vector<uint8_t> fwd;      // [2*m0] 1: topology arc leaves the row's vertex
    std::vector<uint8_t> is_compute;   // [n]
    std::vector<int32_t> compute_ids;  // [N] increasing
    std::vector<int32_t> in_bw;        // [n] in-bandwidth B^-(v) of every vertex
    int64_t sum_bw = 0;                // sum of all link bandwidths
    std::vector<int32_t> src_weight;   // [n] m_c of the non-uniform variant (0 for switches); empty: every compute node 1
    int64_t sum_w = 0;                 // sum of the weights; N while they are uniform
    int64_t min_in_bw = 0;         // min over compute nodes of B^-(v)
    int32_t max_bw = 0, gcd_bw = 0, eulerian = 0;
    int32_t max_row = 0;           // longest residual row
    double row_seen = 0;           // sum of squared row lengths / sum of row lengths: the length of the row a random record lies in
    // ---- device side (valid when on_device)
    bool on_device = false;
    int device = -1;
    int32_t *d_row_ptr = nullptr;      // [n+1]
    void *d_arc_wide = nullptr;        // int4 [2*m0]: {other, pair, bw, fwd}
    void *d_arc_compact = nullptr;     // uint2 [2*m0]: {other | fwd<<15 | pair<<16, bw}; null if ids do not fit 15 bits
    uint8_t *d_is_compute = nullptr;   // [n]
    int32_t *d_compute_ids = nullptr;  // [N]
    int32_t *d_in_bw = nullptr;        // [n]
    int32_t *d_src_weight = nullptr;   // [n], or null while the weights are uniform
    uint32_t *d_sink_cost = nullptr;   // [n] cost of the last problem solved per sink (scheduling hint, updated by the solver)
    uint16_t *d_labels = nullptr;      // [n*n] exact initial labels per sink (row = sink), bit 15 = compute; or null
    uint16_t *d_label_hmax = nullptr;  // [n] highest finite label of a compute node, per sink
    void *d_p1 = nullptr;              // uint4 [n*n] first-pass entries in level order, per sink (null: not built)
    uint16_t *d_level_off = nullptr;   // [n*64] level boundaries in d_p1, per sink
    int32_t *d_tree_ratio = nullptr;   // [n*2] per sink: worst load/bandwidth ratio of its first-arc tree (with d_p1); then [n]: sink too deep for the level table
    int32_t lds_limit = 0;             // bytes of LDS one workgroup may use
    int32_t n_cu = 0;
    // The per-sink tables describe the bandwidths they were built from.  fc_graph_update_arcs either rebuilds them or
    // marks them unusable; launches then start every problem with a search for heights in the kernel instead.
    bool labels_valid = false;         // d_labels / d_label_hmax may be used
    bool p1_valid = false;             // d_p1 / d_level_off / d_tree_ratio may be used
    void *d_edits = nullptr;           // int2 [edits_cap] {record, bandwidth}: staging for fc_graph_update_arcs
    size_t edits_cap = 0;
};

// host-only helpers implemented in fc_host.cpp
// keep_zero_links: an arc of bandwidth zero becomes a link that carries nothing (it has records and can be given
// bandwidth later) instead of being dropped
int fc_host_build(int32_t n_vertices, int64_t n_arcs, const int32_t *tail, const int32_t *head,
                  const int32_t *bandwidth, const uint8_t *is_compute, fc_graph **out, bool keep_zero_links = false);
// Set the bandwidth of existing links on the host side of g (records, in-bandwidths, the facts fc_graph_info reports).
// Either every update is applied or none; `edits` receives {record, new bandwidth} for both records of every link
// whose bandwidth changed.
int fc_host_update_arcs(fc_graph *g, int64_t n_updates, const int32_t *tail, const int32_t *head,
                        const int32_t *bandwidth, std::vector<int32_t> &edits);
