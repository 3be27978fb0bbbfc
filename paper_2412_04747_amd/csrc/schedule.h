// Per-graph, per-layer choice of schedule and layout: which of the alternative kernels and data
// layouts a layer call uses, decided from the statistics of the graph index and the layer
// descriptor (the thesis' point that no single schedule / layout fits every graph, Ch.3 "Compact
// Tensor Materialization and Data Layout" and the evaluation's per-dataset comparison of the
// optimizations).  Plain C++, no device code: layers.hip and the traversal launchers call these
// predicates where they pick a kernel, rgnn_schedule reports them, and the host tests exercise
// this header on its own.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include "../../include/rgnn.h"

namespace rgnn {

// A list of segments gets a batched walk of its single-entry (2..4-entry) whole segments only when it holds
// this many of them: below that the extra kernel phase costs more than the general walk loses on them.
constexpr int kBatchedMin = 4096;
// w_s of single-head RGAT (R x d fp32) stays in LDS for the fused traversal up to this size; beyond it the
// walks read it through the caches.
constexpr size_t kWsLdsMax = 64 * 1024;

inline bool flag_set(uint32_t flags, uint32_t bit) { return (flags & bit) != 0; }

// number of whole segments of one kind the batched walk takes (0: they stay with the general walk)
inline int batched_count(int count, uint32_t flags) {
    return (!flag_set(flags, RGNN_FLAG_NO_BATCHED_WALKS) && count >= kBatchedMin) ? count : 0;
}
// bf16 inputs at width 128: every row tensor (inputs, intermediates, saved tensors, incoming gradients) is bf16 storage
inline bool sched_rows_bf16(int dtype, int d) { return dtype == RGNN_BF16 && d == 128; }
// The gradient row of a (source, relation) pair with one edge is not materialised: the typed-linear backward reads
// it from the destination's gradient row through a row selector.  Built for RGAT up to width 64 with one, two or
// four heads (the fused fp32 backward kernel) and for RGCN with bf16 rows.
inline bool sched_row_select(int layer, int dtype, int d, int heads, uint32_t flags) {
    if (flag_set(flags, RGNN_FLAG_NO_ROW_SELECT)) return false;
    if (layer == RGNN_LAYER_RGAT) return d <= 64 && (heads == 1 || ((heads == 2 || heads == 4) && d % (4 * heads) == 0));
    if (layer == RGNN_LAYER_RGCN) return sched_rows_bf16(dtype, d);
    return false;
}
// HGT: the key and message linears of the nodes are folded into the per-relation weights when every relation's
// sources have one node type.
inline bool sched_hgt_folded(bool rel_src_tied, uint32_t flags) {
    return rel_src_tied && !flag_set(flags, RGNN_FLAG_NO_WEIGHT_FOLDING);
}
// RGAT: edge softmax fused into the aggregation walk (otherwise, one head only, a pass of its own that stores one
// attention weight per edge); the edge-parallel comparison schedule needs the per-edge weights
inline bool sched_fused_softmax(uint32_t flags) {
    return !flag_set(flags, RGNN_FLAG_SEPARATE_SOFTMAX) && !flag_set(flags, RGNN_FLAG_EDGE_PARALLEL_AGGREGATION);
}
inline bool sched_ws_in_lds(int R, int d) { return (size_t)R * d * sizeof(float) <= kWsLdsMax; }

struct ListCounts { int32_t single = 0, short_ = 0; };   // whole segments with 1 / with 2..kShortLen entries
struct ScheduleIn {
    int layer = 0, dtype = 0, d = 0, heads = 1;
    uint32_t flags = 0;
    int R = 1;
    bool rel_src_tied = false;
    int item_len = 0, tile_chunks = 0, wide_chunks = 0;
    ListCounts dst, pair, pair_multi;     // destination-major list, pair-major list, pair-major list of multi-edge pairs
};

inline rgnn_schedule_t pick_schedule(const ScheduleIn& in) {
    rgnn_schedule_t s{};
    s.item_len = in.item_len;
    s.tile_chunks = in.tile_chunks;
    s.wide_chunks = in.wide_chunks;
    s.rows_bf16 = sched_rows_bf16(in.dtype, in.d) && in.layer != RGNN_LAYER_RGAT;
    s.row_select = sched_row_select(in.layer, in.dtype, in.d, in.heads, in.flags);
    s.hgt_folded = in.layer == RGNN_LAYER_HGT && sched_hgt_folded(in.rel_src_tied, in.flags);
    s.fused_softmax = in.layer == RGNN_LAYER_RGAT && sched_fused_softmax(in.flags);
    s.ws_in_lds = s.fused_softmax && sched_ws_in_lds(in.R, in.d);
    s.edge_parallel = in.layer == RGNN_LAYER_RGAT && flag_set(in.flags, RGNN_FLAG_EDGE_PARALLEL_AGGREGATION);
    s.dst_batched_single = batched_count(in.dst.single, in.flags) > 0;
    s.dst_batched_short = batched_count(in.dst.short_, in.flags) > 0;
    // the pair-major backward walk runs over the multi-edge pairs only where the row selector (or, for single-head
    // RGAT, the edge walk itself) serves the single-edge pairs
    const bool multi_only = s.row_select || (in.layer == RGNN_LAYER_RGAT && in.heads == 1);
    const ListCounts& pl = multi_only ? in.pair_multi : in.pair;
    s.pair_batched_single = batched_count(pl.single, in.flags) > 0;
    s.pair_batched_short = batched_count(pl.short_, in.flags) > 0;
    s.pair_walk_multi_only = multi_only;
    return s;
}

}  // namespace rgnn
