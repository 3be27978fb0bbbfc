// Graph index: destination-major CSR, compact (source, relation) pairs, (destination,
// relation) runs, the pair-major transpose and the work lists the kernels walk.
// Integer bookkeeping only.  Built once per graph (dataset preprocessing in the thesis,
// Ch.3 "Code Generation": transposition, COO -> CSR; Ch.3 "Compact Tensor Materialization
// and Data Layout": the (source node, edge type) -> row mapping, precomputed, CSR-like).
// The index arrays are produced on the device (graph_build.hip); this file derives the small
// work lists from their offset arrays on the host and holds the graph entry points of the ABI.
#include "rgnn_internal.h"

#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <algorithm>
#include <map>
#include <mutex>
#include <new>

namespace rgnn {

static thread_local char g_err[512] = "";
void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

rgnn_status_t allow_dynamic_lds(const void* kernel, size_t bytes) {
    static std::mutex mu;
    static std::map<std::pair<const void*, int>, size_t> done;   // (kernel, device) -> limit already set
    int dev = 0;
    RGNN_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(mu);
    size_t& have = done[{kernel, dev}];
    if (have >= bytes) return RGNN_OK;
    RGNN_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    have = bytes;
    return RGNN_OK;
}

rgnn_status_t resident_blocks_per_cu(const void* kernel, int threads, size_t lds, int* out) {
    static std::mutex mu;
    static std::map<std::pair<const void*, std::pair<int, size_t>>, int> done;   // (kernel, (device, lds)) -> blocks
    int dev = 0;
    RGNN_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(mu);
    auto key = std::make_pair(kernel, std::make_pair(dev, lds));
    auto it = done.find(key);
    if (it == done.end()) {
        int n = 0;
        RGNN_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, threads, lds));
        it = done.emplace(key, std::max(n, 1)).first;
    }
    *out = it->second;
    return RGNN_OK;
}

struct Uploader {
    rgnn_graph* g;
    rgnn_status_t st = RGNN_OK;
    template <typename Tv>
    Tv* up(const std::vector<Tv>& h) {
        if (st != RGNN_OK) return nullptr;
        void* d = nullptr;
        const size_t bytes = std::max<size_t>(h.size(), 1) * sizeof(Tv);
        hipError_t e = hipMalloc(&d, bytes);
        if (e != hipSuccess) {
            set_error("hipMalloc(%zu) failed: %s", bytes, hipGetErrorString(e));
            st = (e == hipErrorOutOfMemory) ? RGNN_ENOMEM : RGNN_EHIP;
            return nullptr;
        }
        g->allocs.push_back(d);
        g->index_bytes += bytes;
        if (!h.empty()) {
            e = hipMemcpy(d, h.data(), h.size() * sizeof(Tv), hipMemcpyHostToDevice);
            if (e != hipSuccess) {
                set_error("hipMemcpy H2D failed: %s", hipGetErrorString(e));
                st = RGNN_EHIP;
                return nullptr;
            }
        }
        return static_cast<Tv*>(d);
    }
    void idx(int which, const std::vector<int32_t>& h) {
        g->idx[which] = up(h);
        g->idx_len[which] = (int64_t)h.size();
    }
};

static void build_tiles(Uploader& U, TileList& t, const std::vector<int32_t>& seg_ptr, int tile_rows,
                        int max_chunks = kMaxChunks) {
    const TilePlan p = plan_tiles(seg_ptr, tile_rows, max_chunks);
    t.tile_rows = p.tile_rows; t.num_tiles = p.num_tiles; t.num_chunks = p.num_chunks; t.num_slots = p.num_slots;
    t.num_segs = p.num_segs;
    t.tile_seg = U.up(p.tile_seg); t.tile_row0 = U.up(p.tile_row0); t.tile_row1 = U.up(p.tile_row1);
    t.chunk_tile = U.up(p.chunk_tile); t.chunk_slot = U.up(p.chunk_slot); t.seg_slot_ptr = U.up(p.seg_slot_ptr);
}

static void build_items(Uploader& U, ItemList& L, const std::vector<int32_t>& ptr, int max_len, int min_len = 0) {
    const ItemPlan p = plan_items(ptr, max_len, min_len);
    L.num_items = (int32_t)p.beg.size(); L.num_partials = p.num_partials; L.num_split = p.num_split;
    L.first_single = p.first_single; L.num_single = p.num_single;
    L.first_short = p.first_short; L.num_short = p.num_short;
    L.beg = U.up(p.beg); L.end = U.up(p.end); L.row = U.up(p.row); L.slot = U.up(p.slot);
    L.split_row = U.up(p.split_row); L.split_ptr = U.up(p.split_ptr);
    L.part_item = U.up(p.part_item); L.part_split = U.up(p.part_split);
    L.num_long = (int32_t)p.long_item.size();
    L.long_item = U.up(p.long_item);
}

static void build_long(Uploader& U, LongList& L, const std::vector<int32_t>& ptr) {
    const std::vector<int32_t> ids = long_segments(ptr);
    L.n = (int)ids.size();
    L.ids = U.up(ids);
}

static rgnn_status_t download(std::vector<int32_t>& h, const int32_t* d, size_t n) {
    h.resize(n);
    if (n) RGNN_HIP(hipMemcpy(h.data(), d, n * sizeof(int32_t), hipMemcpyDeviceToHost));
    return RGNN_OK;
}

rgnn_status_t build_index_device(rgnn_graph* g, int format, const int32_t* a, const int32_t* b, const int32_t* relp,
                                 const int32_t* ntypep, const int32_t* rstp, const int32_t* rdtp, int mem);

static rgnn_status_t build(rgnn_graph* g, int format, const int32_t* a, const int32_t* b, const int32_t* relp,
                           const int32_t* ntypep, const int32_t* rstp, const int32_t* rdtp, int mem) {
    RGNN_TRY(build_index_device(g, format, a, b, relp, ntypep, rstp, rdtp, mem));
    // offsets back to the host: statistics and the work lists are cheap linear passes over them
    std::vector<int32_t> in_ptr, out_ptr, pair_ptr, relrun_ptr, srcpair_ptr, ntype_ptr, run_ptr;
    RGNN_TRY(download(in_ptr, g->idx[RGNN_IDX_IN_PTR], (size_t)g->N + 1));
    RGNN_TRY(download(out_ptr, g->idx[RGNN_IDX_OUT_PTR], (size_t)g->P + 1));
    RGNN_TRY(download(pair_ptr, g->idx[RGNN_IDX_PAIR_PTR], (size_t)g->R + 1));
    RGNN_TRY(download(relrun_ptr, g->idx[RGNN_IDX_RELRUN_PTR], (size_t)g->R + 1));
    RGNN_TRY(download(srcpair_ptr, g->idx[RGNN_IDX_SRCPAIR_PTR], (size_t)g->N + 1));
    RGNN_TRY(download(ntype_ptr, g->idx[RGNN_IDX_NTYPE_PTR], (size_t)g->T + 1));
    RGNN_TRY(download(run_ptr, g->idx[RGNN_IDX_RUN_PTR], (size_t)g->Q + 1));
    for (int64_t v = 0; v < g->N; ++v) g->max_in_degree = std::max<int64_t>(g->max_in_degree, in_ptr[v + 1] - in_ptr[v]);
    for (int64_t p = 0; p < g->P; ++p) {
        g->max_pair_out_degree = std::max<int64_t>(g->max_pair_out_degree, out_ptr[p + 1] - out_ptr[p]);
        g->num_single_pairs += (out_ptr[p + 1] - out_ptr[p] == 1);
    }
    Uploader U{g};
    build_tiles(U, g->pair_tiles, pair_ptr, kTileRows);
    build_tiles(U, g->node_tiles, ntype_ptr, kTileRows);
    build_tiles(U, g->all_tiles, std::vector<int32_t>{0, (int32_t)g->N}, kTileRows);
    int dev = 0, cus = 0;
    RGNN_HIP(hipGetDevice(&dev));
    RGNN_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    g->num_cus = std::max(cus, 1);
    const int wide = kWideChunksPerCU * std::max(cus, 1);
    build_tiles(U, g->pair_tiles_wide, pair_ptr, kTileRows, wide);
    build_tiles(U, g->node_tiles_wide, ntype_ptr, kTileRows, wide);
    build_items(U, g->dst_items, in_ptr, item_cut(g->E));
    build_items(U, g->pair_items, out_ptr, item_cut(g->E));
    build_items(U, g->relrun_items, relrun_ptr, item_cut(g->E));
    build_items(U, g->pair_items_multi, out_ptr, item_cut(g->E), 2);
    build_items(U, g->relpair_items, pair_ptr, item_cut(g->P));
    build_items(U, g->srcpair_items, srcpair_ptr, 1 << 30);
    build_long(U, g->long_runs, run_ptr);
    build_long(U, g->long_pairs, out_ptr);
    return U.st;
}

}  // namespace rgnn

using namespace rgnn;

extern "C" const char* rgnn_last_error(void) { return g_err; }

extern "C" rgnn_status_t rgnn_graph_create(rgnn_graph_t** gout, int64_t num_nodes, int32_t num_ntypes, int32_t num_rels,
                                           int64_t num_edges, int32_t format, const int32_t* a, const int32_t* b,
                                           const int32_t* rel, const int32_t* ntype, const int32_t* rel_src_ntype,
                                           const int32_t* rel_dst_ntype, int32_t mem) {
    if (!gout) RGNN_FAIL(RGNN_EINVAL, "g is NULL");
    *gout = nullptr;
    if (num_nodes < 0 || num_edges < 0 || num_rels < 1 || num_ntypes < 1)
        RGNN_FAIL(RGNN_EINVAL, "need num_nodes >= 0, num_edges >= 0, num_rels >= 1, num_ntypes >= 1");
    if (format != RGNN_COO && format != RGNN_CSR_DST) RGNN_FAIL(RGNN_EINVAL, "unknown format %d", format);
    if (mem != RGNN_MEM_HOST && mem != RGNN_MEM_DEVICE) RGNN_FAIL(RGNN_EINVAL, "unknown mem %d", mem);
    if (num_edges > 0 && (!a || !rel)) RGNN_FAIL(RGNN_EINVAL, "edge arrays are NULL");
    if ((format == RGNN_CSR_DST || num_edges > 0) && !b) RGNN_FAIL(RGNN_EINVAL, "dst / rowptr array is NULL");
    if (num_ntypes > 1 && !ntype) RGNN_FAIL(RGNN_EINVAL, "ntype is NULL but num_ntypes > 1");
    if ((rel_src_ntype == nullptr) != (rel_dst_ntype == nullptr))
        RGNN_FAIL(RGNN_EINVAL, "rel_src_ntype and rel_dst_ntype must be given together");
    if (num_edges >= (int64_t)1 << 31 || num_nodes >= (int64_t)1 << 31)
        RGNN_FAIL(RGNN_EUNSUPPORTED, "int32 indices: need fewer than 2^31 nodes and edges");
    {
        const long double bound = (long double)std::max<int64_t>(num_nodes, 1) * std::max<int64_t>(num_nodes, 1) * num_rels;
        if (bound >= 9.2e18L) RGNN_FAIL(RGNN_EUNSUPPORTED, "N*N*R must be below 2^63 for the 64-bit sort keys");
    }
    {   // set-up work for the entry point that allocates nothing: its scratch buffer's address on this device
        void* scratch_ptr = nullptr;
        RGNN_TRY(static_scratch(&scratch_ptr));
    }
    rgnn_graph* g = new (std::nothrow) rgnn_graph();
    if (!g) RGNN_FAIL(RGNN_ENOMEM, "out of host memory");
    g->N = num_nodes; g->E = num_edges; g->R = num_rels; g->T = num_ntypes;
    rgnn_status_t st;
    try {
        st = build(g, format, a, b, rel, ntype, ntype ? rel_src_ntype : nullptr, ntype ? rel_dst_ntype : nullptr, mem);
    } catch (const std::bad_alloc&) {
        set_error("out of host memory while building the graph index");
        st = RGNN_ENOMEM;
    }
    if (st == RGNN_OK && hipDeviceSynchronize() != hipSuccess) { set_error("hipDeviceSynchronize failed"); st = RGNN_EHIP; }
    if (st != RGNN_OK) { rgnn_graph_destroy(g); return st; }
    *gout = g;
    return RGNN_OK;
}

extern "C" rgnn_status_t rgnn_graph_destroy(rgnn_graph_t* g) {
    if (!g) return RGNN_OK;
    for (void* p : g->allocs) (void)hipFree(p);
    delete g;
    return RGNN_OK;
}

extern "C" rgnn_status_t rgnn_graph_info(const rgnn_graph_t* g, rgnn_graph_info_t* out) {
    if (!g || !out) RGNN_FAIL(RGNN_EINVAL, "NULL argument");
    out->num_nodes = g->N; out->num_edges = g->E; out->num_pairs = g->P; out->num_runs = g->Q;
    out->max_in_degree = g->max_in_degree; out->max_pair_out_degree = g->max_pair_out_degree;
    out->index_bytes = (int64_t)g->index_bytes; out->num_rels = g->R; out->num_ntypes = g->T;
    out->num_single_pairs = g->num_single_pairs;
    return RGNN_OK;
}

extern "C" rgnn_status_t rgnn_graph_export(const rgnn_graph_t* g, int32_t which, void* host_dst, size_t bytes) {
    if (!g || (!host_dst && bytes)) RGNN_FAIL(RGNN_EINVAL, "NULL argument");
    if (which < 0 || which >= RGNN_IDX_COUNT) RGNN_FAIL(RGNN_EINVAL, "unknown index array %d", which);
    if (bytes != (size_t)g->idx_len[which] * sizeof(int32_t))
        RGNN_FAIL(RGNN_EINVAL, "index array %d holds %lld int32, caller passed %zu bytes", which, (long long)g->idx_len[which], bytes);
    RGNN_HIP(hipDeviceSynchronize());
    if (bytes) RGNN_HIP(hipMemcpy(host_dst, g->idx[which], bytes, hipMemcpyDeviceToHost));
    return RGNN_OK;
}
