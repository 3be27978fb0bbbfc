// Graph index: destination-major CSR, compact (source, relation) pairs, (destination,
// relation) runs, the pair-major transpose and the work lists the kernels walk.
// Integer bookkeeping only.  Built once per graph (dataset preprocessing in the thesis,
// Ch.3 "Code Generation": transposition, COO -> CSR; Ch.3 "Compact Tensor Materialization
// and Data Layout": the (source node, edge type) -> row mapping, precomputed, CSR-like).
// The sorts run on the host with an LSD radix sort; the arrays then live on the device.
#include "rgnn_internal.h"

#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <algorithm>
#include <new>

namespace rgnn {

static thread_local char g_err[512] = "";
void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

// Stable LSD radix sort of (key, value) pairs by key, 8 bits per pass, over the
// significant bits only.
static void radix_sort_pairs(std::vector<uint64_t>& key, std::vector<uint32_t>& val, uint64_t max_key) {
    const size_t n = key.size();
    if (n < 2) return;
    int bits = 0;
    while (bits < 64 && (max_key >> bits) != 0) ++bits;
    std::vector<uint64_t> k2(n);
    std::vector<uint32_t> v2(n);
    for (int shift = 0; shift < bits; shift += 8) {
        size_t cnt[257] = {0};
        for (size_t i = 0; i < n; ++i) cnt[((key[i] >> shift) & 0xFF) + 1]++;
        for (int b = 0; b < 256; ++b) cnt[b + 1] += cnt[b];
        for (size_t i = 0; i < n; ++i) {
            const size_t p = cnt[(key[i] >> shift) & 0xFF]++;
            k2[p] = key[i];
            v2[p] = val[i];
        }
        key.swap(k2);
        val.swap(v2);
    }
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

// Tiles of `tile_rows` rows over segments seg_ptr[0..S], cut into chunks.
static void build_tiles(Uploader& U, TileList& t, const std::vector<int32_t>& seg_ptr, int tile_rows) {
    const int S = (int)seg_ptr.size() - 1;
    std::vector<int32_t> tseg, r0, r1;
    for (int s = 0; s < S; ++s)
        for (int32_t a = seg_ptr[s]; a < seg_ptr[s + 1]; a += tile_rows) {
            tseg.push_back(s);
            r0.push_back(a);
            r1.push_back(std::min<int32_t>(a + tile_rows, seg_ptr[s + 1]));
        }
    const int nt = (int)tseg.size();
    const int nc = std::min(nt, kMaxChunks);
    std::vector<int32_t> ctile(nc + 1, 0), cslot(std::max(nc, 1), 0), sslot(S + 1, 0);
    int slots = 0;
    std::vector<int32_t> seg_slots(S, 0);
    for (int c = 0; c < nc; ++c) {
        ctile[c] = (int32_t)((int64_t)nt * c / nc);
        ctile[c + 1] = (int32_t)((int64_t)nt * (c + 1) / nc);
        cslot[c] = slots;
        for (int i = ctile[c]; i < ctile[c + 1]; ++i)
            if (i == ctile[c] || tseg[i] != tseg[i - 1]) {
                ++slots;
                seg_slots[tseg[i]]++;
            }
    }
    for (int s = 0; s < S; ++s) sslot[s + 1] = sslot[s] + seg_slots[s];
    t.tile_rows = tile_rows;
    t.num_tiles = nt;
    t.num_chunks = nc;
    t.num_slots = slots;
    t.num_segs = S;
    t.tile_seg = U.up(tseg);
    t.tile_row0 = U.up(r0);
    t.tile_row1 = U.up(r1);
    t.chunk_tile = U.up(ctile);
    t.chunk_slot = U.up(cslot);
    t.seg_slot_ptr = U.up(sslot);
}

// Items of at most max_len entries over segments ptr[0..S].
// Segments shorter than `min_len` are left out (their owner handles them elsewhere).
static void build_items(Uploader& U, ItemList& L, const std::vector<int32_t>& ptr, int max_len, int min_len = 0) {
    const int S = (int)ptr.size() - 1;
    std::vector<int32_t> beg, end, row, slot, srow, sptr, pitem, psplit;
    sptr.push_back(0);
    int partials = 0;
    for (int s = 0; s < S; ++s) {
        const int32_t a = ptr[s], b = ptr[s + 1];
        if (b - a < min_len) continue;
        if (b - a <= max_len) {
            beg.push_back(a); end.push_back(b); row.push_back(s); slot.push_back(-1);
        } else {
            for (int32_t c = a; c < b; c += max_len) {
                pitem.push_back((int32_t)beg.size());
                psplit.push_back((int32_t)srow.size());
                beg.push_back(c); end.push_back(std::min<int32_t>(c + max_len, b));
                row.push_back(s); slot.push_back(partials++);
            }
            srow.push_back(s);
            sptr.push_back(partials);
        }
    }
    // Order the items by length, longest first (stable): the lanes of a wavefront and the
    // wavefronts of a workgroup then walk items of equal length and finish together, and the
    // long items are scheduled before the short ones fill the tail.
    {
        const int n = (int)beg.size();
        int longest = 0;
        for (int i = 0; i < n; ++i) longest = std::max(longest, end[i] - beg[i]);
        std::vector<int32_t> cnt(longest + 2, 0), perm(n), inv(n);
        for (int i = 0; i < n; ++i) cnt[longest - (end[i] - beg[i]) + 1]++;
        for (int l = 0; l <= longest; ++l) cnt[l + 1] += cnt[l];
        for (int i = 0; i < n; ++i) { const int p = cnt[longest - (end[i] - beg[i])]++; perm[p] = i; inv[i] = p; }
        auto apply = [&](std::vector<int32_t>& v) {
            std::vector<int32_t> t(n);
            for (int p = 0; p < n; ++p) t[p] = v[perm[p]];
            v.swap(t);
        };
        apply(beg); apply(end); apply(row); apply(slot);
        for (auto& it : pitem) it = inv[it];
    }
    L.num_items = (int)beg.size();
    L.num_partials = partials;
    L.num_split = (int)srow.size();
    L.beg = U.up(beg); L.end = U.up(end); L.row = U.up(row); L.slot = U.up(slot);
    L.split_row = U.up(srow); L.split_ptr = U.up(sptr);
    L.part_item = U.up(pitem); L.part_split = U.up(psplit);
    std::vector<int32_t> lng;
    for (int i = 0; i < L.num_items; ++i)
        if (end[i] - beg[i] > kSerialMax || slot[i] >= 0) lng.push_back(i);
    L.num_long = (int)lng.size();
    L.long_item = U.up(lng);
}

static void build_long(Uploader& U, LongList& L, const std::vector<int32_t>& ptr) {
    std::vector<int32_t> ids;
    for (size_t i = 0; i + 1 < ptr.size(); ++i)
        if (ptr[i + 1] - ptr[i] > kSerialMax) ids.push_back((int32_t)i);
    L.n = (int)ids.size();
    L.ids = U.up(ids);
}

template <typename Tv>
static rgnn_status_t fetch(std::vector<Tv>& h, const Tv* p, size_t n, int mem) {
    h.resize(n);
    if (n == 0) return RGNN_OK;
    if (mem == RGNN_MEM_DEVICE) RGNN_HIP(hipMemcpy(h.data(), p, n * sizeof(Tv), hipMemcpyDeviceToHost));
    else memcpy(h.data(), p, n * sizeof(Tv));
    return RGNN_OK;
}

static rgnn_status_t build(rgnn_graph* g, int format, const int32_t* a, const int32_t* b, const int32_t* relp,
                           const int32_t* ntypep, const int32_t* rstp, const int32_t* rdtp, int mem) {
    const int64_t N = g->N, E = g->E;
    const int32_t R = g->R, T = g->T;
    std::vector<int32_t> src, dst, rel, ntype, rst, rdt;
    RGNN_TRY(fetch(src, a, (size_t)E, mem));
    RGNN_TRY(fetch(rel, relp, (size_t)E, mem));
    if (format == RGNN_COO) {
        RGNN_TRY(fetch(dst, b, (size_t)E, mem));
    } else {
        std::vector<int32_t> rp;
        RGNN_TRY(fetch(rp, b, (size_t)N + 1, mem));
        if (rp[0] != 0 || rp[N] != E) RGNN_FAIL(RGNN_EINVAL, "CSR rowptr must start at 0 and end at num_edges");
        dst.resize((size_t)E);
        for (int64_t v = 0; v < N; ++v) {
            if (rp[v + 1] < rp[v]) RGNN_FAIL(RGNN_EINVAL, "CSR rowptr is not monotone at row %lld", (long long)v);
            for (int32_t e = rp[v]; e < rp[v + 1]; ++e) dst[e] = (int32_t)v;
        }
    }
    if (ntypep) RGNN_TRY(fetch(ntype, ntypep, (size_t)N, mem));
    else ntype.assign((size_t)N, 0);
    for (int64_t n = 0; n < N; ++n)
        if (ntype[n] < 0 || ntype[n] >= T) RGNN_FAIL(RGNN_EINVAL, "ntype[%lld] = %d out of range [0, %d)", (long long)n, ntype[n], T);
    if (rstp) {
        RGNN_TRY(fetch(rst, rstp, (size_t)R, mem));
        RGNN_TRY(fetch(rdt, rdtp, (size_t)R, mem));
    }
    for (int64_t e = 0; e < E; ++e) {
        if (src[e] < 0 || src[e] >= N || dst[e] < 0 || dst[e] >= N || rel[e] < 0 || rel[e] >= R)
            RGNN_FAIL(RGNN_EINVAL, "edge %lld = (%d -> %d, rel %d) out of range (N = %lld, R = %d)", (long long)e,
                      src[e], dst[e], rel[e], (long long)N, R);
        if (rstp && (ntype[src[e]] != rst[rel[e]] || ntype[dst[e]] != rdt[rel[e]]))
            RGNN_FAIL(RGNN_EINVAL, "edge %lld: node types (%d -> %d) do not match relation %d's (%d -> %d)",
                      (long long)e, ntype[src[e]], ntype[dst[e]], rel[e], rst[rel[e]], rdt[rel[e]]);
    }

    Uploader U{g};
    const uint64_t uN = (uint64_t)std::max<int64_t>(N, 1), uR = (uint64_t)std::max<int32_t>(R, 1);

    // 1. CSR order: (dst, rel, src, input id)
    std::vector<uint64_t> key((size_t)E);
    std::vector<uint32_t> val((size_t)E);
    for (int64_t e = 0; e < E; ++e) {
        key[e] = ((uint64_t)dst[e] * uR + (uint64_t)rel[e]) * uN + (uint64_t)src[e];
        val[e] = (uint32_t)e;
    }
    radix_sort_pairs(key, val, uN * uR * uN);
    std::vector<int32_t> in_ptr((size_t)N + 1, 0), in_src((size_t)E), in_rel((size_t)E), in_dst((size_t)E), in_eid((size_t)E);
    for (int64_t i = 0; i < E; ++i) {
        const int32_t e = (int32_t)val[i];
        in_eid[i] = e; in_src[i] = src[e]; in_rel[i] = rel[e]; in_dst[i] = dst[e];
        in_ptr[dst[e] + 1]++;
    }
    for (int64_t v = 0; v < N; ++v) in_ptr[v + 1] += in_ptr[v];
    for (int64_t v = 0; v < N; ++v) g->max_in_degree = std::max<int64_t>(g->max_in_degree, in_ptr[v + 1] - in_ptr[v]);

    // 2. pairs: CSR positions sorted by ((rel, src), position); the sorted order is the
    //    pair-major transpose, the distinct keys in order are the pairs.
    for (int64_t i = 0; i < E; ++i) {
        key[i] = (uint64_t)in_rel[i] * uN + (uint64_t)in_src[i];
        val[i] = (uint32_t)i;
    }
    radix_sort_pairs(key, val, uR * uN);
    std::vector<int32_t> in_pair((size_t)E), out_epos((size_t)E), out_dst((size_t)E), pair_src, pair_rel, out_ptr;
    std::vector<int32_t> pair_ptr((size_t)R + 1, 0);
    for (int64_t i = 0; i < E; ++i) {
        if (i == 0 || key[i] != key[i - 1]) {
            pair_src.push_back((int32_t)(key[i] % uN));
            pair_rel.push_back((int32_t)(key[i] / uN));
            pair_ptr[pair_rel.back() + 1]++;
            out_ptr.push_back((int32_t)i);
        }
        in_pair[val[i]] = (int32_t)pair_src.size() - 1;
        out_epos[i] = (int32_t)val[i];
        out_dst[i] = in_dst[val[i]];
    }
    out_ptr.push_back((int32_t)E);
    const int64_t P = (int64_t)pair_src.size();
    g->P = P;
    for (int32_t r = 0; r < R; ++r) pair_ptr[r + 1] += pair_ptr[r];
    for (int64_t p = 0; p < P; ++p)
        g->max_pair_out_degree = std::max<int64_t>(g->max_pair_out_degree, out_ptr[p + 1] - out_ptr[p]);

    // 3. runs of equal (dst, rel) in CSR order
    std::vector<int32_t> in_run((size_t)E), in_cnt((size_t)E), run_ptr, run_dst, run_rel, dst_run_ptr((size_t)N + 1, 0);
    for (int64_t i = 0; i < E; ++i) {
        if (i == 0 || in_dst[i] != in_dst[i - 1] || in_rel[i] != in_rel[i - 1]) {
            run_ptr.push_back((int32_t)i);
            run_dst.push_back(in_dst[i]);
            run_rel.push_back(in_rel[i]);
            dst_run_ptr[in_dst[i] + 1]++;
        }
        in_run[i] = (int32_t)run_dst.size() - 1;
    }
    run_ptr.push_back((int32_t)E);
    const int64_t Q = (int64_t)run_dst.size();
    g->Q = Q;
    for (int64_t v = 0; v < N; ++v) dst_run_ptr[v + 1] += dst_run_ptr[v];
    std::vector<float> in_invc((size_t)E);
    for (int64_t i = 0; i < E; ++i) {
        in_cnt[i] = run_ptr[in_run[i] + 1] - run_ptr[in_run[i]];
        in_invc[i] = 1.0f / (float)in_cnt[i];
    }

    // 4. runs sorted by (rel, dst)
    key.resize((size_t)Q); val.resize((size_t)Q);
    for (int64_t q = 0; q < Q; ++q) { key[q] = (uint64_t)run_rel[q] * uN + (uint64_t)run_dst[q]; val[q] = (uint32_t)q; }
    radix_sort_pairs(key, val, uR * uN);
    std::vector<int32_t> relrun_idx((size_t)Q), relrun_ptr((size_t)R + 1, 0);
    for (int64_t i = 0; i < Q; ++i) { relrun_idx[i] = (int32_t)val[i]; relrun_ptr[run_rel[val[i]] + 1]++; }
    for (int32_t r = 0; r < R; ++r) relrun_ptr[r + 1] += relrun_ptr[r];

    // 5. pairs sorted by (src, rel)
    key.resize((size_t)P); val.resize((size_t)P);
    for (int64_t p = 0; p < P; ++p) { key[p] = (uint64_t)pair_src[p] * uR + (uint64_t)pair_rel[p]; val[p] = (uint32_t)p; }
    radix_sort_pairs(key, val, uN * uR);
    std::vector<int32_t> srcpair_idx((size_t)P), srcpair_ptr((size_t)N + 1, 0);
    for (int64_t i = 0; i < P; ++i) { srcpair_idx[i] = (int32_t)val[i]; srcpair_ptr[pair_src[val[i]] + 1]++; }
    for (int64_t v = 0; v < N; ++v) srcpair_ptr[v + 1] += srcpair_ptr[v];

    // 6. nodes sorted by (type, id): counting sort
    std::vector<int32_t> ntype_ptr((size_t)T + 1, 0), ntype_perm((size_t)N);
    for (int64_t n = 0; n < N; ++n) ntype_ptr[ntype[n] + 1]++;
    for (int32_t t = 0; t < T; ++t) ntype_ptr[t + 1] += ntype_ptr[t];
    {
        std::vector<int32_t> fill(ntype_ptr.begin(), ntype_ptr.end() - 1);
        for (int64_t n = 0; n < N; ++n) ntype_perm[fill[ntype[n]]++] = (int32_t)n;
    }

    U.idx(RGNN_IDX_IN_PTR, in_ptr);       U.idx(RGNN_IDX_IN_SRC, in_src);     U.idx(RGNN_IDX_IN_REL, in_rel);
    U.idx(RGNN_IDX_IN_EID, in_eid);       U.idx(RGNN_IDX_IN_PAIR, in_pair);   U.idx(RGNN_IDX_IN_RUN, in_run);
    U.idx(RGNN_IDX_IN_CNT, in_cnt);       U.idx(RGNN_IDX_PAIR_PTR, pair_ptr); U.idx(RGNN_IDX_PAIR_SRC, pair_src);
    U.idx(RGNN_IDX_PAIR_REL, pair_rel);   U.idx(RGNN_IDX_RUN_PTR, run_ptr);   U.idx(RGNN_IDX_RUN_DST, run_dst);
    U.idx(RGNN_IDX_RUN_REL, run_rel);     U.idx(RGNN_IDX_DST_RUN_PTR, dst_run_ptr);
    U.idx(RGNN_IDX_RELRUN_PTR, relrun_ptr); U.idx(RGNN_IDX_RELRUN_IDX, relrun_idx);
    U.idx(RGNN_IDX_OUT_PTR, out_ptr);     U.idx(RGNN_IDX_OUT_EPOS, out_epos); U.idx(RGNN_IDX_OUT_DST, out_dst);
    U.idx(RGNN_IDX_SRCPAIR_PTR, srcpair_ptr); U.idx(RGNN_IDX_SRCPAIR_IDX, srcpair_idx);
    U.idx(RGNN_IDX_NTYPE_PTR, ntype_ptr); U.idx(RGNN_IDX_NTYPE_PERM, ntype_perm);
    g->in_invc = U.up(in_invc);

    // 7. work lists
    build_tiles(U, g->pair_tiles, pair_ptr, kTileRows);
    build_tiles(U, g->node_tiles, ntype_ptr, kTileRows);
    build_tiles(U, g->all_tiles, std::vector<int32_t>{0, (int32_t)N}, kTileRows);
    build_items(U, g->dst_items, in_ptr, kItemMax);
    build_items(U, g->pair_items, out_ptr, kItemMax);
    build_items(U, g->relrun_items, relrun_ptr, kItemMax);
    build_items(U, g->pair_items_multi, out_ptr, kItemMax, 2);
    build_items(U, g->srcpair_items, srcpair_ptr, 1 << 30);
    {   // CSR edge -> pair id, with the top bit set when the pair has this edge only
        std::vector<int32_t> tag((size_t)E);
        for (int64_t i = 0; i < E; ++i) {
            const int32_t p = in_pair[i];
            tag[i] = (out_ptr[p + 1] - out_ptr[p] == 1) ? (int32_t)((uint32_t)p | 0x80000000u) : p;
        }
        g->in_pair_tag = U.up(tag);
    }
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
    rgnn_graph* g = new (std::nothrow) rgnn_graph();
    if (!g) RGNN_FAIL(RGNN_ENOMEM, "out of host memory");
    g->N = num_nodes; g->E = num_edges; g->R = num_rels; g->T = num_ntypes;
    rgnn_status_t st;
    try {
        st = build(g, format, a, b, rel, ntype, rel_src_ntype, rel_dst_ntype, mem);
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
