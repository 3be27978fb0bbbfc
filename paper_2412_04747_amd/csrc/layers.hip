// Layer entry points of the C ABI: argument checks, carving of the caller's workspace, and
// the sequence of kernel launches that makes up each layer.  No allocation, no
// synchronisation; everything is enqueued on the caller's stream.
#include "rgnn_internal.h"
#include "traversal.h"
#include "schedule.h"

#include <map>
#include <mutex>

using namespace rgnn;

namespace {

// Bump allocator over a caller-provided buffer; with base == nullptr it only measures.
struct Carver {
    char* base;
    size_t off = 0;
    explicit Carver(void* b) : base(static_cast<char*>(b)) {}
    template <typename Tv>
    Tv* take(size_t n) {
        Tv* p = base ? reinterpret_cast<Tv*>(base + off) : nullptr;
        off += align_up(std::max<size_t>(n, 1) * sizeof(Tv));
        return p;
    }
    // n elements of a row tensor stored as bf16 (half) or fp32
    void* rows(size_t n, bool half) { return half ? static_cast<void*>(take<uint16_t>(n)) : static_cast<void*>(take<float>(n)); }
};

// bfloat16 workloads at width 128 keep every row tensor (inputs, intermediates, saved tensors,
// incoming gradients) in bf16 storage and run the typed linears on the bf16 matrix cores; sums
// and products are fp32, results handed back to the caller are fp32.  At the other widths the
// bf16 inputs are widened once and the fp32 kernels run on the copies.
inline bool rows_bf16(const rgnn_layer_desc_t* d) { return d->dtype == RGNN_BF16 && d->d_out == 128; }

// bfloat16 inputs that an fp32 kernel consumes are widened to fp32 in a staging area that
// follows the regular carve-out of the workspace.
struct Bf16Stage {
    Carver c;
    bool on;
    hipStream_t st;
    rgnn_status_t status = RGNN_OK;
    Bf16Stage(void* ws, size_t carved, bool bf16, hipStream_t s)
        : c(ws ? static_cast<char*>(ws) + carved : nullptr), on(bf16), st(s) {}
    // returns the fp32 view of `p` (n elements): p itself for fp32 input, the widened copy for bf16
    const float* in(const void* p, size_t n) {
        if (!on || !p) return static_cast<const float*>(p);
        float* d = c.take<float>(n);
        if (c.base && status == RGNN_OK) status = widen_bf16(n, static_cast<const uint16_t*>(p), d, st);
        return d;
    }
    void reserve(size_t n) { if (on) (void)c.take<float>(n); }
};

// A [num_nodes, d] tensor may be NULL when the graph has no nodes.
inline bool missing(const rgnn_graph_t* g, const void* p) { return !p && g->N > 0; }

rgnn_status_t check_desc(const rgnn_graph_t* g, const rgnn_layer_desc_t* d, int layer) {
    if (!g || !d) RGNN_FAIL(RGNN_EINVAL, "graph or desc is NULL");
    if (d->flags & ~RGNN_FLAG_ALL) RGNN_FAIL(RGNN_EINVAL, "unknown bits in desc.flags");
    if ((d->flags & (RGNN_FLAG_EDGE_PARALLEL_AGGREGATION | RGNN_FLAG_SEPARATE_SOFTMAX)) && (layer != RGNN_LAYER_RGAT || d->heads != 1))
        RGNN_FAIL(RGNN_EUNSUPPORTED, "the edge-parallel aggregation and the separate softmax pass are schedules of single-head RGAT only");
    if (d->dtype != RGNN_F32 && d->dtype != RGNN_BF16) RGNN_FAIL(RGNN_EINVAL, "unknown dtype %d", d->dtype);
    // widths: 32, 64 or 128 on both sides; RGCN and RGAT with fp32 inputs also take 32 -> 64 and 64 -> 32
    const bool w_in = d->d_in == 32 || d->d_in == 64 || d->d_in == 128, w_out = d->d_out == 32 || d->d_out == 64 || d->d_out == 128;
    const bool mixed_ok = layer != RGNN_LAYER_HGT && d->dtype == RGNN_F32 && d->d_in <= 64 && d->d_out <= 64;
    if (!w_in || !w_out || (d->d_in != d->d_out && !mixed_ok))
        RGNN_FAIL(RGNN_EUNSUPPORTED, "need d_in == d_out in {32, 64, 128} (RGCN / RGAT with fp32 inputs: also 32 -> 64 and 64 -> 32), got %d -> %d",
                  d->d_in, d->d_out);
    if (layer == RGNN_LAYER_RGAT) {
        if (d->heads < 1 || d->d_out % d->heads != 0) RGNN_FAIL(RGNN_EINVAL, "heads must divide d_out");
        const int dh = d->d_out / d->heads;
        if (d->heads > 1 && dh != 16 && dh != 32 && dh != 64)
            RGNN_FAIL(RGNN_EUNSUPPORTED, "multi-head RGAT needs d_out / heads in {16, 32, 64}, got %d", dh);
        if (std::max<int64_t>(g->N, g->E) * d->heads > INT32_MAX)
            RGNN_FAIL(RGNN_EUNSUPPORTED, "multi-head RGAT needs num_nodes * heads and num_edges * heads < 2^31");
    }
    // with the widths and head widths allowed above the head count is a power of two; the kernels index with shifts
    if ((layer == RGNN_LAYER_RGAT || layer == RGNN_LAYER_HGT) && (d->heads & (d->heads - 1)))
        RGNN_FAIL(RGNN_EUNSUPPORTED, "the head count must be a power of two, got %d", d->heads);
    if (layer == RGNN_LAYER_RGAT && !(d->slope >= 0.f && d->slope <= 1.f))
        RGNN_FAIL(RGNN_EINVAL, "leaky-ReLU slope must be in [0, 1]");
    if (layer == RGNN_LAYER_RGCN) {
        if (d->norm != RGNN_NORM_NONE && d->norm != RGNN_NORM_IN_DEGREE_PER_REL) RGNN_FAIL(RGNN_EINVAL, "unknown norm %d", d->norm);
        if (d->activation != RGNN_ACT_NONE && d->activation != RGNN_ACT_RELU) RGNN_FAIL(RGNN_EINVAL, "unknown activation %d", d->activation);
    }
    if (layer == RGNN_LAYER_HGT) {
        if (d->heads < 1 || d->d_out % d->heads != 0) RGNN_FAIL(RGNN_EINVAL, "heads must divide d_out");
        const int dh = d->d_out / d->heads;
        if (dh != 16 && dh != 32 && dh != 64) RGNN_FAIL(RGNN_EUNSUPPORTED, "HGT needs d_out / heads in {16, 32, 64}, got %d", dh);
        if (std::max<int64_t>(g->N, g->E) * d->heads > INT32_MAX)
            RGNN_FAIL(RGNN_EUNSUPPORTED, "HGT needs num_nodes * heads and num_edges * heads < 2^31");
    }
    return RGNN_OK;
}

// ---- RGNN_FLAG_ACCUMULATE ---------------------------------------------------------------
// The input gradient is accumulated by the kernel that writes it (it reads the row it is about to store).  The
// parameter gradients are small and written by many different kernels, so under the flag they are formed in
// workspace buffers of their own and added to the caller's at the end of the call.
inline bool grads_accumulate(const rgnn_layer_desc_t* d) { return (d->flags & RGNN_FLAG_ACCUMULATE) != 0; }
struct GradAcc {
    static constexpr int kMax = 8;
    int n = 0;
    float* tmp[kMax];
    float* dst[kMax];
    size_t len[kMax];
    // where the backward pass is to write this gradient: the workspace buffer if there is one, else the caller's
    void* route(float* tmp_buf, void* dst_buf, size_t count) {
        if (!tmp_buf || !dst_buf) return dst_buf;
        tmp[n] = tmp_buf; dst[n] = static_cast<float*>(dst_buf); len[n] = count; ++n;
        return tmp_buf;
    }
    rgnn_status_t flush(hipStream_t st) const {
        for (int i = 0; i < n; ++i) RGNN_TRY(add_into(len[i], tmp[i], dst[i], st));
        return RGNN_OK;
    }
};

// ---- RGAT buffers -----------------------------------------------------------------------
// Hs, the destination halves of the logits per (run, head) and (max, sum) of every (destination, head) softmax.
struct RgatSaved { float* Hs; float* s_dst; float* ms; };
struct RgatFwdWs { float* wtp; float* s_src; float* att; float* part_m; float* part_s; float* part_ms; float* partial; };
struct RgatBwdWs {
    float* wtp; float* wsp; float* adz; float* ds_dst; float* ds_src; float* G; float* dXp; float* A; float* U;
    float* tl_part; float* partial;
    float* acc_dW; float* acc_dws; float* acc_dwt;      // RGNN_FLAG_ACCUMULATE: the parameter gradients of this call
};
// Single-head RGAT at widths up to 64: the gradient rows of single-edge pairs are not written per pair;
// the typed-linear backward reads att_e * dOut[dst_e] through its row selector.
inline bool rgat_row_select(const rgnn_layer_desc_t* d) { return sched_row_select(RGNN_LAYER_RGAT, d->dtype, d->d_out, d->heads, d->flags); }
inline bool rgat_edge_parallel(const rgnn_layer_desc_t* d) { return (d->flags & RGNN_FLAG_EDGE_PARALLEL_AGGREGATION) != 0; }
inline bool rgat_fused(const rgnn_layer_desc_t* d) { return sched_fused_softmax(d->flags); }

size_t carve_rgat_saved(const rgnn_graph_t* g, const rgnn_layer_desc_t* d, void* base, RgatSaved* s) {
    Carver c(base);
    s->Hs = c.take<float>((size_t)g->P * d->d_out);
    s->s_dst = c.take<float>((size_t)g->Q * d->heads);
    s->ms = c.take<float>(2 * (size_t)g->N * d->heads);
    return c.off;
}
size_t carve_rgat_fwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* d, void* base, RgatFwdWs* w) {
    Carver c(base);
    const size_t H = d->heads, parts = (size_t)g->dst_items.num_partials;
    w->wtp = c.take<float>(H * g->R * d->d_in);
    w->s_src = w->att = w->part_m = w->part_s = w->part_ms = nullptr;
    if (!rgat_fused(d)) {
        // the comparison schedules (one head): per-pair source logits, a softmax pass of its own, attention weights per edge
        w->s_src = c.take<float>((size_t)g->P);
        w->att = c.take<float>((size_t)g->E);
        w->part_m = c.take<float>(parts);
        w->part_s = c.take<float>(parts);
    } else {
        w->part_ms = c.take<float>(2 * parts * H);
    }
    w->partial = c.take<float>(parts * d->d_out);
    return c.off;
}
size_t carve_rgat_bwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* d, void* base, RgatBwdWs* w) {
    Carver c(base);
    const size_t H = d->heads;
    w->wtp = c.take<float>(H * g->R * d->d_in);
    w->wsp = c.take<float>((size_t)g->R * d->d_in);
    w->adz = c.take<float>((size_t)g->E * 2 * H);                    // per edge: att per head, then dz per head
    w->ds_dst = c.take<float>((size_t)g->Q * H);
    // with the row selector: (ds_src[p], att of the pair's only edge) interleaved, one pair of floats per p
    //   (several heads: 2 H floats per p, ds_src[p][0..H) then, for a pair with one edge, that edge's att[0..H))
    w->ds_src = c.take<float>(2 * (size_t)g->P * H);
    w->G = c.take<float>((size_t)g->P * d->d_out);
    w->dXp = c.take<float>((size_t)g->P * d->d_in);
    w->A = c.take<float>(H * g->R * d->d_in);
    w->U = c.take<float>(H * g->R * d->d_in);
    w->tl_part = c.take<float>(typed_linear_bwd_scratch_floats(d->d_in, d->d_out, g->pair_tiles, (int)H));
    const size_t parts = std::max<size_t>({(size_t)g->pair_items.num_partials, (size_t)g->relrun_items.num_partials,
                                           (size_t)g->relpair_items.num_partials});
    w->partial = c.take<float>(parts * std::max(d->d_in, d->d_out) * H);   // the run walk keeps one partial row per head
    const bool acc = grads_accumulate(d);
    w->acc_dW = acc ? c.take<float>((size_t)g->R * d->d_in * d->d_out) : nullptr;
    w->acc_dws = acc ? c.take<float>((size_t)g->R * d->d_out) : nullptr;
    w->acc_dwt = acc ? c.take<float>((size_t)g->R * d->d_out) : nullptr;
    return c.off;
}

// ---- RGCN buffers -----------------------------------------------------------------------
struct RgcnFwdWs { void* Hs; float* partial; };
struct RgcnBwdWs { void* dPre; float* dPre32; void* G; void* dXp; float* dX0; float* tl_part; float* partial; float* acc_dW; float* acc_dW0; };

size_t carve_rgcn_fwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* d, void* base, RgcnFwdWs* w) {
    Carver c(base);
    w->Hs = c.rows((size_t)g->P * d->d_out, rows_bf16(d));
    w->partial = c.take<float>((size_t)g->dst_items.num_partials * d->d_out);
    return c.off;
}
size_t carve_rgcn_bwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* d, void* base, RgcnBwdWs* w) {
    Carver c(base);
    const bool h = rows_bf16(d), relu = d->activation == RGNN_ACT_RELU;
    w->dPre = c.rows(relu ? (size_t)g->N * d->d_out : 0, h);
    w->dPre32 = c.take<float>(relu && h ? (size_t)g->N * d->d_out : 0);   // fp32 copy for the self-loop kernels
    w->G = c.rows((size_t)g->P * d->d_out, h);
    w->dXp = c.rows((size_t)g->P * d->d_in, h);
    w->dX0 = c.take<float>((size_t)g->N * d->d_in);
    w->tl_part = c.take<float>(std::max(typed_linear_bwd_scratch_floats(d->d_in, d->d_out, g->pair_tiles),
                                        typed_linear_bwd_scratch_floats(d->d_in, d->d_out, g->all_tiles)));
    w->partial = c.take<float>((size_t)g->pair_items.num_partials * d->d_out);
    const bool acc = grads_accumulate(d);
    w->acc_dW = acc ? c.take<float>((size_t)g->R * d->d_in * d->d_out) : nullptr;
    w->acc_dW0 = acc ? c.take<float>((size_t)d->d_in * d->d_out) : nullptr;
    return c.off;
}

// ---- HGT buffers ------------------------------------------------------------------------
// Row tensors (void*) are bf16 when rows_bf16(desc), fp32 otherwise.
// Folded path (the graph ties every relation to one source node type): the key and message linears
// of the nodes are folded into the per-relation weights (Wf = Wk[type] Watt[r], Wv[type] Wmsg[r]), so
// K, V and their gradients do not exist and the per-pair rows come straight from X.
inline bool hgt_folded(const rgnn_graph_t* g, const rgnn_layer_desc_t* d) { return sched_hgt_folded(g->rel_src_tied, d->flags); }
struct HgtSaved { void* K; void* Q; void* V; void* Z; void* Ka; void* M; float* att; };
struct HgtFwdWs { float* Wbd_att; float* Wbd_msg; float* Wf_att; float* Wf_msg; float* part_m; float* part_s; float* partial; };
struct HgtBwdWs {
    float* Wbd_att; float* Wbd_msg; float* dWbd_att; float* dWbd_msg; float* Wf_att; float* Wf_msg; float* dWf_att;
    float* dWf_msg; void* dZ; float* dl; void* dM; void* dKa;
    void* dQ; void* dKp; void* dVp; void* dK; void* dV; float* dXk; float* dXq; float* dXv; float* tl_part;
    float* partial;
    float* acc_node[4]; float* acc_rel[2]; float* acc_mu;     // RGNN_FLAG_ACCUMULATE: dWk, dWq, dWv, dWo; dWatt, dWmsg; dmu
};

size_t carve_hgt_saved(const rgnn_graph_t* g, const rgnn_layer_desc_t* d, void* base, HgtSaved* s) {
    Carver c(base);
    const bool h = rows_bf16(d);
    const size_t nd = (size_t)g->N * d->d_out, pd = (size_t)g->P * d->d_out, kv = hgt_folded(g, d) ? 0 : nd;
    s->K = c.rows(kv, h); s->Q = c.rows(nd, h); s->V = c.rows(kv, h); s->Z = c.rows(nd, h);
    s->Ka = c.rows(pd, h); s->M = c.rows(pd, h);
    s->att = c.take<float>((size_t)g->E * d->heads);
    return c.off;
}
size_t carve_hgt_fwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* d, void* base, HgtFwdWs* w) {
    Carver c(base);
    const size_t rdd = (size_t)g->R * d->d_out * d->d_out, fdd = hgt_folded(g, d) ? rdd : 0;
    w->Wbd_att = c.take<float>(rdd); w->Wbd_msg = c.take<float>(rdd);
    w->Wf_att = c.take<float>(fdd); w->Wf_msg = c.take<float>(fdd);
    w->part_m = c.take<float>((size_t)g->dst_items.num_partials * d->heads);
    w->part_s = c.take<float>((size_t)g->dst_items.num_partials * d->heads);
    w->partial = c.take<float>((size_t)g->dst_items.num_partials * d->d_out);
    return c.off;
}
size_t carve_hgt_bwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* d, void* base, HgtBwdWs* w) {
    Carver c(base);
    const bool h = rows_bf16(d);
    const bool fold = hgt_folded(g, d);
    const size_t D = d->d_out, rdd = (size_t)g->R * D * D, nd = (size_t)g->N * D, pd = (size_t)g->P * D;
    w->Wbd_att = c.take<float>(rdd); w->Wbd_msg = c.take<float>(rdd);
    w->dWbd_att = c.take<float>(rdd); w->dWbd_msg = c.take<float>(rdd);
    w->Wf_att = c.take<float>(fold ? rdd : 0); w->Wf_msg = c.take<float>(fold ? rdd : 0);
    w->dWf_att = c.take<float>(fold ? rdd : 0); w->dWf_msg = c.take<float>(fold ? rdd : 0);
    w->dZ = c.rows(nd, h); w->dl = c.take<float>((size_t)g->E * d->heads);
    w->dM = c.rows(pd, h); w->dKa = c.rows(pd, h); w->dQ = c.rows(nd, h);
    w->dKp = c.rows(pd, h); w->dVp = c.rows(pd, h);
    w->dK = c.rows(fold ? 0 : nd, h); w->dV = c.rows(fold ? 0 : nd, h);
    w->dXk = c.take<float>(h || fold ? 0 : nd); w->dXq = c.take<float>(h && !fold ? 0 : nd); w->dXv = c.take<float>(h || fold ? 0 : nd);
    w->tl_part = c.take<float>(std::max(typed_linear_bwd_scratch_floats(d->d_in, d->d_out, g->pair_tiles),
                                        typed_linear_bwd_scratch_floats(d->d_in, d->d_out, g->node_tiles)));
    w->partial = c.take<float>((size_t)std::max(g->pair_items.num_partials, g->dst_items.num_partials) * D);
    const bool acc = grads_accumulate(d);
    const size_t dh = D / d->heads;
    for (int i = 0; i < 4; ++i) w->acc_node[i] = acc ? c.take<float>((size_t)g->T * D * D) : nullptr;
    for (int i = 0; i < 2; ++i) w->acc_rel[i] = acc ? c.take<float>((size_t)g->R * d->heads * dh * dh) : nullptr;
    w->acc_mu = acc ? c.take<float>((size_t)g->R * d->heads) : nullptr;
    return c.off;
}

// Staging sizes: room for every tensor argument an entry point may widen (an upper bound at width 128,
// where most bf16 arguments are consumed as they are).
size_t stage_bytes(const rgnn_graph_t* g, int layer, const rgnn_layer_desc_t* d, bool bwd) {
    Bf16Stage s(nullptr, 0, d->dtype == RGNN_BF16, nullptr);
    const size_t N = g->N, R = g->R, T = g->T, di = d->d_in, dz = d->d_out;
    s.reserve(N * di);                                   // X
    if (layer == RGNN_LAYER_RGCN) { s.reserve(R * di * dz); s.reserve(di * dz); }
    if (layer == RGNN_LAYER_RGAT) { s.reserve(R * di * dz); s.reserve(R * dz); s.reserve(R * dz); }
    if (layer == RGNN_LAYER_HGT) {
        const size_t dh = dz / d->heads;
        for (int i = 0; i < 4; ++i) s.reserve(T * dz * dz);
        s.reserve(R * d->heads * dh * dh); s.reserve(R * d->heads * dh * dh); s.reserve(R * d->heads);
    }
    if (bwd) s.reserve(N * dz);                          // dOut
    return s.c.off;
}

// Inference calls (saved == NULL): the tensors a backward call would need are still intermediates of
// the forward, and live behind the forward scratch and the staging area in the workspace.
void* saved_or_scratch(const rgnn_graph_t* g, int layer, const rgnn_layer_desc_t* d, void* saved, void* workspace,
                       size_t fwd_carved) {
    if (saved) return saved;
    return static_cast<char*>(workspace) + align_up(fwd_carved + stage_bytes(g, layer, d, false));
}

// Forward typed linear  Y[g(i)] / Y[i] = A[g(i)] W[seg].  In bf16 mode it runs on the bf16 matrix
// cores: an operand whose bf16 form exists (A16 / W16) is used as is, an fp32-only one is split.
// y16: the output rows are stored as bf16 (width 128 only).
// Chunking: the bf16 kernel with the weight in bf16 does best on many short chunks (`tiles`); when
// the weight has to be split, and in the fp32 kernels, loading a segment's weight costs more and one
// resident round of long chunks (`wide`) wins.
// d_in (fp32 kernels only): width of the input rows when it differs from the output width d.
rgnn_status_t tl_fwd(bool bf16, const rgnn::TileList* tiles, const rgnn::TileList* wide, int d, const float* A32,
                     const void* A16, const int32_t* gather, int scatter, const float* W32, const void* W16, void* Y,
                     bool y16, const char* label, hipStream_t st, int d_in = 0) {
    if (d_in == 0) d_in = d;
    if (bf16) {
        if (d_in != d) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear on the bf16 matrix cores: equal widths only");
        TypedLinearBf16Args a{};
        a.tiles = W16 ? tiles : wide; a.A = A16 ? A16 : A32; a.a_bf16 = A16 != nullptr; a.gather = gather; a.scatter_out = scatter;
        a.W = W16 ? W16 : W32; a.w_bf16 = W16 != nullptr; a.Y = Y; a.y_bf16 = y16; a.label = label;
        return typed_linear_bf16(d, a, st);
    }
    TypedLinearArgs a{};
    a.tiles = wide; a.X = A32; a.gather = gather; a.W = W32; a.Y = static_cast<float*>(Y); a.scatter_out = scatter;
    a.label = label;
    return typed_linear_fwd(d_in, d, a, st);
}

// Backward typed linear: dXrow = dY W^T (rows through `gather` on both sides when `both_gathered`),
// dW = sum X^T dY.
//   rows16 (bf16 rows, width 128): X and dY are bf16; two kernels on the bf16 matrix cores (dY W^T with
//     the weight as is when its bf16 form W16 exists, split otherwise; X^T dY into per-chunk slots) and
//     the slot reduction.  dXrow is stored as bf16 (dx16) or fp32.
//   otherwise: the fused fp32 kernel on fp32 X, W, dY.
//   wide: the same tiles in fewer chunks, for the weight-gradient kernel;  dx_acc: dXrow += (fp32 dXrow, rows16)
//   ysel / y_alt (rows16, dY not gathered): row i of dY is dY[ysel[i]], or y_alt[ysel[i] & 0x7FFFFFFF] when the
//     top bit of ysel[i] is set; with yscale it is also multiplied by yscale[i]
rgnn_status_t tl_bwd(bool rows16, const rgnn::TileList* tiles, const rgnn::TileList* wide, int d, const void* X,
                     const int32_t* gather, int both_gathered, const float* W32, const void* W16, const void* dY,
                     void* dXrow, bool dx16, float* dW, float* part, const char* label, hipStream_t st,
                     bool dx_acc = false, const int32_t* ysel = nullptr, const void* y_alt = nullptr,
                     const float* yscale = nullptr, int d_in = 0) {
    if (d_in == 0) d_in = d;
    if (rows16 && d_in != d) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear backward on the bf16 matrix cores: equal widths only");
    if (ysel && (!rows16 || both_gathered)) RGNN_FAIL(RGNN_EUNSUPPORTED, "row selector: bf16 rows and ungathered dY only");
    if (rows16) {
        TypedLinearBf16Args a{};
        a.tiles = W16 ? tiles : wide; a.A = dY; a.a_bf16 = 1; a.gather = both_gathered ? gather : ysel; a.scatter_out = both_gathered;
        a.A_alt = y_alt; a.rowscale = ysel ? yscale : nullptr;
        a.W = W16 ? W16 : W32; a.w_bf16 = W16 != nullptr; a.transpose_w = 1; a.Y = dXrow; a.y_bf16 = dx16; a.accumulate = dx_acc; a.label = label;
        RGNN_TRY(typed_linear_bf16(d, a, st));
        TypedLinearWgradBf16Args w{};
        w.tiles = wide; w.X = X; w.gather = gather; w.dy_gathered = both_gathered; w.dY = dY; w.part = part;
        w.label = wgrad_label(label); w.ysel = ysel; w.dY_alt = y_alt; w.yscale = yscale;
        RGNN_TRY(typed_linear_wgrad_bf16(d, w, st));
        return typed_linear_slot_reduce(d, d, *wide, part, dW, nullptr, st);
    }
    if (dx_acc) RGNN_FAIL(RGNN_EUNSUPPORTED, "accumulating input gradient needs bf16 rows");
    TypedLinearBwdArgs b{};
    b.tiles = wide; b.X = static_cast<const float*>(X); b.gather = gather; b.W = W32; b.dY = static_cast<const float*>(dY);
    b.dy_gathered = both_gathered; b.dXrow = static_cast<float*>(dXrow); b.scatter_dx = both_gathered; b.dW = dW;
    b.part = part; b.label = label;
    return typed_linear_bwd(d_in, d, b, st);
}

}  // namespace

extern "C" rgnn_status_t rgnn_workspace_bytes(const rgnn_graph_t* g, int32_t layer, const rgnn_layer_desc_t* desc,
                                              size_t* fwd_workspace, size_t* bwd_workspace, size_t* saved) {
    if (layer != RGNN_LAYER_RGCN && layer != RGNN_LAYER_RGAT && layer != RGNN_LAYER_HGT)
        RGNN_FAIL(RGNN_EINVAL, "unknown layer %d", layer);
    RGNN_TRY(check_desc(g, desc, layer));
    size_t f = 0, b = 0, s = 0;
    if (layer == RGNN_LAYER_RGAT) {
        RgatFwdWs fw; RgatBwdWs bw; RgatSaved sv;
        f = carve_rgat_fwd(g, desc, nullptr, &fw);
        b = carve_rgat_bwd(g, desc, nullptr, &bw);
        s = carve_rgat_saved(g, desc, nullptr, &sv);
    } else if (layer == RGNN_LAYER_RGCN) {
        RgcnFwdWs fw; RgcnBwdWs bw;
        f = carve_rgcn_fwd(g, desc, nullptr, &fw);
        b = carve_rgcn_bwd(g, desc, nullptr, &bw);
        s = 0;
    } else {
        HgtFwdWs fw; HgtBwdWs bw; HgtSaved sv;
        f = carve_hgt_fwd(g, desc, nullptr, &fw);
        b = carve_hgt_bwd(g, desc, nullptr, &bw);
        s = carve_hgt_saved(g, desc, nullptr, &sv);
    }
    f += stage_bytes(g, layer, desc, false);
    b += stage_bytes(g, layer, desc, true);
    if (fwd_workspace) *fwd_workspace = f;
    if (bwd_workspace) *bwd_workspace = b;
    if (saved) *saved = s;
    return RGNN_OK;
}

extern "C" rgnn_status_t rgnn_schedule(const rgnn_graph_t* g, int32_t layer, const rgnn_layer_desc_t* desc, rgnn_schedule_t* out) {
    if (layer != RGNN_LAYER_RGCN && layer != RGNN_LAYER_RGAT && layer != RGNN_LAYER_HGT)
        RGNN_FAIL(RGNN_EINVAL, "unknown layer %d", layer);
    RGNN_TRY(check_desc(g, desc, layer));
    if (!out) RGNN_FAIL(RGNN_EINVAL, "out is NULL");
    ScheduleIn in;
    in.layer = layer; in.dtype = desc->dtype; in.d = desc->d_out; in.heads = layer == RGNN_LAYER_RGCN ? 1 : desc->heads;
    in.flags = desc->flags; in.R = g->R; in.rel_src_tied = g->rel_src_tied;
    in.item_len = item_cut(g->E); in.tile_chunks = g->pair_tiles.num_chunks; in.wide_chunks = g->pair_tiles_wide.num_chunks;
    in.dst = {g->dst_items.num_single, g->dst_items.num_short};
    in.pair = {g->pair_items.num_single, g->pair_items.num_short};
    in.pair_multi = {g->pair_items_multi.num_single, g->pair_items_multi.num_short};
    *out = pick_schedule(in);
    return RGNN_OK;
}

// =========================================================================== RGCN

extern "C" rgnn_status_t rgnn_rgcn_fwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X,
                                       const void* W, const void* W0, void* out, void* saved, void* workspace,
                                       void* stream) {
    (void)saved;
    RGNN_TRY(check_desc(g, desc, RGNN_LAYER_RGCN));
    ScheduleFlagsScope sched_scope(desc->flags);
    if (missing(g, X) || !W || missing(g, out)) RGNN_FAIL(RGNN_EINVAL, "X, W or out is NULL");
    if (!workspace) RGNN_FAIL(RGNN_EWORKSPACE, "workspace is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int D = desc->d_out;
    RgcnFwdWs w;
    const bool bf16 = desc->dtype == RGNN_BF16, h = rows_bf16(desc);
    const void* X16 = bf16 ? X : nullptr;
    const void* W16 = bf16 ? W : nullptr;
    Bf16Stage stg(workspace, carve_rgcn_fwd(g, desc, workspace, &w), bf16, st);
    // fp32 copies for the fp32 kernels: everything below width 128, only the self-loop operands at 128
    const float* X32 = (!h || W0) ? stg.in(X, (size_t)g->N * desc->d_in) : nullptr;
    const float* W32 = !h ? stg.in(W, (size_t)g->R * desc->d_in * D) : nullptr;
    const float* W032 = stg.in(W0, (size_t)desc->d_in * D);
    RGNN_TRY(stg.status);
    // 1. compact messages: Hs[p] = X[pair_src[p]] W[rel(p)]
    RGNN_TRY(tl_fwd(bf16, &g->pair_tiles, &g->pair_tiles_wide, D, X32, X16, g->idx[RGNN_IDX_PAIR_SRC], 0, W32, W16, w.Hs, h, "typed_linear_fwd", st,
                    desc->d_in));
    // 2. out[v] = sum_e (1/c) Hs[pair_e]
    const float* coef = desc->norm == RGNN_NORM_IN_DEGREE_PER_REL ? g->in_invc : nullptr;
    RGNN_TRY(gather_sum(g->dst_items, D, nullptr, g->idx[RGNN_IDX_IN_PAIR], 0, coef, 1, 0, w.Hs, out, w.partial, st, 0,
                        "aggregate_fwd", "aggregate_fwd.combine", 1, h, 0));
    // 3. self-loop: out += X W0
    if (W0) {
        TypedLinearArgs s{};
        s.tiles = &g->all_tiles; s.X = X32; s.W = W032;
        s.Y = static_cast<float*>(out); s.accumulate = 1; s.label = "self_loop_fwd";
        RGNN_TRY(typed_linear_fwd(desc->d_in, D, s, st));
    }
    if (desc->activation == RGNN_ACT_RELU) RGNN_TRY(relu_inplace((size_t)g->N * D, static_cast<float*>(out), st));
    return RGNN_OK;
}

extern "C" rgnn_status_t rgnn_rgcn_bwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X,
                                       const void* W, const void* W0, const void* out, const void* saved,
                                       const void* dOut, void* dX, void* dW, void* dW0, void* workspace,
                                       void* stream) {
    (void)saved;
    RGNN_TRY(check_desc(g, desc, RGNN_LAYER_RGCN));
    ScheduleFlagsScope sched_scope(desc->flags);
    if (missing(g, X) || !W || missing(g, dOut) || missing(g, dX) || !dW) RGNN_FAIL(RGNN_EINVAL, "a required tensor pointer is NULL");
    if (W0 && !dW0) RGNN_FAIL(RGNN_EINVAL, "dW0 is NULL but W0 is given");
    if (desc->activation != RGNN_ACT_NONE && missing(g, out)) RGNN_FAIL(RGNN_EINVAL, "out is needed for the activation's gradient");
    if (!workspace) RGNN_FAIL(RGNN_EWORKSPACE, "workspace is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int D = desc->d_out, K = desc->d_in;
    RgcnBwdWs w;
    const bool bf16 = desc->dtype == RGNN_BF16, h = rows_bf16(desc), relu = desc->activation == RGNN_ACT_RELU;
    const void* W16 = bf16 ? W : nullptr;
    Bf16Stage stg(workspace, carve_rgcn_bwd(g, desc, workspace, &w), bf16, st);
    const float* X32 = (!h || W0) ? stg.in(X, (size_t)g->N * K) : nullptr;
    const float* W32 = !h ? stg.in(W, (size_t)g->R * K * D) : nullptr;
    const float* W032 = stg.in(W0, (size_t)K * D);
    const float* dO32 = (!h || W0) ? stg.in(dOut, (size_t)g->N * D) : nullptr;
    RGNN_TRY(stg.status);
    const bool acc = grads_accumulate(desc);
    GradAcc ga;
    dW = ga.route(w.acc_dW, dW, (size_t)g->R * K * D);
    dW0 = ga.route(w.acc_dW0, dW0, (size_t)K * D);
    // gradient before the activation, in the storage the traversal reads (dPre) and, where an fp32
    // kernel needs it, in fp32 (dPre32)
    const void* dPre = h ? dOut : dO32;
    const float* dPre32 = dO32;
    if (relu) {
        RGNN_TRY(relu_grad((size_t)g->N * D, static_cast<const float*>(out), dPre, w.dPre, st, h));
        dPre = w.dPre;
        if (h && W0) {
            RGNN_TRY(relu_grad((size_t)g->N * D, static_cast<const float*>(out), dO32, w.dPre32, st, 0));
            dPre32 = w.dPre32;
        } else if (!h) {
            dPre32 = static_cast<const float*>(w.dPre);
        }
    }
    // 1. dHs[p] = sum_{e in out(p)} (1/c_e) dPre[dst_e]
    const float* coef = desc->norm == RGNN_NORM_IN_DEGREE_PER_REL ? g->in_invc : nullptr;
    //    (coefficients from the pair-major copy, so no per-edge indirection is left)
    const float* ocoef = coef ? g->out_invc : nullptr;
    //    With bf16 rows the row of a pair with a single edge is not written per pair: the typed-linear backward
    //    reads dPre[dst_e] through its row selector and multiplies it by 1/c_e on the way in.
    const bool sel = sched_row_select(RGNN_LAYER_RGCN, desc->dtype, D, 1, desc->flags);
    const int32_t* ysel = sel ? g->pair_ysel : nullptr;
    const void* y_alt = sel ? dPre : nullptr;
    const float* yscale = sel && coef ? g->pair_scale : nullptr;
    RGNN_TRY(gather_sum(sel ? g->pair_items_multi : g->pair_items, D, nullptr, g->idx[RGNN_IDX_OUT_DST], 0, ocoef, 1, 0, dPre, w.G,
                        w.partial, st, 1, "aggregate_bwd_pair", "aggregate_bwd_pair.combine", 1, h, h));
    // 2. per pair dXp = dHs W^T; dW[r] = sum X^T dHs
    RGNN_TRY(tl_bwd(h, &g->pair_tiles, &g->pair_tiles_wide, D, h ? X : static_cast<const void*>(X32), g->idx[RGNN_IDX_PAIR_SRC], 0, W32, W16, w.G,
                    w.dXp, h, static_cast<float*>(dW), w.tl_part, "typed_linear_bwd", st, false, ysel, y_alt, yscale, K));
    // 3. self-loop: dX0 = dPre W0^T, dW0 = X^T dPre
    if (W0) {
        TypedLinearBwdArgs s{};
        s.tiles = &g->all_tiles; s.X = X32; s.W = W032; s.dY = dPre32;
        s.dXrow = w.dX0; s.dW = static_cast<float*>(dW0); s.part = w.tl_part; s.label = "self_loop_bwd";
        RGNN_TRY(typed_linear_bwd(K, D, s, st));
    }
    // 4. dX[u] = sum over u's pairs of dXp (+ dX0[u]) (+ what dX holds, when gradients accumulate)
    const float* extra = W0 ? w.dX0 : nullptr;
    if (acc && W0) RGNN_TRY(add_into((size_t)g->N * K, static_cast<const float*>(dX), w.dX0, st));
    else if (acc) extra = static_cast<const float*>(dX);
    RGNN_TRY(node_grad_sum(g, K, w.dXp, nullptr, nullptr, extra, dX, st, h, 0));
    return ga.flush(st);
}

// =========================================================================== RGAT

namespace {

// The library's own scratch for rgnn_rgat_fwd_static: device memory inside the code object, one copy per GPU,
// held until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the
// device address it yields (per device) is what kernels and carve-outs use.
static __device__ __align__(256) unsigned char scratch[RGNN_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

}  // namespace

namespace rgnn {
// Address of the static scratch array on the current device; looked up once per device and kept.
rgnn_status_t static_scratch(void** p) {
    int dev = 0;
    RGNN_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) RGNN_FAIL(RGNN_EUNSUPPORTED, "device ordinal %d is beyond the %d the library tracks", dev, kMaxDevices);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        RGNN_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) RGNN_FAIL(RGNN_EHIP, "hipGetSymbolAddress returned a null address for the static scratch");
        g_scratch_ptr[dev] = ptr;
    }
    *p = g_scratch_ptr[dev];
    return RGNN_OK;
}
}  // namespace rgnn

static rgnn_status_t rgat_fwd_impl(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X, const void* W,
                                   const void* w_s, const void* w_t, void* out, void* saved, void* workspace, void* stream);

extern "C" rgnn_status_t rgnn_rgat_fwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X,
                                       const void* W, const void* w_s, const void* w_t, void* out, void* saved,
                                       void* workspace, void* stream) {
    return rgat_fwd_impl(g, desc, X, W, w_s, w_t, out, saved, workspace, stream);
}

extern "C" rgnn_status_t rgnn_rgat_fwd_static(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X,
                                              const void* W, const void* w_s, const void* w_t, void* out, void* saved,
                                              void* stream) {
    size_t need = 0, sv = 0;
    RGNN_TRY(rgnn_workspace_bytes(g, RGNN_LAYER_RGAT, desc, &need, nullptr, &sv));
    if (!saved) need = align_up(need) + sv;      // inference: the would-be saved tensors are scratch too
    if (need > (size_t)RGNN_STATIC_SCRATCH_BYTES)
        RGNN_FAIL(RGNN_EWORKSPACE, "rgnn_rgat_fwd_static: this call needs %zu bytes of scratch, the static buffer holds %zu",
                  need, (size_t)RGNN_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    RGNN_TRY(static_scratch(&ws));
    return rgat_fwd_impl(g, desc, X, W, w_s, w_t, out, saved, ws, stream);
}

static rgnn_status_t rgat_fwd_impl(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X, const void* W,
                                   const void* w_s, const void* w_t, void* out, void* saved, void* workspace, void* stream) {
    RGNN_TRY(check_desc(g, desc, RGNN_LAYER_RGAT));
    ScheduleFlagsScope sched_scope(desc->flags);
    if (missing(g, X) || !W || !w_s || !w_t || missing(g, out)) RGNN_FAIL(RGNN_EINVAL, "a required tensor pointer is NULL");
    if (!workspace) RGNN_FAIL(RGNN_EWORKSPACE, "workspace is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int D = desc->d_out, K = desc->d_in;
    RgatFwdWs w; RgatSaved sv;
    const size_t carved = carve_rgat_fwd(g, desc, workspace, &w);
    saved = saved_or_scratch(g, RGNN_LAYER_RGAT, desc, saved, workspace, carved);
    Bf16Stage stg(workspace, carved, desc->dtype == RGNN_BF16, st);
    X = stg.in(X, (size_t)g->N * K);
    W = stg.in(W, (size_t)g->R * K * D);
    w_s = stg.in(w_s, (size_t)g->R * D);
    w_t = stg.in(w_t, (size_t)g->R * D);
    RGNN_TRY(stg.status);
    carve_rgat_saved(g, desc, saved, &sv);
    const float *Xf = static_cast<const float*>(X), *Wf = static_cast<const float*>(W);
    const bool fused = rgat_fused(desc);
    // 1. compact messages: Hs[p] = X[pair_src[p]] W[r]
    //    (the comparison schedules also take the source half of the logit per pair, s_src[p] = Hs[p] . w_s[r])
    TypedLinearArgs a{};
    a.tiles = &g->pair_tiles_wide; a.X = Xf; a.gather = g->idx[RGNN_IDX_PAIR_SRC]; a.W = Wf; a.Y = sv.Hs;
    if (!fused) { a.vec = static_cast<const float*>(w_s); a.s_out = w.s_src; }
    RGNN_TRY(typed_linear_fwd(K, D, a, st));
    // 2. destination half, once per (dst, rel) run, reordered: s_dst[q] = X[dst] . (W[r] w_t[r])  (per head: the head's columns)
    const int H = desc->heads;
    if (H > 1) {
        RGNN_TRY(fold_weight_heads(g->R, K, D, H, Wf, static_cast<const float*>(w_t), w.wtp, st));
        RGNN_TRY(run_logit_heads(g, K, H, Xf, w.wtp, sv.s_dst, st));
    } else {
        RGNN_TRY(fold_weight(g->R, K, D, Wf, static_cast<const float*>(w_t), w.wtp, st));
        RGNN_TRY(run_logit(g, K, Xf, w.wtp, sv.s_dst, st));
    }
    if (!fused) {
        // 3'. edge softmax in a pass of its own (one attention weight per edge, and (max, sum) per destination for the
        //     backward call), then the weighted sum: by the destination-segment walk, or edge by edge with atomic adds
        RGNN_TRY(edge_softmax(g, w.s_src, sv.s_dst, desc->slope, w.att, w.part_m, w.part_s, st, sv.ms));
        if (rgat_edge_parallel(desc)) return aggregate_edge_parallel(g, D, w.att, sv.Hs, static_cast<float*>(out), st);
        return gather_sum(g->dst_items, D, nullptr, g->idx[RGNN_IDX_IN_PAIR], 0, w.att, 1, 1, sv.Hs, static_cast<float*>(out),
                          w.partial, st, 0, "aggregate_fwd", "aggregate_fwd.combine");
    }
    // 3. one walk per destination: logit from the gathered row, running-maximum softmax, weighted sum
    return rgat_aggregate_fwd(g, D, H, sv.Hs, static_cast<const float*>(w_s), sv.s_dst, desc->slope, static_cast<float*>(out),
                              sv.ms, w.partial, w.part_ms, st);
}

extern "C" rgnn_status_t rgnn_rgat_bwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X,
                                       const void* W, const void* w_s, const void* w_t, const void* out,
                                       const void* saved, const void* dOut, void* dX, void* dW, void* dw_s,
                                       void* dw_t, void* workspace, void* stream) {
    RGNN_TRY(check_desc(g, desc, RGNN_LAYER_RGAT));
    ScheduleFlagsScope sched_scope(desc->flags);
    if (missing(g, X) || !W || !w_s || !w_t || missing(g, out) || missing(g, dOut) || missing(g, dX) || !dW || !dw_s || !dw_t)
        RGNN_FAIL(RGNN_EINVAL, "a required tensor pointer is NULL");
    if (!workspace || !saved) RGNN_FAIL(RGNN_EWORKSPACE, "workspace or saved is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int D = desc->d_out, K = desc->d_in;
    RgatBwdWs w; RgatSaved sv;
    Bf16Stage stg(workspace, carve_rgat_bwd(g, desc, workspace, &w), desc->dtype == RGNN_BF16, st);
    X = stg.in(X, (size_t)g->N * K);
    W = stg.in(W, (size_t)g->R * K * D);
    w_s = stg.in(w_s, (size_t)g->R * D);
    w_t = stg.in(w_t, (size_t)g->R * D);
    dOut = stg.in(dOut, (size_t)g->N * D);
    RGNN_TRY(stg.status);
    carve_rgat_saved(g, desc, const_cast<void*>(saved), &sv);
    const float* Xf = static_cast<const float*>(X);
    const float* Wf = static_cast<const float*>(W);
    const float* dO = static_cast<const float*>(dOut);
    const bool acc = grads_accumulate(desc);
    GradAcc ga;
    dW = ga.route(w.acc_dW, dW, (size_t)g->R * K * D);
    dw_s = ga.route(w.acc_dws, dw_s, (size_t)g->R * D);
    dw_t = ga.route(w.acc_dwt, dw_t, (size_t)g->R * D);
    const float* dX_old = acc ? static_cast<const float*>(dX) : nullptr;      // added by the kernel that writes dX
    if (desc->heads > 1) {
        const int H = desc->heads;
        const float *ws = static_cast<const float*>(w_s), *wt = static_cast<const float*>(w_t);
        // 1. per CSR edge and head: att recomputed from the gathered row and the saved (m, s), and
        //    dz = att (dOut[v].Hs[pair_e] - dOut[v].out[v])_h * (z > 0 ? 1 : slope);  adz[e] = (att[0..H), dz[0..H))
        //    With the row selector the only edge of a single-edge pair also writes that pair's (dz[0..H), att[0..H)) into
        //    ds_src[p], which holds 2 H floats per pair.
        const bool sel = rgat_row_select(desc);
        RGNN_TRY(rgat_edge_dot_bwd(g, D, H, sv.Hs, ws, sv.s_dst, sv.ms, dO, static_cast<const float*>(out), desc->slope, w.adz,
                                   nullptr, nullptr, sel ? w.ds_src : nullptr, st));
        // 2. per-head sums of dz over runs and over pairs: ds_src[p][h] is element p * 2 H + h (step 1 wrote the pairs
        //    with one edge when the selector is on)
        RGNN_TRY(segment_scalar_sum((int)g->Q, g->idx[RGNN_IDX_RUN_PTR], g->long_runs, nullptr, w.adz, 2 * H, H, w.ds_dst, st,
                                    "ds_dst_sum", 0, H));
        RGNN_TRY(segment_scalar_sum((int)g->P, g->idx[RGNN_IDX_OUT_PTR], g->long_pairs, g->idx[RGNN_IDX_OUT_EPOS], w.adz, 2 * H, H,
                                    w.ds_src, st, "ds_src_sum", sel ? 2 : 0, H, sel, 2 * H));
        // 3. dHs[p] = sum_{e in out(p)} att_e dOut[dst_e] (per head)  +  ds_src[p][h] w_s[r] (per head).  With the
        //    selector only for the pairs with several edges (step 4 forms the other rows from dOut as it reads them),
        //    and the walk sums ds_src[p][h] itself over the same (att, dz) entries; step 2 then covered only the pairs
        //    with more edges than a lane sums, among them the ones the walk cuts into pieces.
        const Rank1 r1{w.ds_src, 2 * H, g->idx[RGNN_IDX_PAIR_REL], ws};      // the second term, added when a pair's row is stored
        RGNN_TRY(gather_sum(sel ? g->pair_items_multi : g->pair_items, D, g->idx[RGNN_IDX_OUT_EPOS], g->idx[RGNN_IDX_OUT_DST], 0, w.adz,
                            2 * H, 0, dO, w.G, w.partial, st, 1, "aggregate_bwd_pair", "aggregate_bwd_pair.combine", H, 0, 0, &r1,
                            sel ? w.ds_src : nullptr, 2 * H));
        // 4. dXp = dHs W^T, dW = sum X^T dHs; with the selector also A[r][h] = sum over r's pairs of ds_src[p][h] X[src_p]
        TypedLinearBwdArgs b{};
        b.tiles = &g->pair_tiles_wide; b.X = Xf; b.gather = g->idx[RGNN_IDX_PAIR_SRC]; b.W = Wf; b.dY = w.G; b.dXrow = w.dXp;
        b.dW = static_cast<float*>(dW); b.part = w.tl_part;
        if (sel) { b.ysel = g->pair_ysel; b.dY_alt = dO; b.hcoef = w.ds_src; b.wvec = ws; b.sel_heads = H; b.Avec = w.A; }
        RGNN_TRY(typed_linear_bwd(K, D, b, st));
        // 5. dw_s[r] = sum over r's pairs of ds_src[p][h] Hs[p] (per head; the pair rows are in relation order);
        //    with the selector from A instead, in step 6: dw_s[r] = (A[r][h] W[r]) on the columns of head h
        if (!sel)
            RGNN_TRY(gather_sum(g->relpair_items, D, nullptr, nullptr, 0, w.ds_src, 2 * H, 0, sv.Hs, dw_s, w.partial, st, 2,
                                "src_vec_grad", "src_vec_grad.combine", H));
        // 6. U[h][r] = sum over r's runs of ds_dst[q][h] X[run_dst[q]];  dw_t and the w_t part of dW from it
        RGNN_TRY(gather_heads_rows(g->relrun_items, K, H, g->R, g->idx[RGNN_IDX_RELRUN_IDX], g->relrun_dst, 0, w.ds_dst,
                                   Xf, w.U, w.partial, st, "dst_side_wgrad", "dst_side_wgrad.combine"));
        RGNN_TRY(rgat_heads_param_finish(g->R, K, D, H, Wf, wt, w.U, sel ? w.A : nullptr, static_cast<float*>(dW),
                                         static_cast<float*>(dw_s), static_cast<float*>(dw_t), st));
        // 7. dX[u] = sum over u's pairs of dXp + sum over u's runs and heads of ds_dst[q][h] (W[r] w_t[r])_h
        RGNN_TRY(fold_weight_heads(g->R, K, D, H, Wf, wt, w.wtp, st));
        RGNN_TRY(node_grad_sum(g, K, w.dXp, w.ds_dst, w.wtp, dX_old, dX, st, 0, 0, H));
        return ga.flush(st);
    }
    // 1. per CSR edge: (att_e, dz_e), att_e recomputed from the gathered row and the saved (m, s); for single-edge pairs also ds_src[p] and G[p] = att_e dOut[dst_e] (or, with
    //    the row selector, only att_e: step 4 then reads the row from dOut).  With the selector ds_src[p] and that
    //    att_e are stored side by side (one 8-byte store here, one 8-byte load per row in step 4): w.ds_src then
    //    holds P pairs of floats and ds_src[p] is element 2 p.
    const bool sel = rgat_row_select(desc);
    const int dss = sel ? 2 : 1;
    RGNN_TRY(rgat_edge_dot_bwd(g, D, 1, sv.Hs, static_cast<const float*>(w_s), sv.s_dst, sv.ms, dO, static_cast<const float*>(out),
                               desc->slope, w.adz, w.G, w.ds_src, sel ? w.ds_src : nullptr, st));
    // 2. ds_dst[q] = sum over the run's edges of dz
    RGNN_TRY(segment_scalar_sum((int)g->Q, g->idx[RGNN_IDX_RUN_PTR], g->long_runs, nullptr, w.adz, 2, 1, w.ds_dst, st, "ds_dst_sum"));
    // 3. for the pairs with several edges (step 1 wrote the others): G[p] = sum_{e in out(p)} att_e dOut[dst_e] and, in
    //    the same walk over (att_e, dz_e), ds_src[p] = sum of dz_e; the pairs with more edges than a lane sums
    //    (among them the ones the walk cuts into pieces) get ds_src from the workgroup-per-segment sum afterwards
    RGNN_TRY(gather_sum(g->pair_items_multi, D, g->idx[RGNN_IDX_OUT_EPOS], g->idx[RGNN_IDX_OUT_DST], 0, w.adz, 2, 0, dO, w.G,
                        w.partial, st, 1, "aggregate_bwd_pair", "aggregate_bwd_pair.combine", 1, 0, 0, nullptr, w.ds_src, dss));
    RGNN_TRY(segment_scalar_sum((int)g->P, g->idx[RGNN_IDX_OUT_PTR], g->long_pairs, g->idx[RGNN_IDX_OUT_EPOS], w.adz, 2, 1, w.ds_src, st,
                                "ds_src_sum", 2, 1, true, dss));
    // 4. with dHs[p] = G[p] + ds_src[p] w_s[r]:
    //    dXp[p] = dHs[p] W[r]^T = G[p] W[r]^T + ds_src[p] (W[r] w_s[r]);  dW[r] = sum X^T G (+ A^T (x) w_s in step 6);
    //    A[r] = sum ds_src X
    RGNN_TRY(fold_weight(g->R, K, D, Wf, static_cast<const float*>(w_s), w.wsp, st, static_cast<const float*>(w_t), w.wtp));   // wtp: step 7
    TypedLinearBwdArgs b{};
    b.tiles = &g->pair_tiles_wide; b.X = Xf; b.gather = g->idx[RGNN_IDX_PAIR_SRC]; b.W = Wf; b.dY = w.G; b.dXrow = w.dXp;
    b.rowscale = sel ? nullptr : w.ds_src; b.vec = w.wsp; b.dW = static_cast<float*>(dW); b.Avec = w.A;
    b.part = w.tl_part;
    if (sel) { b.ysel = g->pair_ysel; b.dY_alt = dO; b.ds_yscale = reinterpret_cast<const float2*>(w.ds_src); }
    RGNN_TRY(typed_linear_bwd(K, D, b, st));
    // 5. U[r] = sum over r's runs of ds_dst[q] X[run_dst[q]]
    RGNN_TRY(gather_sum(g->relrun_items, K, g->idx[RGNN_IDX_RELRUN_IDX], g->relrun_dst, 0, w.ds_dst, 1, 0, Xf,
                        w.U, w.partial, st, 2, "dst_side_wgrad", "dst_side_wgrad.combine"));
    // 6. dw_s = A W, dw_t = U W, dW += A^T (x) w_s + U^T (x) w_t
    RGNN_TRY(rgat_param_finish(g->R, K, D, Wf, static_cast<const float*>(w_s), static_cast<const float*>(w_t), w.A, w.U,
                               static_cast<float*>(dW), static_cast<float*>(dw_s), static_cast<float*>(dw_t), st));
    // 7. dX[u] = sum over u's pairs of dXp + sum over u's runs of ds_dst[q] (W[r] w_t[r])
    RGNN_TRY(node_grad_sum(g, K, w.dXp, w.ds_dst, w.wtp, dX_old, static_cast<float*>(dX), st));
    return ga.flush(st);
}

// =========================================================================== HGT

extern "C" rgnn_status_t rgnn_hgt_fwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X,
                                      const void* Wk, const void* Wq, const void* Wv, const void* Wo, const void* Watt,
                                      const void* Wmsg, const void* mu, void* out, void* saved, void* workspace,
                                      void* stream) {
    RGNN_TRY(check_desc(g, desc, RGNN_LAYER_HGT));
    ScheduleFlagsScope sched_scope(desc->flags);
    if (missing(g, X) || !Wk || !Wq || !Wv || !Wo || !Watt || !Wmsg || missing(g, out)) RGNN_FAIL(RGNN_EINVAL, "a required tensor pointer is NULL");
    if (!workspace) RGNN_FAIL(RGNN_EWORKSPACE, "workspace is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int D = desc->d_out, H = desc->heads;
    HgtFwdWs w; HgtSaved sv;
    const bool bf16 = desc->dtype == RGNN_BF16, h = rows_bf16(desc);
    const void *X16 = bf16 ? X : nullptr, *Wk16 = bf16 ? Wk : nullptr, *Wq16 = bf16 ? Wq : nullptr,
               *Wv16 = bf16 ? Wv : nullptr, *Wo16 = bf16 ? Wo : nullptr;
    const size_t carved = carve_hgt_fwd(g, desc, workspace, &w);
    saved = saved_or_scratch(g, RGNN_LAYER_HGT, desc, saved, workspace, carved);
    Bf16Stage stg(workspace, carved, bf16, st);
    const size_t tdd = (size_t)g->T * D * D, rh = (size_t)g->R * H, dh = D / H;
    // fp32 copies: at width 128 only of the small per-relation parameters (their expansion is an fp32 kernel)
    const bool fold = hgt_folded(g, desc);
    const float* X32 = !h ? stg.in(X, (size_t)g->N * D) : nullptr;
    const float* Wk32 = !h || fold ? stg.in(Wk, tdd) : nullptr;      // folding multiplies weights in fp32
    const float* Wq32 = !h ? stg.in(Wq, tdd) : nullptr;
    const float* Wv32 = !h || fold ? stg.in(Wv, tdd) : nullptr;
    const float* Wo32 = !h ? stg.in(Wo, tdd) : nullptr;
    const float* Watt32 = stg.in(Watt, rh * dh * dh);
    const float* Wmsg32 = stg.in(Wmsg, rh * dh * dh);
    const float* mu32 = stg.in(mu, rh);
    RGNN_TRY(stg.status);
    carve_hgt_saved(g, desc, saved, &sv);
    const int32_t* perm = g->idx[RGNN_IDX_NTYPE_PERM];
    const int32_t* psrc = g->idx[RGNN_IDX_PAIR_SRC];
    // bf16 form of an intermediate row tensor (nullptr when the rows are fp32) and its fp32 form
    auto R16 = [h](const void* p) { return h ? p : nullptr; };
    auto R32 = [h](const void* p) { return h ? nullptr : static_cast<const float*>(p); };
    // 1. per node type: Q, and K, V unless they are folded into the per-pair linears
    RGNN_TRY(tl_fwd(bf16, &g->node_tiles, &g->node_tiles_wide, D, X32, X16, perm, 1, Wq32, Wq16, sv.Q, h, "node_linear_q", st));
    if (!fold) {
        RGNN_TRY(tl_fwd(bf16, &g->node_tiles, &g->node_tiles_wide, D, X32, X16, perm, 1, Wk32, Wk16, sv.K, h, "node_linear_k", st));
        RGNN_TRY(tl_fwd(bf16, &g->node_tiles, &g->node_tiles_wide, D, X32, X16, perm, 1, Wv32, Wv16, sv.V, h, "node_linear_v", st));
    }
    // 2. per (relation, head) matrices as block-diagonal d x d weights; mu / sqrt(dh) folded into the attention one
    RGNN_TRY(hgt_expand(g->R, D, H, Watt32, mu32, 1, w.Wbd_att, st));
    RGNN_TRY(hgt_expand(g->R, D, H, Wmsg32, nullptr, 0, w.Wbd_msg, st));
    // 3. compact per pair: Ka[p] = K[src_p] Watt[r], M[p] = V[src_p] Wmsg[r]
    if (fold) {
        //    = X[src_p] (Wk[type of r's sources] Watt[r]) and X[src_p] (Wv[type] Wmsg[r])
        //    With bf16 rows the products are rounded to bf16 once (as K and V would have been) and feed the
        //    matrix cores as they are; rows in the storage of the intermediates: the caller's bf16 X at width
        //    128, its fp32 copy otherwise.
        RGNN_TRY(hgt_fold(g->R, D, H, g->rel_src_type, Wk32, w.Wbd_att, h ? nullptr : w.Wf_att, h ? w.Wf_att : nullptr, st));
        RGNN_TRY(hgt_fold(g->R, D, H, g->rel_src_type, Wv32, w.Wbd_msg, h ? nullptr : w.Wf_msg, h ? w.Wf_msg : nullptr, st));
        RGNN_TRY(tl_fwd(bf16, &g->pair_tiles, &g->pair_tiles_wide, D, X32, R16(X), psrc, 0, R32(w.Wf_att), R16(w.Wf_att), sv.Ka, h, "pair_linear_att", st));
        RGNN_TRY(tl_fwd(bf16, &g->pair_tiles, &g->pair_tiles_wide, D, X32, R16(X), psrc, 0, R32(w.Wf_msg), R16(w.Wf_msg), sv.M, h, "pair_linear_msg", st));
    } else {
        RGNN_TRY(tl_fwd(bf16, &g->pair_tiles, &g->pair_tiles_wide, D, R32(sv.K), R16(sv.K), psrc, 0, w.Wbd_att, nullptr, sv.Ka, h, "pair_linear_att", st));
        RGNN_TRY(tl_fwd(bf16, &g->pair_tiles, &g->pair_tiles_wide, D, R32(sv.V), R16(sv.V), psrc, 0, w.Wbd_msg, nullptr, sv.M, h, "pair_linear_msg", st));
    }
    // 4. per edge and head: logit, softmax over the destination's edges
    RGNN_TRY(hgt_edge_logit(g, D, H, sv.Ka, sv.Q, sv.att, st, h, w.part_m, w.part_s));     // logits, then softmax per head
    // 5. Z[v][h] = sum_e att[e][h] M[pair_e][h]
    RGNN_TRY(gather_sum(g->dst_items, D, nullptr, g->idx[RGNN_IDX_IN_PAIR], 0, sv.att, H, 0, sv.M, sv.Z, w.partial, st, 0,
                        "aggregate_fwd", "aggregate_fwd.combine", H, h, h));
    // 6. out = Z Wo[type]
    RGNN_TRY(tl_fwd(bf16, &g->node_tiles, &g->node_tiles_wide, D, R32(sv.Z), R16(sv.Z), perm, 1, Wo32, Wo16, out, false, "node_linear_out", st));
    return RGNN_OK;
}

extern "C" rgnn_status_t rgnn_hgt_bwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X,
                                      const void* Wk, const void* Wq, const void* Wv, const void* Wo, const void* Watt,
                                      const void* Wmsg, const void* mu, const void* out, const void* saved,
                                      const void* dOut, void* dX, void* dWk, void* dWq, void* dWv, void* dWo,
                                      void* dWatt, void* dWmsg, void* dmu, void* workspace, void* stream) {
    (void)out;
    RGNN_TRY(check_desc(g, desc, RGNN_LAYER_HGT));
    ScheduleFlagsScope sched_scope(desc->flags);
    if (missing(g, X) || !Wk || !Wq || !Wv || !Wo || !Watt || !Wmsg || missing(g, dOut) || missing(g, dX) || !dWk || !dWq || !dWv || !dWo || !dWatt || !dWmsg)
        RGNN_FAIL(RGNN_EINVAL, "a required tensor pointer is NULL");
    if (mu && !dmu) RGNN_FAIL(RGNN_EINVAL, "dmu is NULL but mu is given");
    if (!workspace || !saved) RGNN_FAIL(RGNN_EWORKSPACE, "workspace or saved is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int D = desc->d_out, H = desc->heads;
    HgtBwdWs w; HgtSaved sv;
    const bool bf16 = desc->dtype == RGNN_BF16, h = rows_bf16(desc);
    const void *Wk16 = bf16 ? Wk : nullptr, *Wq16 = bf16 ? Wq : nullptr, *Wv16 = bf16 ? Wv : nullptr,
               *Wo16 = bf16 ? Wo : nullptr;
    Bf16Stage stg(workspace, carve_hgt_bwd(g, desc, workspace, &w), bf16, st);
    const size_t tdd = (size_t)g->T * D * D, rh = (size_t)g->R * H, dh = D / H;
    const bool fold = hgt_folded(g, desc);
    const float* X32 = !h ? stg.in(X, (size_t)g->N * D) : nullptr;
    const float* Wk32 = !h || fold ? stg.in(Wk, tdd) : nullptr;
    const float* Wq32 = !h ? stg.in(Wq, tdd) : nullptr;
    const float* Wv32 = !h || fold ? stg.in(Wv, tdd) : nullptr;
    const float* Wo32 = !h ? stg.in(Wo, tdd) : nullptr;
    const float* Watt32 = stg.in(Watt, rh * dh * dh);
    const float* Wmsg32 = stg.in(Wmsg, rh * dh * dh);
    const float* mu32 = stg.in(mu, rh);
    const float* dO32 = !h ? stg.in(dOut, (size_t)g->N * D) : nullptr;
    RGNN_TRY(stg.status);
    carve_hgt_saved(g, desc, const_cast<void*>(saved), &sv);
    // row operands in the storage of this mode: the caller's bf16 tensors as they are, or the fp32 copies
    const void* Xr = h ? X : static_cast<const void*>(X32);
    const void* dOr = h ? dOut : static_cast<const void*>(dO32);
    const int32_t* perm = g->idx[RGNN_IDX_NTYPE_PERM];
    const int32_t* psrc = g->idx[RGNN_IDX_PAIR_SRC];
    const bool acc = grads_accumulate(desc);
    GradAcc ga;
    dWk = ga.route(w.acc_node[0], dWk, tdd); dWq = ga.route(w.acc_node[1], dWq, tdd);
    dWv = ga.route(w.acc_node[2], dWv, tdd); dWo = ga.route(w.acc_node[3], dWo, tdd);
    dWatt = ga.route(w.acc_rel[0], dWatt, rh * dh * dh); dWmsg = ga.route(w.acc_rel[1], dWmsg, rh * dh * dh);
    dmu = ga.route(w.acc_mu, dmu, rh);
    // 1. output linear: dZ = dOut Wo^T, dWo = Z^T dOut
    RGNN_TRY(tl_bwd(h, &g->node_tiles, &g->node_tiles_wide, D, sv.Z, perm, 1, Wo32, Wo16, dOr, w.dZ, h, static_cast<float*>(dWo), w.tl_part,
                    "node_linear_out_bwd", st));
    // 2. per edge and head: d logit
    RGNN_TRY(hgt_edge_dot_bwd(g, D, H, sv.att, sv.M, w.dZ, sv.Z, w.dl, st, h));
    // 3. pair-major: dM[p][h] = sum att dZ[dst][h];  dKa[p][h] = sum dl Q[dst][h]
    RGNN_TRY(gather_sum(g->pair_items, D, g->idx[RGNN_IDX_OUT_EPOS], g->idx[RGNN_IDX_OUT_DST], 0, sv.att, H, 0, w.dZ, w.dM,
                        w.partial, st, 1, "aggregate_bwd_msg", "aggregate_bwd_msg.combine", H, h, h));
    RGNN_TRY(gather_sum(g->pair_items, D, g->idx[RGNN_IDX_OUT_EPOS], g->idx[RGNN_IDX_OUT_DST], 0, w.dl, H, 0, sv.Q, w.dKa,
                        w.partial, st, 1, "aggregate_bwd_key", "aggregate_bwd_key.combine", H, h, h));
    // 4. destination-major: dQ[v][h] = sum dl Ka[pair][h]
    RGNN_TRY(gather_sum(g->dst_items, D, nullptr, g->idx[RGNN_IDX_IN_PAIR], 0, w.dl, H, 0, sv.Ka, w.dQ, w.partial, st, 0,
                        "aggregate_bwd_query", "aggregate_bwd_query.combine", H, h, h));
    // 5. per-pair linears backward
    RGNN_TRY(hgt_expand(g->R, D, H, Watt32, mu32, 1, w.Wbd_att, st));
    RGNN_TRY(hgt_expand(g->R, D, H, Wmsg32, nullptr, 0, w.Wbd_msg, st));
    if (fold) {
        // the folded weights take the per-pair gradients straight to X's rows; their own gradients are
        // unfolded into those of the node-type and of the per-relation matrices
        RGNN_TRY(hgt_fold(g->R, D, H, g->rel_src_type, Wk32, w.Wbd_att, h ? nullptr : w.Wf_att, h ? w.Wf_att : nullptr, st));
        RGNN_TRY(hgt_fold(g->R, D, H, g->rel_src_type, Wv32, w.Wbd_msg, h ? nullptr : w.Wf_msg, h ? w.Wf_msg : nullptr, st));
        RGNN_TRY(tl_bwd(h, &g->pair_tiles, &g->pair_tiles_wide, D, Xr, psrc, 0, h ? nullptr : w.Wf_att, h ? w.Wf_att : nullptr, w.dKa, w.dKp,
                        h, w.dWf_att, w.tl_part, "pair_linear_att_bwd", st));
        RGNN_TRY(tl_bwd(h, &g->pair_tiles, &g->pair_tiles_wide, D, Xr, psrc, 0, h ? nullptr : w.Wf_msg, h ? w.Wf_msg : nullptr, w.dM, w.dVp,
                        h, w.dWf_msg, w.tl_part, "pair_linear_msg_bwd", st));
        RGNN_TRY(hgt_fold_bwd(g->T, g->R, D, H, g->rel_src_type, Wk32, w.Wbd_att, w.dWf_att, w.dWbd_att, static_cast<float*>(dWk), st));
        RGNN_TRY(hgt_fold_bwd(g->T, g->R, D, H, g->rel_src_type, Wv32, w.Wbd_msg, w.dWf_msg, w.dWbd_msg, static_cast<float*>(dWv), st));
        RGNN_TRY(hgt_extract(g->R, D, H, w.dWbd_att, Watt32, mu32, 1, static_cast<float*>(dWatt), static_cast<float*>(dmu), st));
        RGNN_TRY(hgt_extract(g->R, D, H, w.dWbd_msg, Wmsg32, nullptr, 0, static_cast<float*>(dWmsg), nullptr, st));
        // dX = dQ Wq^T + sums over each node's pairs of the two per-pair gradients
        RGNN_TRY(tl_bwd(h, &g->node_tiles, &g->node_tiles_wide, D, Xr, perm, 1, Wq32, Wq16, w.dQ, w.dXq, false, static_cast<float*>(dWq),
                        w.tl_part, "node_linear_q_bwd", st));
        if (acc) RGNN_TRY(add_into((size_t)g->N * D, static_cast<const float*>(dX), w.dXq, st));
        RGNN_TRY(node_grad_sum(g, D, w.dKp, nullptr, nullptr, w.dXq, dX, st, h, 0, 1, w.dVp));
        return ga.flush(st);
    }
    RGNN_TRY(tl_bwd(h, &g->pair_tiles, &g->pair_tiles_wide, D, sv.K, psrc, 0, w.Wbd_att, nullptr, w.dKa, w.dKp, h, w.dWbd_att, w.tl_part,
                    "pair_linear_att_bwd", st));
    RGNN_TRY(tl_bwd(h, &g->pair_tiles, &g->pair_tiles_wide, D, sv.V, psrc, 0, w.Wbd_msg, nullptr, w.dM, w.dVp, h, w.dWbd_msg, w.tl_part,
                    "pair_linear_msg_bwd", st));
    RGNN_TRY(hgt_extract(g->R, D, H, w.dWbd_att, Watt32, mu32, 1, static_cast<float*>(dWatt), static_cast<float*>(dmu), st));
    RGNN_TRY(hgt_extract(g->R, D, H, w.dWbd_msg, Wmsg32, nullptr, 0, static_cast<float*>(dWmsg), nullptr, st));
    // 6. dK[u], dV[u] = sums over u's pairs
    RGNN_TRY(node_grad_sum(g, D, w.dKp, nullptr, nullptr, nullptr, w.dK, st, h, h));
    RGNN_TRY(node_grad_sum(g, D, w.dVp, nullptr, nullptr, nullptr, w.dV, st, h, h));
    // 7. node linears backward and dX
    //    (bf16 rows: the three input gradients are accumulated into dX by the kernels themselves)
    RGNN_TRY(tl_bwd(h, &g->node_tiles, &g->node_tiles_wide, D, Xr, perm, 1, Wk32, Wk16, w.dK, h ? dX : static_cast<void*>(w.dXk),
                    false, static_cast<float*>(dWk), w.tl_part, "node_linear_k_bwd", st, h && acc));
    RGNN_TRY(tl_bwd(h, &g->node_tiles, &g->node_tiles_wide, D, Xr, perm, 1, Wq32, Wq16, w.dQ, h ? dX : static_cast<void*>(w.dXq),
                    false, static_cast<float*>(dWq), w.tl_part, "node_linear_q_bwd", st, h));
    RGNN_TRY(tl_bwd(h, &g->node_tiles, &g->node_tiles_wide, D, Xr, perm, 1, Wv32, Wv16, w.dV, h ? dX : static_cast<void*>(w.dXv),
                    false, static_cast<float*>(dWv), w.tl_part, "node_linear_v_bwd", st, h));
    if (!h) {
        if (acc) RGNN_TRY(add_into((size_t)g->N * D, static_cast<const float*>(dX), w.dXk, st));
        RGNN_TRY(add3((size_t)g->N * D, w.dXk, w.dXq, w.dXv, static_cast<float*>(dX), st));
    }
    return ga.flush(st);
}
