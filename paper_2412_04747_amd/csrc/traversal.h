// Launchers of the traversal kernels (traversal.hip).  Internal.
#pragma once
#include "rgnn_internal.h"

namespace rgnn {

// desc.flags of the layer call in progress on this thread: the launchers consult it where they choose between
// the batched and the general walk (set by the entry points for the duration of a call).
uint32_t current_schedule_flags();
struct ScheduleFlagsScope {
    explicit ScheduleFlagsScope(uint32_t flags);
    ~ScheduleFlagsScope();
    uint32_t prev;
};

// wv[r] = W[r] w[r]; optionally a second vector per relation in the same pass (wv2[r] = W[r] w2[r])
rgnn_status_t fold_weight(int R, int kd, int nd, const float* W, const float* w, float* wv, hipStream_t st,
                          const float* w2 = nullptr, float* wv2 = nullptr);
rgnn_status_t run_logit(const rgnn_graph* g, int D, const float* X, const float* wtp, float* s_dst, hipStream_t st);
rgnn_status_t segment_scalar_sum(int n, const int32_t* ptr, const LongList& lng, const int32_t* via, const float* val,
                                 int stride, int off, float* out, hipStream_t st, const char* label, int min_len = 0,
                                 int heads = 1, bool long_only = false, int ostride = 0);   // ostride 0: heads
// ms (optional, [N] pairs of floats): (max, sum of exp) of the logits of every destination with edges
rgnn_status_t edge_softmax(const rgnn_graph* g, const float* s_src, const float* s_dst, float slope, float* att,
                           float* part_m, float* part_s, hipStream_t st, float* ms = nullptr);
// rgat_fused.hip: RGAT (H heads; head h owns column slice h) with the edge softmax fused into the traversal.
//   forward: out[v] = sum_e att_e Hs[pair_e] per head, att = softmax over v's edges of leakyrelu(Hs[pair_e] . w_s[r_e] + s_dst[run_e][h]);
//   ms[v][h] = (max logit, sum of exp(logit - max)) as pairs of floats; partial / part_ms: scratch rows and (m, s) pairs of the
//   pieces of cut destinations
rgnn_status_t rgat_aggregate_fwd(const rgnn_graph* g, int D, int H, const float* Hs, const float* w_s, const float* s_dst,
                                 float slope, float* out, float* ms, float* partial, float* part_ms, hipStream_t st);
//   backward: adz[e] = (att_e[0..H), dz_e[0..H)) with att_e recomputed from the gathered row and ms; one head: the only edge
//   of a single-edge pair also writes dsy[p] = (dz_e, att_e), or without dsy: ds_src[p] = dz_e and G[p] = att_e dOut[v]
rgnn_status_t rgat_edge_dot_bwd(const rgnn_graph* g, int D, int H, const float* Hs, const float* w_s, const float* s_dst,
                                const float* ms, const float* dOut, const float* out, float slope, float* adz, float* G,
                                float* ds_src, float* dsy, hipStream_t st);
// workgroups of `threads` threads with `lds` bytes of dynamic LDS that stay resident per compute unit (cached per kernel)
rgnn_status_t resident_blocks_per_cu(const void* kernel, int threads, size_t lds, int* out);
// Optional rank-1 term of a gather-sum: out[i] += coef[i * stride + head] * vec[seg[i]] (fp32 vec rows of the output width)
struct Rank1 { const float* coef; int stride; const int32_t* seg; const float* vec; };
rgnn_status_t gather_sum(const ItemList& L, int D, const int32_t* via, const int32_t* rowidx, int row_by_k,
                         const float* coef, int cstride, int cabs, const void* src, void* out, float* partial,
                         hipStream_t st, int role, const char* label, const char* combine_label, int heads = 1,
                         int src_bf16 = 0, int out_bf16 = 0, const Rank1* r1 = nullptr, float* sum2 = nullptr,
                         int sum2_stride = 1);
// H weighted sums of the same gathered rows in one walk (coef [entries][H]); out [H][out_rows][D]
rgnn_status_t gather_heads_rows(const ItemList& L, int D, int H, int out_rows, const int32_t* via, const int32_t* rowidx,
                                int row_by_k, const float* coef, const float* src, float* out, float* partial,
                                hipStream_t st, const char* label, const char* combine_label);
rgnn_status_t node_grad_sum(const rgnn_graph* g, int D, const void* dXp, const float* ds_dst, const float* wtp,
                            const float* extra, void* dX, hipStream_t st, int in_bf16 = 0, int out_bf16 = 0, int heads = 1,
                            const void* dXp2 = nullptr);
// hgt.hip: products of a node-type weight with the expanded per-relation weight of the relation's source type
//   Wf[r] = Wnode[rel_type[r]] Wbd[r], stored as fp32 (Wf) or rounded to bf16 (Wf16); pass one of the two
rgnn_status_t hgt_fold(int R, int d, int H, const int32_t* rel_type, const float* Wnode, const float* Wbd, float* Wf,
                       void* Wf16, hipStream_t st);
//   dWbd[r] (entries inside the head blocks) = Wnode[rel_type[r]]^T dWf[r]
//   dWnode[t] = sum over the relations r of source type t, in ascending r, of dWf[r] Wbd[r]^T
rgnn_status_t hgt_fold_bwd(int T, int R, int d, int H, const int32_t* rel_type, const float* Wnode, const float* Wbd,
                           const float* dWf, float* dWbd, float* dWnode, hipStream_t st);
rgnn_status_t rgat_param_finish(int R, int kd, int nd, const float* W, const float* w_s, const float* w_t,
                                const float* A, const float* U, float* dW, float* dw_s, float* dw_t, hipStream_t st);
// hgt.hip
rgnn_status_t hgt_expand(int R, int d, int H, const float* W, const float* mu, int scaled, float* Wbd, hipStream_t st);
rgnn_status_t hgt_extract(int R, int d, int H, const float* dWbd, const float* W, const float* mu, int scaled, float* dW,
                          float* dmu, hipStream_t st);
// with part_m / part_s: followed by the per-head softmax over each destination's edges (in the same walk where the
// lane layout allows), so that logit holds the attention weights afterwards
rgnn_status_t hgt_edge_logit(const rgnn_graph* g, int D, int H, const void* Ka, const void* Q, float* logit,
                             hipStream_t st, int rows_bf16 = 0, float* part_m = nullptr, float* part_s = nullptr);
rgnn_status_t hgt_softmax_finish(const rgnn_graph* g, int H, float* att, const float* part_m, const float* part_s, hipStream_t st);
rgnn_status_t hgt_softmax(const rgnn_graph* g, int H, float* att, float* part_m, float* part_s, hipStream_t st);
// dl = att (g - gbar)
rgnn_status_t hgt_edge_dot_bwd(const rgnn_graph* g, int D, int H, const float* att, const void* M, const void* dZ,
                               const void* Z, float* dl, hipStream_t st, int rows_bf16 = 0);
// rgat_heads.hip: pieces of multi-head RGAT
rgnn_status_t fold_weight_heads(int R, int kd, int nd, int H, const float* W, const float* w, float* wv, hipStream_t st);
rgnn_status_t run_logit_heads(const rgnn_graph* g, int D, int H, const float* X, const float* wtp, float* s_dst,
                              hipStream_t st);
rgnn_status_t rgat_heads_param_finish(int R, int kd, int nd, int H, const float* W, const float* w_t, const float* U, const float* A,
                                      float* dW, float* dw_s, float* dw_t, hipStream_t st);
// out[v] = sum_e |att_e| Hs[pair_e] edge by edge with atomic adds (zeroes out first); fp32 rows
rgnn_status_t aggregate_edge_parallel(const rgnn_graph* g, int D, const float* att, const float* Hs, float* out,
                                      hipStream_t st);
rgnn_status_t add3(size_t n, const float* a, const float* b, const float* c, float* out, hipStream_t st);

rgnn_status_t widen_bf16(size_t n, const uint16_t* src, float* dst, hipStream_t st);
rgnn_status_t add_into(size_t n, const float* src, float* dst, hipStream_t st);     // dst += src
rgnn_status_t relu_inplace(size_t n, float* x, hipStream_t st);
rgnn_status_t relu_grad(size_t n, const float* ref, const void* gin, void* y, hipStream_t st, int bf16 = 0);

}  // namespace rgnn
