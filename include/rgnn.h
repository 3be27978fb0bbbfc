/*
 * rgnn.h - C ABI of the MI355X (gfx950) relational-GNN layer library.
 *
 * One layer of RGCN, RGAT or HGT, forward and backward, over a heterogeneous
 * graph with typed nodes and typed edges (thesis Ch.3, "RGNN Formulation and
 * Operators").  The library is built from three pieces: a relation-segmented
 * typed-linear kernel on the matrix cores (Ch.3 "Inefficiency in Existing
 * Computation Stack": segment MM, Y[i] = X[i] W[T[i]] without replicating W),
 * destination-major edge-traversal kernels (edge softmax and weighted
 * aggregation, Ch.3 listing "attention calculation in a single-headed RGAT
 * model"), and compact materialization (Ch.3 "Compact Tensor Materialization
 * and Data Layout": edge data that depends only on (source node, edge type)
 * is stored once per unique pair).
 *
 * Conventions
 *   - Every function returns rgnn_status_t; nothing throws or aborts.
 *     rgnn_last_error() gives the message of the calling thread's last failure.
 *   - All tensor arguments of the layer calls are DEVICE pointers, row-major,
 *     contiguous, 16-byte aligned, owned by the caller.  The library owns only
 *     the opaque graph object.
 *   - Layer calls allocate nothing and do not synchronise; they enqueue kernels
 *     on `stream` (a hipStream_t cast to void*, NULL = default stream).
 *     `workspace` and `saved` are caller-provided device buffers of at least the
 *     sizes rgnn_workspace_bytes reports; `saved` must be kept unchanged between
 *     a forward call and its backward call, `workspace` is scratch.
 *   - Inference: a forward call with saved == NULL keeps nothing for a backward
 *     call; its `workspace` must then hold fwd_workspace + saved bytes (the
 *     tensors that would have been saved become scratch).
 *   - Weights are stored [type][d_in][d_out] so that y = x W (row vector times
 *     matrix), as in Eq. (rgcn).
 *   - Gradients are overwritten, unless desc.flags carries RGNN_FLAG_ACCUMULATE (then every gradient output of
 *     the backward call is added to what the buffer holds).
 *   - A graph may have no nodes or no edges; a [num_nodes, d] tensor of a graph
 *     without nodes may be NULL.  Parameter gradients are then written as zeros.
 *   - Index arrays are int32; graphs with 2^31 or more edges are rejected.
 */
#ifndef RGNN_H
#define RGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RGNN_OK = 0,
    RGNN_EINVAL = 1,        /* NULL pointer, bad size, id out of range */
    RGNN_EUNSUPPORTED = 2,  /* valid request the kernels do not cover (dimension, dtype, heads) */
    RGNN_ENOMEM = 3,        /* host or device allocation failed (graph_create only) */
    RGNN_EHIP = 4,          /* a HIP runtime call failed; see rgnn_last_error() */
    RGNN_EWORKSPACE = 5     /* workspace / saved pointer NULL while its size is non-zero */
} rgnn_status_t;

typedef enum { RGNN_F32 = 0, RGNN_BF16 = 1 } rgnn_dtype_t;
enum { RGNN_LAYER_RGCN = 0, RGNN_LAYER_RGAT = 1, RGNN_LAYER_HGT = 2 };
enum { RGNN_NORM_NONE = 0, RGNN_NORM_IN_DEGREE_PER_REL = 1 };
enum { RGNN_ACT_NONE = 0, RGNN_ACT_RELU = 1 };
enum { RGNN_MEM_HOST = 0, RGNN_MEM_DEVICE = 1 };
enum { RGNN_COO = 0, RGNN_CSR_DST = 1 };

typedef struct rgnn_graph rgnn_graph_t;

typedef struct {
    int64_t num_nodes;           /* N */
    int64_t num_edges;           /* E */
    int64_t num_pairs;           /* P: unique (source node, relation) pairs; P/E is the thesis's entity compaction ratio */
    int64_t num_runs;            /* Q: unique (destination node, relation) pairs */
    int64_t max_in_degree;
    int64_t max_pair_out_degree; /* most edges sharing one (source, relation) pair */
    int64_t index_bytes;         /* device memory held by the graph */
    int32_t num_rels;            /* R */
    int32_t num_ntypes;          /* T */
    int64_t num_single_pairs;    /* pairs with exactly one edge */
} rgnn_graph_info_t;

/* Parameters of one layer call.  Fields a layer does not use are ignored.
 *   dtype      storage type of the INPUT tensor arguments (X, every weight, dOut):
 *              RGNN_F32, or RGNN_BF16 = bfloat16 inputs.  Sums and products are fp32 and
 *              every output (out, all gradients) and the `out` argument of the backward
 *              calls are fp32 in both cases.  With RGNN_BF16 at width 128 the RGCN and HGT
 *              layers also keep their intermediate row tensors (projected messages, keys,
 *              queries, values and their gradients, in the workspace and in `saved`) in
 *              bfloat16, rounded to nearest even from the fp32 accumulators; results then
 *              agree with an fp64 evaluation to a few 1e-3 relative to the largest entry.
 *   d_in,d_out feature widths.  Supported: d_in == d_out in {32, 64, 128}; RGCN and RGAT with fp32 inputs also
 *              take d_in, d_out in {32, 64} with d_in != d_out.
 *   heads      number of attention heads H of HGT and RGAT (d_out % H == 0; d_out/H in {16, 32, 64},
 *              any width for single-head RGAT).  With H > 1, num_nodes * H and num_edges * H
 *              must stay below 2^31 (EUNSUPPORTED otherwise).
 *   slope      RGAT leaky-ReLU negative slope (the derivative at 0 is `slope`).
 *   norm       RGCN: RGNN_NORM_IN_DEGREE_PER_REL divides each message by c_{v,r},
 *              the number of incoming edges of v with relation r (Eq. (rgcn)).
 *   activation RGCN: sigma of Eq. (rgcn), RGNN_ACT_NONE or RGNN_ACT_RELU.
 *   flags      0, or a combination of RGNN_FLAG_* bits.  Each bit forces an alternative to a schedule or layout
 *              the library would otherwise pick for the graph (rgnn_schedule reports the pick); results agree
 *              within rounding, and all but the first are bit-reproducible.  They exist so that the choices can
 *              be compared on a given graph (thesis Ch.3: no schedule or layout fits every graph). */
/* single-head RGAT forward: the weighted sum over a destination's incoming edges is formed edge by edge with atomic
 * adds on the output rows (the thesis's traversal template, Alg. "traversal template": partial results are added
 * atomically to global memory) instead of by the destination-segment walk; the order of the additions then varies
 * from run to run.  Implies RGNN_FLAG_SEPARATE_SOFTMAX. */
#define RGNN_FLAG_EDGE_PARALLEL_AGGREGATION 1u
/* every segment takes the general walk: no batched kernels for the segments with one or with 2..4 entries */
#define RGNN_FLAG_NO_BATCHED_WALKS 2u
/* RGAT with 1, 2 or 4 heads (width <= 64), RGCN with bf16 rows: the gradient row of every (source, relation) pair is
 * written per pair, also for the pairs with one edge, instead of being read through the row selector */
#define RGNN_FLAG_NO_ROW_SELECT 4u
/* HGT: keep the key / message node linears and the per-relation matrices apart even when every relation's
 * sources have one node type (`saved` then holds the K and V rows as well) */
#define RGNN_FLAG_NO_WEIGHT_FOLDING 8u
/* single-head RGAT forward: source logit per pair as an epilogue of the typed linear, edge softmax as a pass of its
 * own that stores one attention weight per edge, then the weighted sum (three passes instead of the fused walk) */
#define RGNN_FLAG_SEPARATE_SOFTMAX 16u
/* backward calls: every gradient output is added to the buffer's contents instead of overwriting them (dX in the
 * kernel that writes it; the parameter gradients are formed in the workspace and added at the end, so
 * rgnn_workspace_bytes() asks for their size on top).  Forward calls ignore the bit. */
#define RGNN_FLAG_ACCUMULATE 32u
#define RGNN_FLAG_ALL 63u
typedef struct {
    int32_t dtype;
    int32_t d_in;
    int32_t d_out;
    int32_t heads;
    float slope;
    int32_t norm;
    int32_t activation;
    uint32_t flags;              /* 0, or RGNN_FLAG_* bits */
} rgnn_layer_desc_t;

/* Message of the last failing call made by this thread ("" if none). */
const char* rgnn_last_error(void);

/*
 * Build the graph index (dataset preprocessing in the thesis: "transposition,
 * converting COO to CSR", Ch.3 "Code Generation"; the compact-materialization
 * mapping is "precompute[d] ... in a CSR-like format").
 *
 *   format RGNN_COO:     a = src[E], b = dst[E]
 *   format RGNN_CSR_DST: a = col (source ids)[E], b = rowptr[N+1] over destinations
 *   rel[E]               relation (edge type) id in [0, num_rels)
 *   ntype[N]             node type id in [0, num_ntypes); may be NULL iff num_ntypes == 1
 *   rel_src_ntype[R], rel_dst_ntype[R]  optional (both or neither): when given, every
 *                        edge is checked to connect the node types its relation is tied to
 *   mem                  RGNN_MEM_HOST or RGNN_MEM_DEVICE: where ALL the input arrays live
 *
 * Edges may be in any order, with duplicates and self-loops.  The index is
 * canonical: destination-major CSR sorted by (dst, rel, src, input edge id);
 * pair ids are ranks in ascending (rel, src) order.
 * Streams: the build runs on the default (NULL) stream and the call returns only after
 * hipDeviceSynchronize(), so on return the index is complete and may be used by layer calls on
 * any stream without further ordering; work the caller has in flight on other streams is waited
 * for as well.  It is the one call that allocates device memory (freed by rgnn_graph_destroy).
 * Errors: EINVAL for NULLs / negative sizes / ids out of range / type mismatch,
 * EUNSUPPORTED for E >= 2^31 or N*N*R >= 2^63, ENOMEM, EHIP.  *g is NULL on failure.
 */
rgnn_status_t rgnn_graph_create(rgnn_graph_t** g, int64_t num_nodes, int32_t num_ntypes, int32_t num_rels,
                                int64_t num_edges, int32_t format, const int32_t* a, const int32_t* b,
                                const int32_t* rel, const int32_t* ntype, const int32_t* rel_src_ntype,
                                const int32_t* rel_dst_ntype, int32_t mem);

/* Free the graph and its device arrays.  NULL is accepted. */
rgnn_status_t rgnn_graph_destroy(rgnn_graph_t* g);

rgnn_status_t rgnn_graph_info(const rgnn_graph_t* g, rgnn_graph_info_t* out);

/* Index arrays that can be copied out (all int32) for bit-exact checks. */
enum {
    RGNN_IDX_IN_PTR = 0,      /* [N+1] CSR offsets by destination */
    RGNN_IDX_IN_SRC = 1,      /* [E] source of the CSR edge */
    RGNN_IDX_IN_REL = 2,      /* [E] relation of the CSR edge */
    RGNN_IDX_IN_EID = 3,      /* [E] input position of the CSR edge */
    RGNN_IDX_IN_PAIR = 4,     /* [E] pair id of the CSR edge */
    RGNN_IDX_IN_RUN = 5,      /* [E] run id ((dst, rel) group) of the CSR edge */
    RGNN_IDX_IN_CNT = 6,      /* [E] length of that run = c_{v,r} */
    RGNN_IDX_PAIR_PTR = 7,    /* [R+1] pairs of each relation (thesis: unique_etype_ptr) */
    RGNN_IDX_PAIR_SRC = 8,    /* [P] source node of the pair (thesis: unique_row_idx) */
    RGNN_IDX_PAIR_REL = 9,    /* [P] relation of the pair */
    RGNN_IDX_RUN_PTR = 10,    /* [Q+1] CSR edge range of each run */
    RGNN_IDX_RUN_DST = 11,    /* [Q] */
    RGNN_IDX_RUN_REL = 12,    /* [Q] */
    RGNN_IDX_DST_RUN_PTR = 13,/* [N+1] runs of each destination */
    RGNN_IDX_RELRUN_PTR = 14, /* [R+1] */
    RGNN_IDX_RELRUN_IDX = 15, /* [Q] run ids sorted by (rel, dst) */
    RGNN_IDX_OUT_PTR = 16,    /* [P+1] pair-major transpose offsets */
    RGNN_IDX_OUT_EPOS = 17,   /* [E] CSR position, sorted by (pair, CSR position) */
    RGNN_IDX_OUT_DST = 18,    /* [E] destination of that edge */
    RGNN_IDX_SRCPAIR_PTR = 19,/* [N+1] pairs of each source node */
    RGNN_IDX_SRCPAIR_IDX = 20,/* [P] pair ids sorted by (src, rel) */
    RGNN_IDX_NTYPE_PTR = 21,  /* [T+1] */
    RGNN_IDX_NTYPE_PERM = 22, /* [N] node ids sorted by (type, id) */
    RGNN_IDX_RELRUN_DST = 23, /* [Q] run_dst[relrun_idx[i]]: destinations in (rel, dst) order */
    RGNN_IDX_IN_PAIR_TAG = 24,/* [E] in_pair, with the top bit set when the pair has no other edge */
    RGNN_IDX_PAIR_SEL_DST = 25,/* [P] pair id, or for a pair with one edge: top bit | destination of that edge */
    RGNN_IDX_REL_SRC_TYPE = 26,/* [R] node type of the source of the relation's first pair (0 if it has no edge) */
    RGNN_IDX_COUNT = 27
};

/* Copy index array `which` to host memory.  `bytes` must equal 4 * its length,
 * else EINVAL.  Synchronises the device. */
rgnn_status_t rgnn_graph_export(const rgnn_graph_t* g, int32_t which, void* host_dst, size_t bytes);

/* Sizes (bytes) of the buffers the layer calls need: forward scratch, backward
 * scratch, and the `saved` buffer the forward fills for the backward.  Any out
 * pointer may be NULL. */
rgnn_status_t rgnn_workspace_bytes(const rgnn_graph_t* g, int32_t layer, const rgnn_layer_desc_t* desc,
                                   size_t* fwd_workspace, size_t* bwd_workspace, size_t* saved);

/* What the library picks for a layer configuration on a graph (1 = yes). */
typedef struct {
    int32_t item_len;            /* longest traversal item in edges: longer segments (hub nodes) are cut into pieces */
    int32_t tile_chunks;         /* workgroups of the typed-linear kernels over the pair tiles (short chunks) */
    int32_t wide_chunks;         /* the same tiles in one resident round of long chunks (fp32 kernels, weight gradients) */
    int32_t rows_bf16;           /* intermediate row tensors stored as bfloat16 */
    int32_t row_select;          /* single-edge pairs: gradient row read through the row selector, not materialised */
    int32_t hgt_folded;          /* HGT key / message linears folded into the per-relation weights */
    int32_t fused_softmax;       /* RGAT: edge softmax fused into the aggregation walk */
    int32_t ws_in_lds;           /* ... with w_s held in LDS */
    int32_t edge_parallel;       /* forward aggregation edge by edge with atomic adds */
    int32_t dst_batched_single;  /* destination-major walk: batched kernel phase for destinations with one edge */
    int32_t dst_batched_short;   /* ... and for those with 2..4 edges */
    int32_t pair_walk_multi_only;/* pair-major backward walk visits only the pairs with several edges */
    int32_t pair_batched_single; /* pair-major walk: batched phase for pairs with one edge */
    int32_t pair_batched_short;  /* ... and for those with 2..4 edges */
} rgnn_schedule_t;

/* The schedule and layout choices a call of `layer` with `desc` makes on this graph: from the statistics of the
 * graph index (item and segment counts, source types per relation), the descriptor (dtype, width, heads) and
 * desc.flags.  No device work.  Errors as rgnn_workspace_bytes. */
rgnn_status_t rgnn_schedule(const rgnn_graph_t* g, int32_t layer, const rgnn_layer_desc_t* desc, rgnn_schedule_t* out);

/*
 * RGCN (Eq. (rgcn)):  out[v] = act( X[v] W0 + sum_{e=(u->v,r)} (1/c_{v,r}) X[u] W[r] ).
 *   X [N, d_in]; W [R, d_in, d_out]; W0 [d_in, d_out] or NULL (no self-loop term);
 *   out [N, d_out].  Nodes without incoming edges get act(X[v] W0) (0 without W0).
 * Backward: given dOut [N, d_out] (gradient w.r.t. out) writes dX [N, d_in],
 *   dW [R, d_in, d_out], dW0 [d_in, d_out] (ignored when W0 is NULL).  `out` is the
 *   forward result (read only when activation != NONE).
 */
rgnn_status_t rgnn_rgcn_fwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X, const void* W,
                            const void* W0, void* out, void* saved, void* workspace, void* stream);
rgnn_status_t rgnn_rgcn_bwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X, const void* W,
                            const void* W0, const void* out, const void* saved, const void* dOut, void* dX,
                            void* dW, void* dW0, void* workspace, void* stream);

/*
 * RGAT (Ch.3 listing "attention calculation in a single-headed RGAT model"; the
 * message of an edge is hs):
 *   hs = X[u] W[r];  ht = X[v] W[r];  z_e = hs.w_s[r] + ht.w_t[r];
 *   att_e = softmax over ALL incoming edges of v of leakyrelu(z_e);
 *   out[v] = sum_{e in in(v)} att_e hs.
 *   X [N, d_in]; W [R, d_in, d_out]; w_s, w_t [R, d_out]; out [N, d_out].
 * With desc.heads = H > 1 the d_out columns form H slices of d_out/H; every head
 * applies the formulas above to its slice of hs, ht, w_s[r], w_t[r] (its own
 * logit, its own softmax) and the outputs are concatenated; tensor shapes are
 * unchanged.
 * Nodes without incoming edges get 0.
 * Backward writes dX [N, d_in], dW [R, d_in, d_out], dw_s, dw_t [R, d_out].
 * Layout of `saved` after the forward (exposed for tests), each part starting at a
 * multiple of 256 bytes: Hs [P, d_out] fp32, the compact messages; s_dst [Q, H] fp32,
 * the destination half ht . w_t[r] of the logit per (destination, relation) run and
 * head; ms [N, H, 2] fp32 = (max_e l_e, sum_e exp(l_e - max)) per head over the incoming
 * edges of each destination that has any, l_e = leakyrelu(z_e): the attention weight
 * of an edge is exp(l_e - m) / s and is recomputed by the backward call.
 */
rgnn_status_t rgnn_rgat_fwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X, const void* W,
                            const void* w_s, const void* w_t, void* out, void* saved, void* workspace,
                            void* stream);
rgnn_status_t rgnn_rgat_bwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X, const void* W,
                            const void* w_s, const void* w_t, const void* out, const void* saved,
                            const void* dOut, void* dX, void* dW, void* dw_s, void* dw_t, void* workspace,
                            void* stream);

/*
 * rgnn_rgat_fwd for callers that cannot allocate device memory or have no workspace to hand over: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, same kernels and
 * bit-identical results as rgnn_rgat_fwd, but the forward scratch is a buffer of RGNN_STATIC_SCRATCH_BYTES that
 * lives inside the library (one copy per GPU, held until the process ends) instead of a `workspace` argument.
 * The call allocates nothing.  X, W, w_s, w_t, out and `saved` are the caller's, as in rgnn_rgat_fwd; with
 * saved == NULL (inference) the tensors that would have been saved are placed in the static buffer as well.
 *   - The scratch a call needs is the forward size rgnn_workspace_bytes reports (plus, with saved == NULL, that
 *     size rounded up to 256 and the saved size); a call that needs more than RGNN_STATIC_SCRATCH_BYTES fails
 *     with RGNN_EWORKSPACE before anything is enqueued.
 *   - Every call on a GPU uses that GPU's one buffer: calls that overlap in time on one GPU (two streams, two
 *     threads) race; serialise them.  The buffer keeps the previous call's contents; no kernel of the forward
 *     reads scratch it has not written in the same call, so nothing has to be cleared.
 *   - The buffer's device address is looked up once per GPU, by rgnn_graph_create on the graph's GPU or else by
 *     the first call of this function there; make that first call outside a stream capture.
 */
#define RGNN_STATIC_SCRATCH_BYTES (64u << 20)
rgnn_status_t rgnn_rgat_fwd_static(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X, const void* W,
                                   const void* w_s, const void* w_t, void* out, void* saved, void* stream);

/*
 * HGT (caption of the figure "HGT and RGAT layer"): per node type tau(n) the
 * linears Wk, Wq, Wv, Wo [T, d, d]; per relation and head the attention and
 * message matrices Watt, Wmsg [R, H, dh, dh] (dh = d/H); optional prior mu [R, H]
 * (NULL = 1):
 *   k = X[u] Wk[tau(u)], q = X[v] Wq[tau(v)], val = X[u] Wv[tau(u)];
 *   logit_e^h = mu[r,h] ((k^h Watt[r,h]) . q^h) / sqrt(dh); att^h = edge softmax per head;
 *   out[v] = ( ||_h sum_e att_e^h (val^h Wmsg[r,h]) ) Wo[tau(v)].
 * Backward writes dX and the gradient of every weight (dmu ignored when mu is NULL).
 * When all sources of every relation have one node type (the usual heterogeneous
 * graph, where an edge type fixes its endpoint types; found when the graph is built,
 * with or without rel_src_ntype), k^h Watt[r,h] and val^h Wmsg[r,h] are computed as
 * X[u] (Wk[tau] Watt[r]) and X[u] (Wv[tau] Wmsg[r]) with the weight products formed
 * first (linear operator reordering, Ch.3 "Linear Operator Reordering"); the result
 * is the same up to rounding, and `saved` is smaller by the K and V rows.
 */
rgnn_status_t rgnn_hgt_fwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X, const void* Wk,
                           const void* Wq, const void* Wv, const void* Wo, const void* Watt, const void* Wmsg,
                           const void* mu, void* out, void* saved, void* workspace, void* stream);
rgnn_status_t rgnn_hgt_bwd(const rgnn_graph_t* g, const rgnn_layer_desc_t* desc, const void* X, const void* Wk,
                           const void* Wq, const void* Wv, const void* Wo, const void* Watt, const void* Wmsg,
                           const void* mu, const void* out, const void* saved, const void* dOut, void* dX,
                           void* dWk, void* dWq, void* dWv, void* dWo, void* dWatt, void* dWmsg, void* dmu,
                           void* workspace, void* stream);

/*
 * Per-kernel timing for benchmarks (not part of the layer definition).  Between
 * rgnn_profile_start() and rgnn_profile_stop() every kernel the layer calls launch is
 * bracketed by HIP events on the caller's stream.  rgnn_profile_stop() synchronises the
 * device and writes one text line per kernel name, "name launches total_ms\n", in first
 * launch order, into `report` (NUL-terminated, truncated at whole lines to fit
 * report_bytes).  Events are created on demand while profiling is on.
 */
rgnn_status_t rgnn_profile_start(void);
rgnn_status_t rgnn_profile_stop(char* report, size_t report_bytes);
/* Restricts the timing to the kernels launched under one name (a host string of at most 63 characters, copied), so
 * that a timed run carries two events per step instead of two per kernel; NULL or "" times every kernel again.
 * Takes effect at the next rgnn_profile_start().  RGNN_EINVAL if the name is too long. */
rgnn_status_t rgnn_profile_select(const char* name);

#ifdef __cplusplus
}
#endif
#endif /* RGNN_H */
