/*
 * CPU oracle for one relational-GNN layer (RGCN, RGAT, HGT), forward and
 * backward.  TEST INFRASTRUCTURE ONLY: it exists to check the HIP library and
 * to be timed beside it as a baseline.  Nothing on the product path may call
 * it, and it shares no code with the HIP path.
 *
 * Every routine is the plain per-edge ("vanilla") definition of the layer in
 * double precision: one message per edge, no compaction, no operator
 * reordering, no blocking.  OpenMP is used only on loops whose iterations own
 * disjoint outputs (destination nodes, source nodes) or, for the parameter
 * gradients, with one private accumulator per thread that is summed at the
 * end.
 *
 * Definitions followed:
 *   RGCN  - thesis Ch.3 "RGNN Formulation and Operators", Eq. (rgcn):
 *           h'_v = sigma( h_v W_0 + sum_r sum_{u in N_v^r} (1/c_{v,r}) h_u W_r )
 *   RGAT  - Ch.3 listing "attention calculation in a single-headed RGAT model"
 *           (hs, atts, ht, attt, leakyrelu, edge_softmax over incoming edges)
 *           and the caption of the figure "HGT and RGAT layer"; the message of
 *           an edge is hs (figure "RGAT edge message computation").
 *   HGT   - same caption: node-type weights W_{tau(n)} (K, Q, V, output),
 *           edge-type weights W_{a,tau(e)} (attention) and W_{m,tau(e)}
 *           (message); attention is an edgewise dot product; msg depends only
 *           on (source node, edge type).
 * Readings where the text is silent: softmax is over all incoming edges of a
 * node regardless of relation and is evaluated in the max-subtracted form;
 * leaky-ReLU derivative at 0 is the negative-side slope; c_{v,r} is the
 * number of incoming edges of v with relation r (multi-edges counted);
 * a node with no incoming edge aggregates the zero vector; HGT keeps the
 * 1/sqrt(d_head) scale and an optional per-(relation, head) prior mu, and has
 * no GELU / skip connection.
 *
 * Parity status: every routine here is pinned by tests/test_oracle_*.py
 * (sparse-matrix closed forms, hand-computed examples, invariants, dense
 * attention special case, central finite differences).  No value printed in
 * the thesis is usable as a pin (it prints speed-ups only).
 *
 * Layouts: all matrices row-major doubles.  X[N][d_in]; W[R][d_in][d_out]
 * (y = x W); edges in COO (src, dst, rel), any order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#else
static int omp_get_max_threads(void) { return 1; }
static int omp_get_thread_num(void) { return 0; }
#endif

int oracle_num_threads(void) { return omp_get_max_threads(); }

/* y[0..n) = x[0..k) * W[k][n] */
static void vec_mat(const double *x, const double *W, int k, int n, double *y) {
    for (int j = 0; j < n; ++j) y[j] = 0.0;
    for (int i = 0; i < k; ++i) {
        const double xi = x[i];
        const double *w = W + (size_t)i * n;
        for (int j = 0; j < n; ++j) y[j] += xi * w[j];
    }
}
/* x[0..k) += y[0..n) * W^T, W[k][n] */
static void vec_matT_acc(const double *y, const double *W, int k, int n, double *x) {
    for (int i = 0; i < k; ++i) {
        const double *w = W + (size_t)i * n;
        double s = 0.0;
        for (int j = 0; j < n; ++j) s += y[j] * w[j];
        x[i] += s;
    }
}
/* G[k][n] += x^T y */
static void outer_acc(const double *x, const double *y, int k, int n, double *G) {
    for (int i = 0; i < k; ++i) {
        const double xi = x[i];
        double *g = G + (size_t)i * n;
        for (int j = 0; j < n; ++j) g[j] += xi * y[j];
    }
}
static double dot(const double *a, const double *b, int n) {
    double s = 0.0;
    for (int j = 0; j < n; ++j) s += a[j] * b[j];
    return s;
}

/* out[i] = sum over the nt per-thread copies part[k*sz + i]; out may be NULL. */
static void reduce_parts(double *out, const double *part, size_t sz, int nt) {
    if (!out) return;
    for (size_t i = 0; i < sz; ++i) {
        double s = 0.0;
        for (int k = 0; k < nt; ++k) s += part[sz * k + i];
        out[i] = s;
    }
}

/* Adjacency lists by `key` (dst or src), edges kept in input order. */
static void bucket_edges(int64_t N, int64_t E, const int32_t *key, int64_t **ptr_out, int64_t **list_out) {
    int64_t *ptr = (int64_t *)calloc((size_t)N + 1, sizeof(int64_t));
    int64_t *list = (int64_t *)malloc(sizeof(int64_t) * (size_t)(E > 0 ? E : 1));
    for (int64_t e = 0; e < E; ++e) ptr[key[e] + 1]++;
    for (int64_t v = 0; v < N; ++v) ptr[v + 1] += ptr[v];
    int64_t *fill = (int64_t *)malloc(sizeof(int64_t) * (size_t)(N > 0 ? N : 1));
    memcpy(fill, ptr, sizeof(int64_t) * (size_t)N);
    for (int64_t e = 0; e < E; ++e) list[fill[key[e]]++] = e;
    free(fill);
    *ptr_out = ptr;
    *list_out = list;
}

static int64_t max_degree(int64_t N, const int64_t *ptr) {
    int64_t m = 0;
    for (int64_t v = 0; v < N; ++v)
        if (ptr[v + 1] - ptr[v] > m) m = ptr[v + 1] - ptr[v];
    return m;
}

/* ------------------------------------------------------------------ RGCN */

/* c_{v,r} for edge e: number of incoming edges of dst[e] with relation rel[e]
 * (norm = 1), or 1 (norm = 0). */
static double *rgcn_edge_norm(int64_t N, int64_t E, const int32_t *dst, const int32_t *rel, int norm,
                              const int64_t *in_ptr, const int64_t *in_list) {
    double *c = (double *)malloc(sizeof(double) * (size_t)(E > 0 ? E : 1));
    for (int64_t e = 0; e < E; ++e) c[e] = 1.0;
    if (!norm) return c;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < N; ++v) {
        for (int64_t a = in_ptr[v]; a < in_ptr[v + 1]; ++a) {
            int64_t cnt = 0;
            for (int64_t b = in_ptr[v]; b < in_ptr[v + 1]; ++b)
                if (rel[in_list[b]] == rel[in_list[a]]) cnt++;
            c[in_list[a]] = (double)cnt;
        }
    }
    (void)dst;
    return c;
}

/* out[v] = act( x_v W0 + sum_{e=(u->v,r)} (1/c_{v,r}) x_u W_r ); W0 may be NULL.
 * act: 0 none, 1 ReLU. */
void oracle_rgcn_fwd(int64_t N, int64_t E, int32_t R, int32_t d_in, int32_t d_out,
                     const int32_t *src, const int32_t *dst, const int32_t *rel,
                     const double *X, const double *W, const double *W0, int32_t norm, int32_t act,
                     double *out) {
    int64_t *in_ptr, *in_list;
    bucket_edges(N, E, dst, &in_ptr, &in_list);
    double *c = rgcn_edge_norm(N, E, dst, rel, norm, in_ptr, in_list);
    (void)R;
#pragma omp parallel
    {
        double *msg = (double *)malloc(sizeof(double) * (size_t)d_out);
#pragma omp for schedule(dynamic, 64)
        for (int64_t v = 0; v < N; ++v) {
            double *o = out + (size_t)v * d_out;
            if (W0) vec_mat(X + (size_t)v * d_in, W0, d_in, d_out, o);
            else for (int j = 0; j < d_out; ++j) o[j] = 0.0;
            for (int64_t a = in_ptr[v]; a < in_ptr[v + 1]; ++a) {
                const int64_t e = in_list[a];
                vec_mat(X + (size_t)src[e] * d_in, W + (size_t)rel[e] * d_in * d_out, d_in, d_out, msg);
                for (int j = 0; j < d_out; ++j) o[j] += msg[j] / c[e];
            }
            if (act == 1) for (int j = 0; j < d_out; ++j) o[j] = o[j] > 0.0 ? o[j] : 0.0;
        }
        free(msg);
    }
    free(c); free(in_ptr); free(in_list);
}

/* Gradients of <out, dOut> w.r.t. X, W, W0.  `out` (the forward result) is
 * needed only for act = ReLU.  dW0 may be NULL iff W0 is NULL. */
void oracle_rgcn_bwd(int64_t N, int64_t E, int32_t R, int32_t d_in, int32_t d_out,
                     const int32_t *src, const int32_t *dst, const int32_t *rel,
                     const double *X, const double *W, const double *W0, int32_t norm, int32_t act,
                     const double *out, const double *dOut,
                     double *dX, double *dW, double *dW0) {
    int64_t *in_ptr, *in_list, *out_ptr, *out_list;
    bucket_edges(N, E, dst, &in_ptr, &in_list);
    bucket_edges(N, E, src, &out_ptr, &out_list);
    double *c = rgcn_edge_norm(N, E, dst, rel, norm, in_ptr, in_list);
    /* gradient at the pre-activation */
    double *dPre = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1) * d_out);
    for (int64_t i = 0; i < N * (int64_t)d_out; ++i)
        dPre[i] = (act == 1 && !(out[i] > 0.0)) ? 0.0 : dOut[i];
    const size_t wsz = (size_t)R * d_in * d_out, w0sz = (size_t)d_in * d_out;
    const int nt = omp_get_max_threads();
    double *dWp = (double *)calloc(wsz * nt, sizeof(double));
    double *dW0p = (double *)calloc(w0sz * nt, sizeof(double));
#pragma omp parallel
    {
        double *t = (double *)malloc(sizeof(double) * (size_t)d_out);
        /* dX[u]: self-loop term plus one term per outgoing edge of u */
#pragma omp for schedule(dynamic, 64)
        for (int64_t u = 0; u < N; ++u) {
            double *dx = dX + (size_t)u * d_in;
            for (int i = 0; i < d_in; ++i) dx[i] = 0.0;
            if (W0) vec_matT_acc(dPre + (size_t)u * d_out, W0, d_in, d_out, dx);
            for (int64_t a = out_ptr[u]; a < out_ptr[u + 1]; ++a) {
                const int64_t e = out_list[a];
                for (int j = 0; j < d_out; ++j) t[j] = dPre[(size_t)dst[e] * d_out + j] / c[e];
                vec_matT_acc(t, W + (size_t)rel[e] * d_in * d_out, d_in, d_out, dx);
            }
        }
        /* dW_r += (1/c) x_u^T dPre[v] per edge; dW0 += x_v^T dPre[v] per node */
        double *myW = dWp + wsz * omp_get_thread_num();
        double *myW0 = dW0p + w0sz * omp_get_thread_num();
#pragma omp for schedule(static)
        for (int64_t e = 0; e < E; ++e) {
            for (int j = 0; j < d_out; ++j) t[j] = dPre[(size_t)dst[e] * d_out + j] / c[e];
            outer_acc(X + (size_t)src[e] * d_in, t, d_in, d_out, myW + (size_t)rel[e] * d_in * d_out);
        }
        if (W0) {
#pragma omp for schedule(static)
            for (int64_t v = 0; v < N; ++v)
                outer_acc(X + (size_t)v * d_in, dPre + (size_t)v * d_out, d_in, d_out, myW0);
        }
        free(t);
    }
    for (size_t i = 0; i < wsz; ++i) { double s = 0.0; for (int k = 0; k < nt; ++k) s += dWp[wsz * k + i]; dW[i] = s; }
    if (W0 && dW0)
        for (size_t i = 0; i < w0sz; ++i) { double s = 0.0; for (int k = 0; k < nt; ++k) s += dW0p[w0sz * k + i]; dW0[i] = s; }
    free(dWp); free(dW0p); free(dPre); free(c);
    free(in_ptr); free(in_list); free(out_ptr); free(out_list);
}

/* ------------------------------------------------------------------ RGAT */

/* Per destination v: logits z_e, attention alpha_e over incoming edges, and
 * (optionally) the messages hs_e.  hs must hold deg*d_out doubles. */
static void rgat_node_attention(int64_t v, const int64_t *in_ptr, const int64_t *in_list,
                                const int32_t *src, const int32_t *rel,
                                int32_t d_in, int32_t d_out,
                                const double *X, const double *W, const double *w_s, const double *w_t,
                                double slope, double *hs, double *ht, double *z, double *alpha) {
    const int64_t b = in_ptr[v], deg = in_ptr[v + 1] - b;
    for (int64_t a = 0; a < deg; ++a) {
        const int64_t e = in_list[b + a];
        const double *Wr = W + (size_t)rel[e] * d_in * d_out;
        vec_mat(X + (size_t)src[e] * d_in, Wr, d_in, d_out, hs + (size_t)a * d_out);   /* hs = e.src.feature * W[etype] */
        const double atts = dot(hs + (size_t)a * d_out, w_s + (size_t)rel[e] * d_out, d_out);
        vec_mat(X + (size_t)v * d_in, Wr, d_in, d_out, ht);                             /* ht = e.dst.feature * W[etype] */
        const double attt = dot(ht, w_t + (size_t)rel[e] * d_out, d_out);
        z[a] = atts + attt;
    }
    /* edge softmax of leakyrelu(z) over the incoming edges of v */
    double m = -INFINITY, sum = 0.0;
    for (int64_t a = 0; a < deg; ++a) {
        const double l = z[a] > 0.0 ? z[a] : slope * z[a];
        alpha[a] = l;
        if (l > m) m = l;
    }
    for (int64_t a = 0; a < deg; ++a) { alpha[a] = exp(alpha[a] - m); sum += alpha[a]; }
    for (int64_t a = 0; a < deg; ++a) alpha[a] /= sum;
}

/* out[v] = sum_{e in in(v)} alpha_e * hs_e.  alpha_out / z_out (length E,
 * indexed by input edge id) may be NULL. */
void oracle_rgat_fwd(int64_t N, int64_t E, int32_t R, int32_t d_in, int32_t d_out,
                     const int32_t *src, const int32_t *dst, const int32_t *rel,
                     const double *X, const double *W, const double *w_s, const double *w_t, double slope,
                     double *out, double *alpha_out, double *z_out) {
    int64_t *in_ptr, *in_list;
    bucket_edges(N, E, dst, &in_ptr, &in_list);
    const int64_t md = max_degree(N, in_ptr);
    (void)R;
#pragma omp parallel
    {
        double *hs = (double *)malloc(sizeof(double) * (size_t)(md > 0 ? md : 1) * d_out);
        double *ht = (double *)malloc(sizeof(double) * (size_t)d_out);
        double *z = (double *)malloc(sizeof(double) * (size_t)(md > 0 ? md : 1));
        double *al = (double *)malloc(sizeof(double) * (size_t)(md > 0 ? md : 1));
#pragma omp for schedule(dynamic, 16)
        for (int64_t v = 0; v < N; ++v) {
            double *o = out + (size_t)v * d_out;
            for (int j = 0; j < d_out; ++j) o[j] = 0.0;
            const int64_t deg = in_ptr[v + 1] - in_ptr[v];
            if (deg == 0) continue;
            rgat_node_attention(v, in_ptr, in_list, src, rel, d_in, d_out, X, W, w_s, w_t, slope, hs, ht, z, al);
            for (int64_t a = 0; a < deg; ++a) {
                for (int j = 0; j < d_out; ++j) o[j] += al[a] * hs[(size_t)a * d_out + j];
                if (alpha_out) alpha_out[in_list[in_ptr[v] + a]] = al[a];
                if (z_out) z_out[in_list[in_ptr[v] + a]] = z[a];
            }
        }
        free(hs); free(ht); free(z); free(al);
    }
    free(in_ptr); free(in_list);
}

/* Gradients of <out, dOut> w.r.t. X, W, w_s, w_t (chain rule through the
 * forward above):
 *   g_e = dOut[v].hs_e ; dl_e = alpha_e (g_e - sum_e' alpha_e' g_e') ;
 *   dz_e = dl_e * (z_e > 0 ? 1 : slope) ;
 *   dhs_e = alpha_e dOut[v] + dz_e w_s[r] ; dht_e = dz_e w_t[r] ;
 *   dw_s[r] += dz_e hs_e ; dw_t[r] += dz_e ht_e ;
 *   dW_r += x_u^T dhs_e + x_v^T dht_e ; dX[u] += dhs_e W_r^T ; dX[v] += dht_e W_r^T. */
void oracle_rgat_bwd(int64_t N, int64_t E, int32_t R, int32_t d_in, int32_t d_out,
                     const int32_t *src, const int32_t *dst, const int32_t *rel,
                     const double *X, const double *W, const double *w_s, const double *w_t, double slope,
                     const double *dOut,
                     double *dX, double *dW, double *dw_s, double *dw_t) {
    int64_t *in_ptr, *in_list, *out_ptr, *out_list;
    bucket_edges(N, E, dst, &in_ptr, &in_list);
    bucket_edges(N, E, src, &out_ptr, &out_list);
    const int64_t md = max_degree(N, in_ptr);
    double *alpha = (double *)malloc(sizeof(double) * (size_t)(E > 0 ? E : 1));
    double *dz = (double *)malloc(sizeof(double) * (size_t)(E > 0 ? E : 1));
    const size_t wsz = (size_t)R * d_in * d_out, vsz = (size_t)R * d_out;
    const int nt = omp_get_max_threads();
    double *dWp = (double *)calloc(wsz * nt, sizeof(double));
    double *dsp = (double *)calloc(vsz * nt, sizeof(double));
    double *dtp = (double *)calloc(vsz * nt, sizeof(double));
#pragma omp parallel
    {
        double *hs = (double *)malloc(sizeof(double) * (size_t)(md > 0 ? md : 1) * d_out);
        double *ht = (double *)malloc(sizeof(double) * (size_t)d_out);
        double *z = (double *)malloc(sizeof(double) * (size_t)(md > 0 ? md : 1));
        double *al = (double *)malloc(sizeof(double) * (size_t)(md > 0 ? md : 1));
        double *t = (double *)malloc(sizeof(double) * (size_t)d_out);
        /* pass 1, per destination: alpha_e and dz_e */
#pragma omp for schedule(dynamic, 16)
        for (int64_t v = 0; v < N; ++v) {
            const int64_t b = in_ptr[v], deg = in_ptr[v + 1] - b;
            if (deg == 0) continue;
            rgat_node_attention(v, in_ptr, in_list, src, rel, d_in, d_out, X, W, w_s, w_t, slope, hs, ht, z, al);
            const double *go = dOut + (size_t)v * d_out;
            double gbar = 0.0;
            for (int64_t a = 0; a < deg; ++a) gbar += al[a] * dot(go, hs + (size_t)a * d_out, d_out);
            for (int64_t a = 0; a < deg; ++a) {
                const double g = dot(go, hs + (size_t)a * d_out, d_out);
                const double dl = al[a] * (g - gbar);
                alpha[in_list[b + a]] = al[a];
                dz[in_list[b + a]] = dl * (z[a] > 0.0 ? 1.0 : slope);
            }
        }
        /* pass 2, per node n: dX[n] = sum over outgoing edges dhs_e W_r^T + sum over incoming edges dht_e W_r^T */
#pragma omp for schedule(dynamic, 16)
        for (int64_t n = 0; n < N; ++n) {
            double *dx = dX + (size_t)n * d_in;
            for (int i = 0; i < d_in; ++i) dx[i] = 0.0;
            for (int64_t a = out_ptr[n]; a < out_ptr[n + 1]; ++a) {
                const int64_t e = out_list[a];
                for (int j = 0; j < d_out; ++j)
                    t[j] = alpha[e] * dOut[(size_t)dst[e] * d_out + j] + dz[e] * w_s[(size_t)rel[e] * d_out + j];
                vec_matT_acc(t, W + (size_t)rel[e] * d_in * d_out, d_in, d_out, dx);
            }
            for (int64_t a = in_ptr[n]; a < in_ptr[n + 1]; ++a) {
                const int64_t e = in_list[a];
                for (int j = 0; j < d_out; ++j) t[j] = dz[e] * w_t[(size_t)rel[e] * d_out + j];
                vec_matT_acc(t, W + (size_t)rel[e] * d_in * d_out, d_in, d_out, dx);
            }
        }
        /* pass 3, per edge: parameter gradients (private accumulators per thread) */
        double *myW = dWp + wsz * omp_get_thread_num();
        double *mys = dsp + vsz * omp_get_thread_num();
        double *myt = dtp + vsz * omp_get_thread_num();
#pragma omp for schedule(static)
        for (int64_t e = 0; e < E; ++e) {
            const int32_t r = rel[e];
            const double *Wr = W + (size_t)r * d_in * d_out;
            const double *xu = X + (size_t)src[e] * d_in, *xv = X + (size_t)dst[e] * d_in;
            vec_mat(xu, Wr, d_in, d_out, hs);
            vec_mat(xv, Wr, d_in, d_out, ht);
            for (int j = 0; j < d_out; ++j) {
                mys[(size_t)r * d_out + j] += dz[e] * hs[j];
                myt[(size_t)r * d_out + j] += dz[e] * ht[j];
            }
            for (int j = 0; j < d_out; ++j)
                t[j] = alpha[e] * dOut[(size_t)dst[e] * d_out + j] + dz[e] * w_s[(size_t)r * d_out + j];
            outer_acc(xu, t, d_in, d_out, myW + (size_t)r * d_in * d_out);
            for (int j = 0; j < d_out; ++j) t[j] = dz[e] * w_t[(size_t)r * d_out + j];
            outer_acc(xv, t, d_in, d_out, myW + (size_t)r * d_in * d_out);
        }
        free(hs); free(ht); free(z); free(al); free(t);
    }
    for (size_t i = 0; i < wsz; ++i) { double s = 0.0; for (int k = 0; k < nt; ++k) s += dWp[wsz * k + i]; dW[i] = s; }
    for (size_t i = 0; i < vsz; ++i) {
        double s = 0.0, u = 0.0;
        for (int k = 0; k < nt; ++k) { s += dsp[vsz * k + i]; u += dtp[vsz * k + i]; }
        dw_s[i] = s; dw_t[i] = u;
    }
    free(dWp); free(dsp); free(dtp); free(alpha); free(dz);
    free(in_ptr); free(in_list); free(out_ptr); free(out_list);
}

/* ------------------------------------------------------------------- HGT */

/* K, Q, V of every node: k_n = x_n W^K_{tau(n)} etc. (d = H*dh columns, head h
 * is columns [h*dh, (h+1)*dh)). */
static void hgt_node_kqv(int64_t N, int32_t d, const int32_t *ntype, const double *X,
                         const double *Wk, const double *Wq, const double *Wv,
                         double *K, double *Q, double *V) {
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const size_t t = (size_t)(ntype ? ntype[n] : 0) * d * d;
        vec_mat(X + (size_t)n * d, Wk + t, d, d, K + (size_t)n * d);
        vec_mat(X + (size_t)n * d, Wq + t, d, d, Q + (size_t)n * d);
        vec_mat(X + (size_t)n * d, Wv + t, d, d, V + (size_t)n * d);
    }
}

/* For destination v: raw scores s[a][h] = (k_u^h W^att_{r,h}) . q_v^h, attention
 * alpha[a][h] (softmax over incoming edges, per head, of mu*s/sqrt(dh)) and
 * messages msg[a] = ||_h v_u^h W^msg_{r,h}.  ka[a] keeps k_u^h W^att_{r,h}. */
static void hgt_node_attention(int64_t v, const int64_t *in_ptr, const int64_t *in_list,
                               const int32_t *src, const int32_t *rel, int32_t d, int32_t H,
                               const double *K, const double *Q, const double *V,
                               const double *Watt, const double *Wmsg, const double *mu,
                               double *ka, double *msg, double *s, double *alpha) {
    const int dh = d / H;
    const double scale = 1.0 / sqrt((double)dh);
    const int64_t b = in_ptr[v], deg = in_ptr[v + 1] - b;
    for (int64_t a = 0; a < deg; ++a) {
        const int64_t e = in_list[b + a];
        const int32_t u = src[e], r = rel[e];
        for (int h = 0; h < H; ++h) {
            const size_t wo = ((size_t)r * H + h) * dh * dh;
            vec_mat(K + (size_t)u * d + h * dh, Watt + wo, dh, dh, ka + (size_t)a * d + h * dh);
            vec_mat(V + (size_t)u * d + h * dh, Wmsg + wo, dh, dh, msg + (size_t)a * d + h * dh);
            s[a * H + h] = dot(ka + (size_t)a * d + h * dh, Q + (size_t)v * d + h * dh, dh);
        }
    }
    for (int h = 0; h < H; ++h) {
        double m = -INFINITY, sum = 0.0;
        for (int64_t a = 0; a < deg; ++a) {
            const int32_t r = rel[in_list[b + a]];
            const double l = (mu ? mu[(size_t)r * H + h] : 1.0) * s[a * H + h] * scale;
            alpha[a * H + h] = l;
            if (l > m) m = l;
        }
        for (int64_t a = 0; a < deg; ++a) { alpha[a * H + h] = exp(alpha[a * H + h] - m); sum += alpha[a * H + h]; }
        for (int64_t a = 0; a < deg; ++a) alpha[a * H + h] /= sum;
    }
}

/* out_v = ( ||_h sum_{e in in(v)} alpha_e^h m_e^h ) W^out_{tau(v)}.
 * ntype may be NULL (single node type); mu may be NULL (all ones);
 * alpha_out (E*H, by input edge id) may be NULL. */
void oracle_hgt_fwd(int64_t N, int64_t E, int32_t T, int32_t R, int32_t d, int32_t H,
                    const int32_t *src, const int32_t *dst, const int32_t *rel, const int32_t *ntype,
                    const double *X, const double *Wk, const double *Wq, const double *Wv, const double *Wo,
                    const double *Watt, const double *Wmsg, const double *mu,
                    double *out, double *alpha_out) {
    int64_t *in_ptr, *in_list;
    bucket_edges(N, E, dst, &in_ptr, &in_list);
    const int64_t md = max_degree(N, in_ptr);
    const size_t nd = (size_t)(N > 0 ? N : 1) * d, mdd = (size_t)(md > 0 ? md : 1);
    double *K = (double *)malloc(sizeof(double) * nd), *Q = (double *)malloc(sizeof(double) * nd),
           *V = (double *)malloc(sizeof(double) * nd);
    hgt_node_kqv(N, d, ntype, X, Wk, Wq, Wv, K, Q, V);
    (void)T; (void)R;
#pragma omp parallel
    {
        double *ka = (double *)malloc(sizeof(double) * mdd * d), *msg = (double *)malloc(sizeof(double) * mdd * d);
        double *s = (double *)malloc(sizeof(double) * mdd * H), *al = (double *)malloc(sizeof(double) * mdd * H);
        double *zv = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 16)
        for (int64_t v = 0; v < N; ++v) {
            const int64_t deg = in_ptr[v + 1] - in_ptr[v];
            for (int j = 0; j < d; ++j) zv[j] = 0.0;
            if (deg > 0) {
                hgt_node_attention(v, in_ptr, in_list, src, rel, d, H, K, Q, V, Watt, Wmsg, mu, ka, msg, s, al);
                const int dh = d / H;
                for (int64_t a = 0; a < deg; ++a)
                    for (int h = 0; h < H; ++h) {
                        for (int j = 0; j < dh; ++j) zv[h * dh + j] += al[a * H + h] * msg[(size_t)a * d + h * dh + j];
                        if (alpha_out) alpha_out[(size_t)in_list[in_ptr[v] + a] * H + h] = al[a * H + h];
                    }
            }
            vec_mat(zv, Wo + (size_t)(ntype ? ntype[v] : 0) * d * d, d, d, out + (size_t)v * d);
        }
        free(ka); free(msg); free(s); free(al); free(zv);
    }
    free(K); free(Q); free(V); free(in_ptr); free(in_list);
}

/* Gradients of <out, dOut> w.r.t. X and every weight; dmu may be NULL. */
void oracle_hgt_bwd(int64_t N, int64_t E, int32_t T, int32_t R, int32_t d, int32_t H,
                    const int32_t *src, const int32_t *dst, const int32_t *rel, const int32_t *ntype,
                    const double *X, const double *Wk, const double *Wq, const double *Wv, const double *Wo,
                    const double *Watt, const double *Wmsg, const double *mu, const double *dOut,
                    double *dX, double *dWk, double *dWq, double *dWv, double *dWo,
                    double *dWatt, double *dWmsg, double *dmu) {
    const int dh = d / H;
    const double scale = 1.0 / sqrt((double)dh);
    int64_t *in_ptr, *in_list, *out_ptr, *out_list;
    bucket_edges(N, E, dst, &in_ptr, &in_list);
    bucket_edges(N, E, src, &out_ptr, &out_list);
    const int64_t md = max_degree(N, in_ptr);
    const size_t nd = (size_t)(N > 0 ? N : 1) * d, mdd = (size_t)(md > 0 ? md : 1), eh = (size_t)(E > 0 ? E : 1) * H;
    double *K = (double *)malloc(sizeof(double) * nd), *Q = (double *)malloc(sizeof(double) * nd),
           *V = (double *)malloc(sizeof(double) * nd);
    double *dK = (double *)calloc(nd, sizeof(double)), *dQ = (double *)calloc(nd, sizeof(double)),
           *dV = (double *)calloc(nd, sizeof(double)), *dZ = (double *)calloc(nd, sizeof(double)),
           *Z = (double *)calloc(nd, sizeof(double));
    double *alpha = (double *)malloc(sizeof(double) * eh), *ds = (double *)malloc(sizeof(double) * eh),
           *sraw = (double *)malloc(sizeof(double) * eh);
    hgt_node_kqv(N, d, ntype, X, Wk, Wq, Wv, K, Q, V);
    const size_t tsz = (size_t)T * d * d, rsz = (size_t)R * H * dh * dh, msz = (size_t)R * H;
    const int nt = omp_get_max_threads();
    double *pk = (double *)calloc(tsz * nt, sizeof(double)), *pq = (double *)calloc(tsz * nt, sizeof(double)),
           *pv = (double *)calloc(tsz * nt, sizeof(double)), *po = (double *)calloc(tsz * nt, sizeof(double)),
           *pa = (double *)calloc(rsz * nt, sizeof(double)), *pm = (double *)calloc(rsz * nt, sizeof(double)),
           *pu = (double *)calloc(msz * nt, sizeof(double));
#pragma omp parallel
    {
        const int me = omp_get_thread_num();
        double *ka = (double *)malloc(sizeof(double) * mdd * d), *msg = (double *)malloc(sizeof(double) * mdd * d);
        double *s = (double *)malloc(sizeof(double) * mdd * H), *al = (double *)malloc(sizeof(double) * mdd * H);
        double *t = (double *)malloc(sizeof(double) * (size_t)d), *t2 = (double *)malloc(sizeof(double) * (size_t)d);
        /* pass 1, per destination v: Z_v, dZ_v = dOut_v Wo^T, alpha, d(score), dQ_v */
#pragma omp for schedule(dynamic, 16)
        for (int64_t v = 0; v < N; ++v) {
            const int64_t b = in_ptr[v], deg = in_ptr[v + 1] - b;
            double *dz = dZ + (size_t)v * d, *z = Z + (size_t)v * d;
            vec_matT_acc(dOut + (size_t)v * d, Wo + (size_t)(ntype ? ntype[v] : 0) * d * d, d, d, dz);
            if (deg == 0) continue;
            hgt_node_attention(v, in_ptr, in_list, src, rel, d, H, K, Q, V, Watt, Wmsg, mu, ka, msg, s, al);
            for (int h = 0; h < H; ++h) {
                double gbar = 0.0;
                for (int64_t a = 0; a < deg; ++a) {
                    for (int j = 0; j < dh; ++j) z[h * dh + j] += al[a * H + h] * msg[(size_t)a * d + h * dh + j];
                    gbar += al[a * H + h] * dot(dz + h * dh, msg + (size_t)a * d + h * dh, dh);
                }
                for (int64_t a = 0; a < deg; ++a) {
                    const int64_t e = in_list[b + a];
                    const double g = dot(dz + h * dh, msg + (size_t)a * d + h * dh, dh);
                    const double dl = al[a * H + h] * (g - gbar);                 /* d/d logit */
                    const double m_ = mu ? mu[(size_t)rel[e] * H + h] : 1.0;
                    alpha[(size_t)e * H + h] = al[a * H + h];
                    sraw[(size_t)e * H + h] = s[a * H + h];
                    ds[(size_t)e * H + h] = dl * m_ * scale;                      /* d/d raw score */
                    for (int j = 0; j < dh; ++j) dQ[(size_t)v * d + h * dh + j] += ds[(size_t)e * H + h] * ka[(size_t)a * d + h * dh + j];
                }
            }
        }
        /* pass 2, per source u: dK_u, dV_u over outgoing edges */
#pragma omp for schedule(dynamic, 16)
        for (int64_t u = 0; u < N; ++u) {
            for (int64_t a = out_ptr[u]; a < out_ptr[u + 1]; ++a) {
                const int64_t e = out_list[a];
                const int32_t v = dst[e], r = rel[e];
                for (int h = 0; h < H; ++h) {
                    const size_t wo = ((size_t)r * H + h) * dh * dh;
                    for (int j = 0; j < dh; ++j) {
                        t[j] = ds[(size_t)e * H + h] * Q[(size_t)v * d + h * dh + j];          /* d ka */
                        t2[j] = alpha[(size_t)e * H + h] * dZ[(size_t)v * d + h * dh + j];     /* d msg */
                    }
                    vec_matT_acc(t, Watt + wo, dh, dh, dK + (size_t)u * d + h * dh);
                    vec_matT_acc(t2, Wmsg + wo, dh, dh, dV + (size_t)u * d + h * dh);
                }
            }
        }
        /* pass 3, per edge: dWatt, dWmsg, dmu */
#pragma omp for schedule(static)
        for (int64_t e = 0; e < E; ++e) {
            const int32_t u = src[e], v = dst[e], r = rel[e];
            for (int h = 0; h < H; ++h) {
                const size_t wo = ((size_t)r * H + h) * dh * dh;
                for (int j = 0; j < dh; ++j) {
                    t[j] = ds[(size_t)e * H + h] * Q[(size_t)v * d + h * dh + j];
                    t2[j] = alpha[(size_t)e * H + h] * dZ[(size_t)v * d + h * dh + j];
                }
                outer_acc(K + (size_t)u * d + h * dh, t, dh, dh, pa + rsz * me + wo);
                outer_acc(V + (size_t)u * d + h * dh, t2, dh, dh, pm + rsz * me + wo);
                /* logit = mu * s * scale  =>  d logit / d mu = s * scale; d logit = ds / (mu*scale) */
                const double m_ = mu ? mu[(size_t)r * H + h] : 1.0;
                const double dl = (m_ != 0.0) ? ds[(size_t)e * H + h] / (m_ * scale) : 0.0;
                pu[msz * me + (size_t)r * H + h] += dl * sraw[(size_t)e * H + h] * scale;
            }
        }
        /* pass 4, per node: dX and the node-type weights */
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            const size_t to = (size_t)(ntype ? ntype[n] : 0) * d * d;
            double *dx = dX + (size_t)n * d;
            const double *x = X + (size_t)n * d;
            for (int i = 0; i < d; ++i) dx[i] = 0.0;
            vec_matT_acc(dK + (size_t)n * d, Wk + to, d, d, dx);
            vec_matT_acc(dQ + (size_t)n * d, Wq + to, d, d, dx);
            vec_matT_acc(dV + (size_t)n * d, Wv + to, d, d, dx);
            outer_acc(x, dK + (size_t)n * d, d, d, pk + tsz * me + to);
            outer_acc(x, dQ + (size_t)n * d, d, d, pq + tsz * me + to);
            outer_acc(x, dV + (size_t)n * d, d, d, pv + tsz * me + to);
            outer_acc(Z + (size_t)n * d, dOut + (size_t)n * d, d, d, po + tsz * me + to);
        }
        free(ka); free(msg); free(s); free(al); free(t); free(t2);
    }
    reduce_parts(dWk, pk, tsz, nt); reduce_parts(dWq, pq, tsz, nt); reduce_parts(dWv, pv, tsz, nt);
    reduce_parts(dWo, po, tsz, nt); reduce_parts(dWatt, pa, rsz, nt); reduce_parts(dWmsg, pm, rsz, nt);
    reduce_parts(dmu, pu, msz, nt);
    free(pk); free(pq); free(pv); free(po); free(pa); free(pm); free(pu);
    free(K); free(Q); free(V); free(dK); free(dQ); free(dV); free(dZ); free(Z);
    free(alpha); free(ds); free(sraw);
    free(in_ptr); free(in_list); free(out_ptr); free(out_list);
}
