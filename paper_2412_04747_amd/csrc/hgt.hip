// Kernels of the HGT layer: block-diagonal expansion of the per-(relation, head) matrices, the
// per-head edge logits, the per-head edge softmax and the per-head backward edge dot.
// (Caption of the thesis figure "HGT and RGAT layer": attention of HGT is an edgewise dot
// product between the relation-transformed key of the source and the query of the
// destination; the message depends only on (source node, edge type), so both are stored
// once per pair.)
//
// The d_head x d_head matrices W[r][h] are expanded to one block-diagonal d x d matrix per
// relation so that the relation-segmented typed-linear kernel serves them unchanged; with
// bf16 or fp32 inputs that kernel is bound by HBM traffic at these widths, so the extra
// zero blocks cost no time.
#include "rgnn_internal.h"
#include "traversal.h"
#include "device_utils.h"

namespace rgnn {

// Wbd[r][i][j] = c(r, h) * W[r][h][i % dh][j % dh] if i and j lie in the same head h, else 0.
// c = (mu ? mu[r][h] : 1) / sqrt(dh) when `scaled` (attention), 1 otherwise (message).
__global__ void hgt_expand_kernel(int R, int d, int H, const float* __restrict__ W, const float* __restrict__ mu,
                                  int scaled, float* __restrict__ Wbd) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t total = (size_t)R * d * d;
    if (i >= total) return;
    const int dh = d / H;
    const int r = (int)(i / ((size_t)d * d)), a = (int)(i / d % d), b = (int)(i % d);
    const int ha = a / dh, hb = b / dh;
    float v = 0.f;
    if (ha == hb) {
        float c = 1.f;
        if (scaled) c = (mu ? mu[r * H + ha] : 1.f) * rsqrtf((float)dh);
        v = c * W[(((size_t)r * H + ha) * dh + a % dh) * dh + b % dh];
    }
    Wbd[i] = v;
}

// One workgroup per (relation, head): dW[r][h] = c * block(dWbd[r], h); for the attention
// matrices also dmu[r][h] = sum(block .* W[r][h]) / sqrt(dh).
__global__ void hgt_extract_kernel(int d, int H, const float* __restrict__ dWbd, const float* __restrict__ W,
                                   const float* __restrict__ mu, int scaled, float* __restrict__ dW,
                                   float* __restrict__ dmu) {
    __shared__ float red[256];
    const int r = blockIdx.x / H, h = blockIdx.x % H, dh = d / H;
    const float inv = rsqrtf((float)dh);
    const float c = scaled ? (mu ? mu[r * H + h] : 1.f) * inv : 1.f;
    float s = 0.f;
    for (int i = threadIdx.x; i < dh * dh; i += blockDim.x) {
        const int a = i / dh, b = i % dh;
        const float g = dWbd[((size_t)r * d + h * dh + a) * d + h * dh + b];
        const size_t wi = ((size_t)r * H + h) * dh * dh + i;
        dW[wi] = c * g;
        s += g * W[wi];
    }
    if (!(scaled && dmu)) return;
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = blockDim.x / 2; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) dmu[r * H + h] = red[0] * inv;
}

// Linear operator reordering (Ch.3 "Linear Operator Reordering": two linear operators in a row may be
// switched when that leaves a product between weights).  When every pair of a relation r has a source
// of one node type t(r), K[src] Watt[r] = X[src] (Wk[t(r)] Watt[r]): the per-pair key and message rows
// come straight from X with a folded per-relation weight, and K and V are never formed.
//   Wf[r][k][n] = sum over j in the head of n of Wnode[t(r)][k][j] * Wbd[r][j][n]
// Written as fp32 (Wf) or rounded to bf16 (Wf16), whichever is given.
__global__ void hgt_fold_kernel(int R, int d, int H, const int32_t* __restrict__ rel_type,
                                const float* __restrict__ Wnode, const float* __restrict__ Wbd, float* __restrict__ Wf,
                                bf16_t* __restrict__ Wf16) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)R * d * d) return;
    const int dh = d / H;
    const int r = (int)(i / ((size_t)d * d)), k = (int)(i / d % d), n = (int)(i % d);
    const float* Wn = Wnode + ((size_t)rel_type[r] * d + k) * d;
    const float* Wb = Wbd + (size_t)r * d * d;
    const int j0 = n / dh * dh;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;      // dh is a multiple of 16: four independent chains
#pragma unroll 2
    for (int j = j0; j < j0 + dh; j += 4) {
        const float4 w4 = *reinterpret_cast<const float4*>(Wn + j);
        s0 += w4.x * Wb[(size_t)j * d + n];
        s1 += w4.y * Wb[(size_t)(j + 1) * d + n];
        s2 += w4.z * Wb[(size_t)(j + 2) * d + n];
        s3 += w4.w * Wb[(size_t)(j + 3) * d + n];
    }
    const float s = (s0 + s1) + (s2 + s3);
    if (Wf) Wf[i] = s;
    if (Wf16) Wf16[i] = (bf16_t)(bf16_pack2(s, 0.f) & 0xFFFFu);
}

// dWbd[r][j][n] = sum_k Wnode[t(r)][k][j] * dWf[r][k][n] for j, n in the same head (other entries are not written)
__global__ void hgt_fold_bwd_rel_kernel(int R, int d, int H, const int32_t* __restrict__ rel_type,
                                        const float* __restrict__ Wnode, const float* __restrict__ dWf,
                                        float* __restrict__ dWbd) {
    const int dh = d / H;
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;    // (r, j, n') with n' inside the head of j
    if (i >= (size_t)R * d * dh) return;
    const int r = (int)(i / ((size_t)d * dh)), j = (int)(i / dh % d), n = j / dh * dh + (int)(i % dh);
    const float* Wn = Wnode + (size_t)rel_type[r] * d * d;
    const float* G = dWf + (size_t)r * d * d;
    // four partial sums over k = 4 i + q keep eight independent loads in flight (d is a multiple of 32)
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll 2
    for (int k = 0; k < d; k += 4) {
        s0 += Wn[(size_t)k * d + j] * G[(size_t)k * d + n];
        s1 += Wn[(size_t)(k + 1) * d + j] * G[(size_t)(k + 1) * d + n];
        s2 += Wn[(size_t)(k + 2) * d + j] * G[(size_t)(k + 2) * d + n];
        s3 += Wn[(size_t)(k + 3) * d + j] * G[(size_t)(k + 3) * d + n];
    }
    dWbd[((size_t)r * d + j) * d + n] = (s0 + s1) + (s2 + s3);
}

// dWnode[t][k][j] = sum over relations r with t(r) = t, ascending, of sum over n in the head of j of dWf[r][k][n] * Wbd[r][j][n]
__global__ void hgt_fold_bwd_node_kernel(int T, int R, int d, int H, const int32_t* __restrict__ rel_type,
                                         const float* __restrict__ Wbd, const float* __restrict__ dWf,
                                         float* __restrict__ dWnode) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)T * d * d) return;
    const int dh = d / H;
    const int t = (int)(i / ((size_t)d * d)), k = (int)(i / d % d), j = (int)(i % d);
    const int n0 = j / dh * dh;
    float s = 0.f;
    for (int r = 0; r < R; ++r) {
        if (rel_type[r] != t) continue;
        const float* G = dWf + ((size_t)r * d + k) * d;
        const float* Wb = Wbd + ((size_t)r * d + j) * d;
        float p = 0.f;     // dh is a multiple of 16 and n0 of dh: 16-byte loads
        for (int n = n0; n < n0 + dh; n += 4) {
            const float4 gv = *reinterpret_cast<const float4*>(G + n), wv = *reinterpret_cast<const float4*>(Wb + n);
            p += (gv.x * wv.x + gv.y * wv.y) + (gv.z * wv.z + gv.w * wv.w);
        }
        s += p;
    }
    dWnode[i] = s;
}

// logit[e][h] = Ka[pair_e][h] . Q[v][h]   (Ka already carries mu / sqrt(dh)); TI = storage type of the rows.
// SM (heads of at least four lanes): the per-head softmax over the destination's edges rides along.  The lanes of a
// head keep a running maximum and the sum of exp(logit - maximum) over the batches; a whole destination then
// turns the logits it has just written into weights (each lane re-reads the entries it stored itself), a piece of a
// cut destination stores its (maximum, sum) per head for the finish kernel, which normalises the pieces' entries.
template <int D, typename TI, bool SM>
__global__ __launch_bounds__(256) void hgt_edge_logit_kernel(Items it, int H, const int32_t* __restrict__ in_pair,
                                                             const TI* __restrict__ Ka, const TI* __restrict__ Q,
                                                             float* logit, float* __restrict__ part_m,
                                                             float* __restrict__ part_s) {
    constexpr int V = RowT<TI>::V, LPR = D / V, IPB = 256 / LPR;
    const int i = blockIdx.x * IPB + threadIdx.x / LPR, cv = threadIdx.x % LPR;
    if (i >= it.n) return;
    const int b = it.beg[i], e = it.end[i];
    if (e == b) return;
    const int lph = LPR / H, head = cv / lph;
    float q[V];
    load_cols(Q + (size_t)it.row[i] * D + cv * V, q);
    // pair ids run one batch of four ahead of the rows (positions past the end repeat the last edge)
    int pr[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) pr[u] = in_pair[min(b + u, e - 1)];
    float mx = -INFINITY, sum = 0.f;
    const int sl = SM ? it.slot[i] : -1;
    const bool one = SM && e - b <= 4 && sl < 0;
    for (int j = b; j < e; j += 4) {
        float k[4][V];
#pragma unroll
        for (int u = 0; u < 4; ++u) load_cols(Ka + (size_t)pr[u] * D + cv * V, k[u]);
        if (j + 4 < e) {
#pragma unroll
            for (int u = 0; u < 4; ++u) pr[u] = in_pair[min(j + 4 + u, e - 1)];
        }
        // lane t < 4 of a head's lanes stores edge j + t (every lane of the head holds all four sums), so the
        // 4 x H results of a batch leave in one store instruction; heads of fewer than 4 lanes store one by one
        float mine = 0.f, sv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float s = group_sum_dyn(dot_cols(q, k[u]), lph);
            sv[u] = j + u < e ? s : -INFINITY;
            if (lph >= 4) { if (cv % lph == u) mine = s; }
            else if (cv % lph == 0 && j + u < e) logit[(size_t)(j + u) * H + head] = s;
        }
        if (SM) {
            const float mn = fmaxf(fmaxf(mx, fmaxf(sv[0], sv[1])), fmaxf(sv[2], sv[3]));     // sv[0] is finite: j < e
            sum = sum * __expf(mx - mn) + ((__expf(sv[0] - mn) + __expf(sv[1] - mn)) + (__expf(sv[2] - mn) + __expf(sv[3] - mn)));
            mx = mn;
            if (one) mine = __expf(mine - mx) / sum;      // a whole destination of up to four edges: the weights at once
        }
        if (lph >= 4 && cv % lph < 4 && j + cv % lph < e) logit[(size_t)(j + cv % lph) * H + head] = mine;
    }
    if (SM) {
        if (one) return;
        const int t = cv % lph;
        if (sl >= 0) {
            if (t == 0) {
                part_m[(size_t)sl * H + head] = mx;
                part_s[(size_t)sl * H + head] = sum;
            }
            return;
        }
        if (t >= 4) return;
        const float inv = 1.f / sum;
        for (int j = b + t; j < e; j += 4) {
            float* x = logit + (size_t)j * H + head;
            *x = __expf(*x - mx) * inv;
        }
    }
}

// Per-head softmax of att[e][h] (holding logits on entry) over each destination's edges, as a pass of its own: for
// the shapes whose heads span fewer than four lanes (bf16 rows with 16 columns per head); the others take the
// softmax in the logit walk.
// Short nodes: one lane per (node, head).  Long items and pieces of cut nodes: one wavefront
// per item, heads in turn; pieces store (max, sum) per head for the finish kernel.
__device__ __forceinline__ float soft_out(float l, float m, float inv) { return expf(l - m) * inv; }
__global__ __launch_bounds__(256) void hgt_softmax_kernel(int N, int H, const int32_t* __restrict__ in_ptr,
                                                          float* __restrict__ att) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)N * H) return;
    const int lh = 31 - __clz(H);                 // the head count is a power of two
    const int v = (int)(t >> lh), h = (int)(t & (H - 1));
    const int b = in_ptr[v], len = in_ptr[v + 1] - b;
    if (len == 0 || len > kSerialMax) return;
    float l[kSerialMax];               // the logits stay in registers: one read and one write of att
#pragma unroll
    for (int c = 0; c < kSerialMax; c += 8) {
#pragma unroll
        for (int u = 0; u < 8; ++u) l[c + u] = -INFINITY;
        if (c < len) {
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (c + u < len) l[c + u] = att[(size_t)(b + c + u) * H + h];
        }
    }
    float m = -INFINITY, s = 0.f;
#pragma unroll
    for (int k = 0; k < kSerialMax; ++k) m = fmaxf(m, l[k]);
#pragma unroll
    for (int k = 0; k < kSerialMax; ++k) s += expf(l[k] - m);
    const float inv = 1.f / s;
#pragma unroll
    for (int k = 0; k < kSerialMax; ++k)
        if (k < len) att[(size_t)(b + k) * H + h] = soft_out(l[k], m, inv);
}
__global__ __launch_bounds__(256) void hgt_softmax_long_kernel(Items it, int n_long, const int32_t* __restrict__ long_item,
                                                               int H, float* __restrict__ att, float* __restrict__ part_m,
                                                               float* __restrict__ part_s) {
    constexpr int PER = kItemMax / 64;     // an item has at most kItemMax entries
    const int w = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (w >= n_long) return;
    const int i = long_item[w];
    const int bb = it.beg[i], ee = it.end[i], sl = it.slot[i];
    for (int h = 0; h < H; ++h) {
        float l[PER];
        float m = -INFINITY, s = 0.f;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int j = bb + lane + 64 * u;
            l[u] = j < ee ? att[(size_t)j * H + h] : -INFINITY;
            m = fmaxf(m, l[u]);
        }
        m = wave_max(m);
#pragma unroll
        for (int u = 0; u < PER; ++u) s += expf(l[u] - m);
        s = group_sum<64>(s);
        if (sl < 0) {
            const float inv = 1.f / s;
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int j = bb + lane + 64 * u;
                if (j < ee) att[(size_t)j * H + h] = soft_out(l[u], m, inv);
            }
        } else if (lane == 0) {
            part_m[(size_t)sl * H + h] = m;
            part_s[(size_t)sl * H + h] = s;
        }
    }
}
// Cut nodes: one wavefront per piece.  The head count is a power of two, so lane l always meets head
// l & (H - 1): it combines that head's (m, sum) over the node's pieces (the lanes of a head take the
// pieces in turn and are then reduced across the wavefront), and the piece's att entries, H per edge
// and contiguous, are normalised with consecutive lanes on consecutive addresses.
__global__ void hgt_softmax_finish_kernel(int num_partials, const int32_t* __restrict__ part_item,
                                          const int32_t* __restrict__ part_split,
                                          const int32_t* __restrict__ split_ptr, Items it, int H,
                                          const float* __restrict__ part_m, const float* __restrict__ part_s,
                                          float* __restrict__ att) {
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (t >= num_partials) return;
    const int sp = part_split[t];
    const int p0 = split_ptr[sp], p1 = split_ptr[sp + 1];
    const int item = part_item[t];
    const int lh = 31 - __clz(H), h = lane & (H - 1), step = 64 >> lh;
    float m = -INFINITY;
    for (int p = p0 + (lane >> lh); p < p1; p += step) m = fmaxf(m, part_m[(size_t)p * H + h]);
    for (int o = 32; o >= H; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    float s = 0.f;
    for (int p = p0 + (lane >> lh); p < p1; p += step) s += part_s[(size_t)p * H + h] * expf(part_m[(size_t)p * H + h] - m);
    for (int o = 32; o >= H; o >>= 1) s += __shfl_xor(s, o);
    const float inv = 1.f / s;
    const size_t a0 = (size_t)it.beg[item] * H, a1 = (size_t)it.end[item] * H;
    for (size_t x = a0 + lane; x < a1; x += 64) att[x] = soft_out(att[x], m, inv);   // a0 and 64 are multiples of H: entry x is head h
}

// dl[e][h] = att[e][h] * (dZ[v][h] . M[pair_e][h] - dZ[v][h] . Z[v][h])
// (the second term is sum_e att_e g_e because Z[v][h] = sum_e att_e M[pair_e][h]).
template <int D, typename TI>
__global__ __launch_bounds__(256) void hgt_edge_dot_bwd_kernel(Items it, int H, const int32_t* __restrict__ in_pair,
                                                               const float* __restrict__ att,
                                                               const TI* __restrict__ M, const TI* __restrict__ dZ,
                                                               const TI* __restrict__ Z, float* __restrict__ dl) {
    constexpr int V = RowT<TI>::V, LPR = D / V, IPB = 256 / LPR;
    const int i = blockIdx.x * IPB + threadIdx.x / LPR, cv = threadIdx.x % LPR;
    if (i >= it.n) return;
    const int b = it.beg[i], e = it.end[i];
    if (e == b) return;
    const int lph = LPR / H, head = cv / lph;
    const size_t v = (size_t)it.row[i];
    float gz[V], zz[V];
    load_cols(dZ + v * D + cv * V, gz);
    load_cols(Z + v * D + cv * V, zz);
    // pair ids and attention weights run one batch of four ahead of the rows
    int pr[4];
    float an[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int jj = min(b + u, e - 1);
        pr[u] = in_pair[jj];
        an[u] = att[(size_t)jj * H + head];
    }
    const float gbar = group_sum_dyn(dot_cols(gz, zz), lph);
    for (int j = b; j < e; j += 4) {
        float mm[4][V];
        float a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            load_cols(M + (size_t)pr[u] * D + cv * V, mm[u]);
            a[u] = an[u];
        }
        if (j + 4 < e) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int jj = min(j + 4 + u, e - 1);
                pr[u] = in_pair[jj];
                an[u] = att[(size_t)jj * H + head];
            }
        }
        float mine = 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float g = group_sum_dyn(dot_cols(gz, mm[u]), lph);
            const float w = a[u];
            if (lph >= 4) { if (cv % lph == u) mine = w * (g - gbar); }
            else if (cv % lph == 0 && j + u < e) dl[(size_t)(j + u) * H + head] = w * (g - gbar);
        }
        // one store instruction for the 4 x H results of the batch (see hgt_edge_logit_kernel)
        if (lph >= 4 && cv % lph < 4 && j + cv % lph < e) dl[(size_t)(j + cv % lph) * H + head] = mine;
    }
}

__global__ void add3_kernel(size_t n, const float* __restrict__ a, const float* __restrict__ b,
                            const float* __restrict__ c, float* __restrict__ out) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = a[i] + b[i] + c[i];
}

// ---------------------------------------------------------------------------------------- launchers

rgnn_status_t hgt_expand(int R, int d, int H, const float* W, const float* mu, int scaled, float* Wbd, hipStream_t st) {
    KernelTimer kt(st, "hgt_expand");
    hipLaunchKernelGGL(hgt_expand_kernel, dim3(blocks_for((size_t)R * d * d, 256)), dim3(256), 0, st, R, d, H, W, mu,
                       scaled, Wbd);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}
rgnn_status_t hgt_extract(int R, int d, int H, const float* dWbd, const float* W, const float* mu, int scaled, float* dW,
                          float* dmu, hipStream_t st) {
    KernelTimer kt(st, "hgt_extract");
    hipLaunchKernelGGL(hgt_extract_kernel, dim3(R * H), dim3(256), 0, st, d, H, dWbd, W, mu, scaled, dW, dmu);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}
// part_m / part_s given: the softmax is taken in the same walk (logit then holds the attention weights) where a head
// spans at least four lanes; otherwise, and without them, logit holds the logits and hgt_softmax follows.
static bool hgt_softmax_rides(int D, int H, int rows_bf16) { return (D / (rows_bf16 ? 8 : 4)) / H >= 4; }
rgnn_status_t hgt_edge_logit(const rgnn_graph* g, int D, int H, const void* Ka, const void* Q, float* logit,
                             hipStream_t st, int rows_bf16, float* part_m, float* part_s) {
    const ItemList& L = g->dst_items;
    if (L.num_items == 0 || g->E == 0) return RGNN_OK;
    const bool sm = part_m && part_s && hgt_softmax_rides(D, H, rows_bf16);
    {
        KernelTimer kt(st, "hgt_edge_logit");
        if (rows_bf16) {
            if (D != 128) RGNN_FAIL(RGNN_EUNSUPPORTED, "bf16 rows need width 128, got %d", D);
            const dim3 grid(blocks_for(L.num_items, 256 / (128 / 8)));
            if (sm)
                hipLaunchKernelGGL((hgt_edge_logit_kernel<128, bf16_t, true>), grid, dim3(256), 0, st, dev_items(L), H, g->idx[RGNN_IDX_IN_PAIR],
                                   static_cast<const bf16_t*>(Ka), static_cast<const bf16_t*>(Q), logit, part_m, part_s);
            else
                hipLaunchKernelGGL((hgt_edge_logit_kernel<128, bf16_t, false>), grid, dim3(256), 0, st, dev_items(L), H, g->idx[RGNN_IDX_IN_PAIR],
                                   static_cast<const bf16_t*>(Ka), static_cast<const bf16_t*>(Q), logit, part_m, part_s);
        } else if (sm) {
            RGNN_DISPATCH_D(D, hipLaunchKernelGGL((hgt_edge_logit_kernel<DD, float, true>), dim3(blocks_for(L.num_items, 256 / (DD / 4))),
                                                  dim3(256), 0, st, dev_items(L), H, g->idx[RGNN_IDX_IN_PAIR],
                                                  static_cast<const float*>(Ka), static_cast<const float*>(Q), logit, part_m, part_s));
        } else {
            RGNN_DISPATCH_D(D, hipLaunchKernelGGL((hgt_edge_logit_kernel<DD, float, false>), dim3(blocks_for(L.num_items, 256 / (DD / 4))),
                                                  dim3(256), 0, st, dev_items(L), H, g->idx[RGNN_IDX_IN_PAIR],
                                                  static_cast<const float*>(Ka), static_cast<const float*>(Q), logit, part_m, part_s));
        }
        RGNN_CHECK_LAUNCH();
    }
    if (sm) return hgt_softmax_finish(g, H, logit, part_m, part_s, st);
    if (part_m && part_s) return hgt_softmax(g, H, logit, part_m, part_s, st);
    return RGNN_OK;
}
rgnn_status_t hgt_softmax(const rgnn_graph* g, int H, float* att, float* part_m, float* part_s, hipStream_t st) {
    const ItemList& L = g->dst_items;
    if (g->E == 0) return RGNN_OK;
    {
        KernelTimer kt(st, "hgt_softmax");
        hipLaunchKernelGGL(hgt_softmax_kernel, dim3(blocks_for((size_t)g->N * H, 256)), dim3(256), 0, st, (int)g->N, H,
                           g->idx[RGNN_IDX_IN_PTR], att);
        RGNN_CHECK_LAUNCH();
        if (L.num_long > 0) {
            hipLaunchKernelGGL(hgt_softmax_long_kernel, dim3(blocks_for((size_t)L.num_long * 64, 256)), dim3(256), 0, st,
                               dev_items(L), L.num_long, L.long_item, H, att, part_m, part_s);
            RGNN_CHECK_LAUNCH();
        }
    }
    return hgt_softmax_finish(g, H, att, part_m, part_s, st);
}
rgnn_status_t hgt_softmax_finish(const rgnn_graph* g, int H, float* att, const float* part_m, const float* part_s, hipStream_t st) {
    const ItemList& L = g->dst_items;
    if (L.num_partials == 0) return RGNN_OK;
    KernelTimer kt(st, "hgt_softmax.finish");
    hipLaunchKernelGGL(hgt_softmax_finish_kernel, dim3(blocks_for((size_t)L.num_partials * 64, 256)), dim3(256), 0,
                       st, L.num_partials, L.part_item, L.part_split, L.split_ptr, dev_items(L), H, part_m, part_s,
                       att);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}
rgnn_status_t hgt_edge_dot_bwd(const rgnn_graph* g, int D, int H, const float* att, const void* M, const void* dZ,
                               const void* Z, float* dl, hipStream_t st, int rows_bf16) {
    const ItemList& L = g->dst_items;
    if (L.num_items == 0 || g->E == 0) return RGNN_OK;
    KernelTimer kt(st, "hgt_edge_dot_bwd");
    if (rows_bf16) {
        if (D != 128) RGNN_FAIL(RGNN_EUNSUPPORTED, "bf16 rows need width 128, got %d", D);
        hipLaunchKernelGGL((hgt_edge_dot_bwd_kernel<128, bf16_t>), dim3(blocks_for(L.num_items, 256 / (128 / 8))), dim3(256), 0,
                           st, dev_items(L), H, g->idx[RGNN_IDX_IN_PAIR], att, static_cast<const bf16_t*>(M),
                           static_cast<const bf16_t*>(dZ), static_cast<const bf16_t*>(Z), dl);
    } else {
        RGNN_DISPATCH_D(D, hipLaunchKernelGGL((hgt_edge_dot_bwd_kernel<DD, float>), dim3(blocks_for(L.num_items, 256 / (DD / 4))),
                                              dim3(256), 0, st, dev_items(L), H, g->idx[RGNN_IDX_IN_PAIR], att,
                                              static_cast<const float*>(M), static_cast<const float*>(dZ),
                                              static_cast<const float*>(Z), dl));
    }
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}
rgnn_status_t hgt_fold(int R, int d, int H, const int32_t* rel_type, const float* Wnode, const float* Wbd, float* Wf,
                       void* Wf16, hipStream_t st) {
    KernelTimer kt(st, "hgt_fold");
    hipLaunchKernelGGL(hgt_fold_kernel, dim3(blocks_for((size_t)R * d * d, 256)), dim3(256), 0, st, R, d, H, rel_type, Wnode,
                       Wbd, Wf, static_cast<bf16_t*>(Wf16));
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}
rgnn_status_t hgt_fold_bwd(int T, int R, int d, int H, const int32_t* rel_type, const float* Wnode, const float* Wbd,
                           const float* dWf, float* dWbd, float* dWnode, hipStream_t st) {
    KernelTimer kt(st, "hgt_fold_bwd");
    hipLaunchKernelGGL(hgt_fold_bwd_rel_kernel, dim3(blocks_for((size_t)R * d * (d / H), 256)), dim3(256), 0, st, R, d, H,
                       rel_type, Wnode, dWf, dWbd);
    RGNN_CHECK_LAUNCH();
    hipLaunchKernelGGL(hgt_fold_bwd_node_kernel, dim3(blocks_for((size_t)T * d * d, 256)), dim3(256), 0, st, T, R, d, H,
                       rel_type, Wbd, dWf, dWnode);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}
rgnn_status_t add3(size_t n, const float* a, const float* b, const float* c, float* out, hipStream_t st) {
    if (n == 0) return RGNN_OK;
    KernelTimer kt(st, "add3");
    hipLaunchKernelGGL(add3_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, st, n, a, b, c, out);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}

}  // namespace rgnn
