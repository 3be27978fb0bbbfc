// RGAT traversal (one head or several), forward and backward, with the edge softmax fused into the walks
// (thesis Ch.3 listing "attention calculation in a single-headed RGAT model": logit, softmax over
// the incoming edges of a destination, weighted sum of the messages).
//
// Forward, one destination-major walk per destination v: the message row Hs[pair_e] of an edge is
// gathered once; its source half of the logit, Hs[pair_e] . w_s[r_e], is formed from the row in
// registers (w_s sits in LDS), the destination half s_dst[run_e] comes from the per-run array; the
// softmax is the running-maximum form (max m, sum s of exp(l - m), accumulator rescaled when m grows),
// so the row is weighted and summed in the same pass.  What is kept for the backward pass is (m, s)
// per destination, 8 bytes per node, not an attention weight per edge.
//
// Backward, same walk: the edge's row is gathered again for g_e = dOut[v] . Hs[pair_e]; the logit is
// recomputed from that row exactly as in the forward pass and att_e = exp(l_e - m_v) / s_v.
//
// Several heads: the D/4 lanes of a row split into H groups of LPH lanes, one per head (column slice); every
// head has its own logit, running maximum and sum, and the reductions run over the head's LPH lanes only.
//
// Work distribution: persistent workgroups, each holding w_s in LDS, take the items of the
// destination-major list (longest first) in a grid-stride loop; a group of D/4 lanes owns an item.
// The indices of D/4 consecutive edges are fetched by one coalesced load per array (lane c takes
// edge c of the chunk) and handed round with cross-lane reads, one chunk ahead of the rows.
#include "rgnn_internal.h"
#include "traversal.h"
#include "device_utils.h"
#include "schedule.h"

namespace rgnn {

namespace {

constexpr int kFusedThreads = 512;

struct FusedArgs {
    Items it;
    const int32_t* in_pair;   // [E] pair of the CSR edge (backward: top bit set when the pair has no other edge)
    const int32_t* in_rel;    // [E]
    const int32_t* in_run;    // [E]
    const float* Hs;          // [P][D]
    const float* w_s;         // [R][D]
    const float* s_dst;       // [Q][H]
    float slope;
    int R;
    int own_singles;          // backward: the only edge of a single-edge pair writes that pair's entries
    // forward
    float* out;               // [N][D]
    float2* ms;               // [N][H] (m, s) of the destination's softmax
    float* partial;           // [num_partials][D] unnormalised sums of the pieces of cut destinations
    float2* part_ms;          // [num_partials][H]
    int general_n;            // items [0, skip_first) and [skip_first + skip_n, n) take the general walk
    int skip_first, skip_n;
    int short_first, short_n, single_first, single_n;
    // backward
    const float* dOut;        // [N][D]
    const float* fout;        // [N][D] forward output
    float* adz;               // [E][2][H]: att_e per head, then dz_e per head
    float* G;                 // [P][D] (only without dsy)
    float* ds_src;            // [P]    (only without dsy)
    float2* dsy;              // [P] (dz_e, att_e) of the only edge of a single-edge pair; H > 1: [P][2][H] floats, dz then att
};

__device__ __forceinline__ float leaky(float z, float slope) { return z > 0.f ? z : slope * z; }

// row of w_s for relation r: columns 4c..4c+3
template <int D, bool LDSW>
__device__ __forceinline__ float4 ws_row(const FusedArgs& a, const float* ws_lds, int r, int c) {
    if (LDSW) return *reinterpret_cast<const float4*>(ws_lds + r * D + c * 4);
    return *reinterpret_cast<const float4*>(a.w_s + (size_t)r * D + c * 4);
}
__device__ __forceinline__ float4 load_row_nt(const float* p) {
    const rgnn_v4f t = __builtin_nontemporal_load(reinterpret_cast<const rgnn_v4f*>(p));
    return make_float4(t[0], t[1], t[2], t[3]);
}

// ---------------------------------------------------------------- forward

// General items: any length, whole destinations or pieces of cut ones.
template <int D, int LPH, bool LDSW>
__device__ __forceinline__ void fwd_general(const FusedArgs& a, const float* ws_lds, int i, int c) {
    constexpr int LPR = D / 4, H = LPR / LPH;
    const int head = c / LPH;
    const int b = a.it.beg[i], e = a.it.end[i];
    const int slot = a.it.slot[i];
    const size_t v = (size_t)a.it.row[i];
    float4 acc0 = make_float4(0.f, 0.f, 0.f, 0.f), acc1 = acc0;
    float m = -INFINITY, s = 0.f;
    if (b < e) {
        // indices of chunk 0 (entries past the end repeat the last edge; they get weight zero)
        int jj = min(b + c, e - 1);
        // one head: lane c also fetches the destination half of edge c's logit; several heads: the run id, and every
        // lane reads its own head's entry when the batch is formed
        int cpr = a.in_pair[jj], crl = a.in_rel[jj], crn = a.in_run[jj];
        float csd = H == 1 ? a.s_dst[crn] : 0.f;
        for (int jc = b; jc < e; jc += LPR) {
            const bool more = jc + LPR < e;
            int npr = cpr, nrl = crl, nrn = 0;
            if (more) {
                jj = min(jc + LPR + c, e - 1);
                npr = a.in_pair[jj];
                nrl = a.in_rel[jj];
                nrn = a.in_run[jj];
            }
            const int cend = min(LPR, e - jc);
#pragma unroll
            for (int k = 0; k < LPR; k += 4) {
                if (k >= cend) break;
                float4 h[4];
                float sd[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int pr = group_lane<LPR>(cpr, k + u);
                    h[u] = load_row_nt(a.Hs + (size_t)pr * D + c * 4);
                    if (H > 1) sd[u] = a.s_dst[(size_t)group_lane<LPR>(crn, k + u) * H + head];
                }
                __builtin_amdgcn_sched_barrier(0);      // the w_s rows are read when the message rows arrive, not held meanwhile
                float l[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float4 w = ws_row<D, LDSW>(a, ws_lds, group_lane<LPR>(crl, k + u), c);
                    const float z = group_sum<LPH>(dot4(h[u], w)) + (H == 1 ? group_lane<LPR>(csd, k + u) : sd[u]);
                    l[u] = k + u < cend ? leaky(z, a.slope) : -INFINITY;
                }
                const float mn = fmaxf(fmaxf(m, fmaxf(l[0], l[1])), fmaxf(l[2], l[3]));
                const float sc = __expf(m - mn);              // 0 in the first batch (m = -inf), 1 while the maximum stands
                const float p0 = __expf(l[0] - mn), p1 = __expf(l[1] - mn), p2 = __expf(l[2] - mn), p3 = __expf(l[3] - mn);
                s = s * sc + ((p0 + p1) + (p2 + p3));
                acc0.x *= sc; acc0.y *= sc; acc0.z *= sc; acc0.w *= sc;
                acc1.x *= sc; acc1.y *= sc; acc1.z *= sc; acc1.w *= sc;
                fma4(acc0, p0, h[0]);
                fma4(acc1, p1, h[1]);
                fma4(acc0, p2, h[2]);
                fma4(acc1, p3, h[3]);
                m = mn;
            }
            if (more) {
                if (H == 1) csd = a.s_dst[nrn];
                cpr = npr;
                crl = nrl;
                crn = nrn;
            }
        }
    }
    fma4(acc0, 1.f, acc1);
    if (slot < 0) {
        const float inv = s > 0.f ? 1.f / s : 0.f;           // a destination without edges gets the zero row
        *reinterpret_cast<float4*>(a.out + v * D + c * 4) = make_float4(acc0.x * inv, acc0.y * inv, acc0.z * inv, acc0.w * inv);
        if (c % LPH == 0) a.ms[v * H + head] = make_float2(b < e ? m : 0.f, b < e ? s : 1.f);
    } else {
        *reinterpret_cast<float4*>(a.partial + (size_t)slot * D + c * 4) = acc0;
        if (c % LPH == 0) a.part_ms[(size_t)slot * H + head] = make_float2(m, s);
    }
}

// Whole destinations with 2..kShortLen edges: two per lane group, every load of both independent.
template <int D, int LPH, bool LDSW>
__device__ __forceinline__ void fwd_short(const FusedArgs& a, const float* ws_lds, int g2, int c) {
    constexpr int LPR = D / 4, H = LPR / LPH;
    const int head = c / LPH;
    const int i0 = 2 * g2;
    int b[2], e[2], orow[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int i = a.short_first + min(i0 + q, a.short_n - 1);
        b[q] = a.it.beg[i];
        e[q] = a.it.end[i];
        orow[q] = a.it.row[i];
    }
    int pr[2][kShortLen], rl[2][kShortLen], rn[2][kShortLen];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int u = 0; u < kShortLen; ++u) {
            const int jj = min(b[q] + u, e[q] - 1);
            pr[q][u] = a.in_pair[jj];
            rl[q][u] = a.in_rel[jj];
            rn[q][u] = a.in_run[jj];
        }
    float4 h[2][kShortLen];
    float sd[2][kShortLen];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int u = 0; u < kShortLen; ++u) {
            h[q][u] = load_row_nt(a.Hs + (size_t)pr[q][u] * D + c * 4);
            sd[q][u] = a.s_dst[(size_t)rn[q][u] * H + head];
        }
    __builtin_amdgcn_sched_barrier(0);      // the w_s rows are read when the message rows arrive, not held meanwhile
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        float l[kShortLen], m = -INFINITY;
#pragma unroll
        for (int u = 0; u < kShortLen; ++u) {
            const float4 w = ws_row<D, LDSW>(a, ws_lds, rl[q][u], c);
            const float z = group_sum<LPH>(dot4(h[q][u], w)) + sd[q][u];
            l[u] = b[q] + u < e[q] ? leaky(z, a.slope) : -INFINITY;
            m = fmaxf(m, l[u]);
        }
        float s = 0.f;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < kShortLen; ++u) {
            const float p = __expf(l[u] - m);
            s += p;
            fma4(acc, p, h[q][u]);
        }
        if (i0 + q < a.short_n) {
            const float inv = 1.f / s;
            *reinterpret_cast<float4*>(a.out + (size_t)orow[q] * D + c * 4) = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
            if (c % LPH == 0) a.ms[(size_t)orow[q] * H + head] = make_float2(m, s);
        }
    }
}

// Whole destinations with one edge (attention weight 1): four per lane group.
template <int D, int LPH, bool LDSW>
__device__ __forceinline__ void fwd_single(const FusedArgs& a, const float* ws_lds, int g4, int c) {
    constexpr int LPR = D / 4, H = LPR / LPH;
    const int head = c / LPH;
    const int i0 = 4 * g4;
    int j[4], orow[4], pr[4], rl[4], rn[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = a.single_first + min(i0 + u, a.single_n - 1);
        j[u] = a.it.beg[i];
        orow[u] = a.it.row[i];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        pr[u] = a.in_pair[j[u]];
        rl[u] = a.in_rel[j[u]];
        rn[u] = a.in_run[j[u]];
    }
    float4 h[4];
    float sd[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        h[u] = load_row_nt(a.Hs + (size_t)pr[u] * D + c * 4);
        sd[u] = a.s_dst[(size_t)rn[u] * H + head];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const float4 w = ws_row<D, LDSW>(a, ws_lds, rl[u], c);
        const float z = group_sum<LPH>(dot4(h[u], w)) + sd[u];
        if (i0 + u < a.single_n) {
            *reinterpret_cast<float4*>(a.out + (size_t)orow[u] * D + c * 4) = h[u];
            if (c % LPH == 0) a.ms[(size_t)orow[u] * H + head] = make_float2(leaky(z, a.slope), 1.f);
        }
    }
}

template <int D, bool LDSW>
__device__ __forceinline__ const float* stage_ws(const FusedArgs& a) {
    extern __shared__ __align__(16) float ws_lds[];
    if (LDSW) {
        const int n4 = a.R * D / 4;
        for (int i = threadIdx.x; i < n4; i += kFusedThreads)
            reinterpret_cast<float4*>(ws_lds)[i] = reinterpret_cast<const float4*>(a.w_s)[i];
        __syncthreads();
    }
    return ws_lds;
}

template <int D, int LPH, bool LDSW>
__global__ __launch_bounds__(kFusedThreads) void rgat_aggregate_fwd_kernel(FusedArgs a) {
    constexpr int LPR = D / 4, GPB = kFusedThreads / LPR;
    const float* ws_lds = stage_ws<D, LDSW>(a);
    const int grp = threadIdx.x / LPR, c = threadIdx.x % LPR;
    const int stride = gridDim.x * GPB, first = blockIdx.x * GPB + grp;
    for (int i = first; i < a.general_n; i += stride) fwd_general<D, LPH, LDSW>(a, ws_lds, i >= a.skip_first ? i + a.skip_n : i, c);
    for (int g2 = first; 2 * g2 < a.short_n; g2 += stride) fwd_short<D, LPH, LDSW>(a, ws_lds, g2, c);
    for (int g4 = first; 4 * g4 < a.single_n; g4 += stride) fwd_single<D, LPH, LDSW>(a, ws_lds, g4, c);
}

// Cut destinations: out[v] = sum_i exp(m_i - M) partial_i / S with M = max_i m_i, S = sum_i s_i exp(m_i - M) over the
// destination's pieces i, in piece order, per head.  One workgroup per cut destination; a lane works on the head its
// columns belong to (every lane walks the piece statistics of its head itself: a destination has few pieces).
template <int D, int LPH>
__global__ __launch_bounds__(1024) void rgat_combine_fwd_kernel(const int32_t* __restrict__ split_row,
                                                                const int32_t* __restrict__ split_ptr,
                                                                const float* __restrict__ partial,
                                                                const float2* __restrict__ part_ms, float* __restrict__ out,
                                                                float2* __restrict__ ms) {
    constexpr int LPR = D / 4, G = 1024 / LPR, H = LPR / LPH;
    __shared__ float4 red[1024];
    __shared__ float redw[H][16];
    const int sidx = blockIdx.x, g = threadIdx.x / LPR, c = threadIdx.x % LPR, head = c / LPH;
    const int p0 = split_ptr[sidx], p1 = split_ptr[sidx + 1];
    // maximum and sum per head over the pieces: thread t takes head t % H of pieces t / H, t / H + 1024 / H, ...;
    // the lanes of a wavefront that share a head are reduced with a butterfly over the strides H, 2H, ..., 32, the
    // sixteen wavefronts' results are combined in wavefront order
    const int rh = threadIdx.x % H, wv = threadIdx.x >> 6;
    float mloc = -INFINITY;
    for (int p = p0 + (int)threadIdx.x / H; p < p1; p += 1024 / H) mloc = fmaxf(mloc, part_ms[(size_t)p * H + rh].x);
#pragma unroll
    for (int o = 32; o >= H; o >>= 1) mloc = fmaxf(mloc, __shfl_xor(mloc, o));
    if ((threadIdx.x & 63) < H) redw[rh][wv] = mloc;
    __syncthreads();
    float M = redw[head][0];
    for (int k = 1; k < 16; ++k) M = fmaxf(M, redw[head][k]);
    float Mr = redw[rh][0];
    for (int k = 1; k < 16; ++k) Mr = fmaxf(Mr, redw[rh][k]);
    __syncthreads();
    float sloc = 0.f;
    for (int p = p0 + (int)threadIdx.x / H; p < p1; p += 1024 / H) {
        const float2 t = part_ms[(size_t)p * H + rh];
        sloc += t.y * __expf(t.x - Mr);
    }
#pragma unroll
    for (int o = 32; o >= H; o >>= 1) sloc += __shfl_xor(sloc, o);
    if ((threadIdx.x & 63) < H) redw[rh][wv] = sloc;
    __syncthreads();
    float S = redw[head][0];
    for (int k = 1; k < 16; ++k) S += redw[head][k];
    float4 acc0 = make_float4(0.f, 0.f, 0.f, 0.f), acc1 = acc0;
    for (int p = p0 + g; p < p1; p += 2 * G) {
        fma4(acc0, __expf(part_ms[(size_t)p * H + head].x - M), *reinterpret_cast<const float4*>(partial + (size_t)p * D + c * 4));
        if (p + G < p1)
            fma4(acc1, __expf(part_ms[(size_t)(p + G) * H + head].x - M), *reinterpret_cast<const float4*>(partial + (size_t)(p + G) * D + c * 4));
    }
    fma4(acc0, 1.f, acc1);
    red[threadIdx.x] = acc0;
    __syncthreads();
    if (g == 0) {
        float4 t = red[c];
        for (int k = 1; k < G; ++k) fma4(t, 1.f, red[k * LPR + c]);
        const float inv = 1.f / S;
        const size_t v = (size_t)split_row[sidx];
        *reinterpret_cast<float4*>(out + v * D + c * 4) = make_float4(t.x * inv, t.y * inv, t.z * inv, t.w * inv);
        if (c % LPH == 0) ms[v * H + head] = make_float2(M, S);
    }
}

// ---------------------------------------------------------------- backward

// For every CSR edge e of destination v, with the row h = Hs[pair_e] gathered once:
//   z_e = h . w_s[r_e] + s_dst[run_e];  att_e = exp(leakyrelu(z_e) - m_v) / s_v;  g_e = dOut[v] . h;
//   gbar_v = sum_e att_e g_e = dOut[v] . out[v]   (because out[v] = sum_e att_e Hs[pair_e]);
//   dz_e = att_e (g_e - gbar_v) (z_e > 0 ? 1 : slope);   adz[e] = (att_e, dz_e).
// Nothing is reduced over the destination's edges, so the pieces of a cut destination are independent.
// An edge that is the only edge of its (source, relation) pair also owns that pair's entries of the
// pair-major backward aggregation and writes them here: (dz_e, att_e) into dsy[p] (the typed-linear
// backward then reads the pair's gradient row as att_e * dOut[v]), or, without dsy, ds_src[p] = dz_e
// and the row G[p] = att_e * dOut[v] itself.  With several heads only the first form exists, and dsy
// holds 2 H floats per pair: dz_e per head, then att_e per head.
template <int D, int LPH, bool LDSW>
__device__ __forceinline__ void bwd_item(const FusedArgs& a, const float* ws_lds, int i, int c) {
    constexpr int LPR = D / 4, H = LPR / LPH;
    const int head = c / LPH;
    const int b = a.it.beg[i], e = a.it.end[i];
    if (b >= e) return;
    const size_t v = (size_t)a.it.row[i];
    const float4 go = *reinterpret_cast<const float4*>(a.dOut + v * D + c * 4);
    const float4 ov = *reinterpret_cast<const float4*>(a.fout + v * D + c * 4);
    const float2 st = a.ms[v * H + head];
    int jj = min(b + c, e - 1);
    int cpr = a.in_pair[jj], crl = a.in_rel[jj], crn = a.in_run[jj];
    float csd = H == 1 ? a.s_dst[crn] : 0.f;
    const float gbar = group_sum<LPH>(dot4(go, ov));
    const float m = st.x, inv = 1.f / st.y;
    for (int jc = b; jc < e; jc += LPR) {
        const bool more = jc + LPR < e;
        int npr = cpr, nrl = crl, nrn = 0;
        if (more) {
            jj = min(jc + LPR + c, e - 1);
            npr = a.in_pair[jj];
            nrl = a.in_rel[jj];
            nrn = a.in_run[jj];
        }
        const int cend = min(LPR, e - jc);
#pragma unroll
        for (int k = 0; k < LPR; k += 4) {
            if (k >= cend) break;
            float4 h[4];
            float sd[4];
            int pr[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                pr[u] = group_lane<LPR>(cpr, k + u);
                h[u] = load_row_nt(a.Hs + (size_t)(pr[u] & 0x7FFFFFFF) * D + c * 4);
                if (H > 1) sd[u] = a.s_dst[(size_t)group_lane<LPR>(crn, k + u) * H + head];
            }
            __builtin_amdgcn_sched_barrier(0);      // the w_s rows are read when the message rows arrive, not held meanwhile
            float2 mine = make_float2(0.f, 0.f);      // (att, dz) of edge jc + k + (c % LPH): lanes 0..3 of a head store one each
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float4 w = ws_row<D, LDSW>(a, ws_lds, group_lane<LPR>(crl, k + u), c);
                const float z = group_sum<LPH>(dot4(h[u], w)) + (H == 1 ? group_lane<LPR>(csd, k + u) : sd[u]);
                const float g = group_sum<LPH>(dot4(go, h[u]));
                const float al = __expf(leaky(z, a.slope) - m) * inv;
                const float dz = al * (g - gbar) * (z > 0.f ? 1.f : a.slope);
                if (c % LPH == u) mine = make_float2(al, dz);
                if (H == 1 && a.own_singles && k + u < cend && pr[u] < 0) {     // single-edge pair
                    const size_t p = (size_t)(pr[u] & 0x7FFFFFFF);
                    if (!a.dsy) *reinterpret_cast<float4*>(a.G + p * D + c * 4) = make_float4(al * go.x, al * go.y, al * go.z, al * go.w);
                    if (c == 0) {
                        if (a.dsy) a.dsy[p] = make_float2(dz, al);
                        else a.ds_src[p] = dz;
                    }
                }
                if (H > 1 && a.own_singles && k + u < cend && pr[u] < 0 && c % LPH == 0) {
                    float* hc = reinterpret_cast<float*>(a.dsy) + (size_t)(pr[u] & 0x7FFFFFFF) * 2 * H;
                    hc[head] = dz;
                    hc[H + head] = al;
                }
            }
            if (H == 1) {
                if (c < 4 && k + c < cend) *reinterpret_cast<float2*>(a.adz + (size_t)(jc + k + c) * 2) = mine;
            } else {
                // lane (head h, t) holds edge k + t of head h; the values change lanes so that lane t * H + h stores them:
                // the H lanes of an edge then write neighbouring floats
                const int t = c / H, h = c % H;
                const float al = __shfl(mine.x, h * LPH + t, LPR), dz = __shfl(mine.y, h * LPH + t, LPR);
                if (c < 4 * H && k + t < cend) {
                    float* o = a.adz + (size_t)(jc + k + t) * 2 * H + h;
                    o[0] = al;
                    o[H] = dz;
                }
            }
        }
        if (more) {
            if (H == 1) csd = a.s_dst[nrn];
            cpr = npr;
            crl = nrl;
            crn = nrn;
        }
    }
}

template <int D, int LPH, bool LDSW>
__global__ __launch_bounds__(kFusedThreads) void rgat_edge_dot_bwd_kernel(FusedArgs a) {
    constexpr int LPR = D / 4, GPB = kFusedThreads / LPR;
    const float* ws_lds = stage_ws<D, LDSW>(a);
    const int grp = threadIdx.x / LPR, c = threadIdx.x % LPR;
    const int stride = gridDim.x * GPB;
    for (int i = blockIdx.x * GPB + grp; i < a.it.n; i += stride) bwd_item<D, LPH, LDSW>(a, ws_lds, i, c);
}

// Launch with as many workgroups as stay resident at once (LDS, registers and wavefront slots decide), never more
// than the work needs: the grid-stride loops then see the items in list order, longest first, on every workgroup.
template <typename K>
rgnn_status_t launch_fused(K kernel, const rgnn_graph* g, size_t lds, size_t groups_needed, int lanes_per_row,
                           const FusedArgs& a, hipStream_t st) {
    const void* fn = reinterpret_cast<const void*>(kernel);
    if (lds) RGNN_TRY(allow_dynamic_lds(fn, lds));
    int per_cu = 1;
    RGNN_TRY(resident_blocks_per_cu(fn, kFusedThreads, lds, &per_cu));
    const size_t gpb = kFusedThreads / lanes_per_row;
    const size_t need = (groups_needed + gpb - 1) / gpb;
    const size_t grid = std::max<size_t>(1, std::min<size_t>(need, (size_t)per_cu * std::max(g->num_cus, 1)));
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(kFusedThreads), lds, st, a);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}

}  // namespace

// Runs the statement with DD = width and LL = lanes per head for the (width, heads) combinations the layer accepts
// (head widths 16, 32, 64, or one head of any width): LL = DD / 4 / heads.
#define RGNN_DISPATCH_DH(D_, H_, ...)                                                                              \
    do {                                                                                                           \
        const int lph_ = (D_) / 4 / (H_);                                                                          \
        if ((D_) == 64 && lph_ == 16) { constexpr int DD = 64, LL = 16; __VA_ARGS__; }                             \
        else if ((D_) == 64 && lph_ == 8) { constexpr int DD = 64, LL = 8; __VA_ARGS__; }                          \
        else if ((D_) == 64 && lph_ == 4) { constexpr int DD = 64, LL = 4; __VA_ARGS__; }                          \
        else if ((D_) == 32 && lph_ == 8) { constexpr int DD = 32, LL = 8; __VA_ARGS__; }                          \
        else if ((D_) == 32 && lph_ == 4) { constexpr int DD = 32, LL = 4; __VA_ARGS__; }                          \
        else if ((D_) == 128 && lph_ == 32) { constexpr int DD = 128, LL = 32; __VA_ARGS__; }                      \
        else if ((D_) == 128 && lph_ == 16) { constexpr int DD = 128, LL = 16; __VA_ARGS__; }                      \
        else if ((D_) == 128 && lph_ == 8) { constexpr int DD = 128, LL = 8; __VA_ARGS__; }                        \
        else if ((D_) == 128 && lph_ == 4) { constexpr int DD = 128, LL = 4; __VA_ARGS__; }                        \
        else RGNN_FAIL(RGNN_EUNSUPPORTED, "fused RGAT traversal: width %d with %d heads is not built", (int)(D_), (int)(H_)); \
    } while (0)

rgnn_status_t rgat_aggregate_fwd(const rgnn_graph* g, int D, int H, const float* Hs, const float* w_s, const float* s_dst,
                                 float slope, float* out, float* ms, float* partial, float* part_ms, hipStream_t st) {
    const ItemList& L = g->dst_items;
    if (L.num_items == 0) return RGNN_OK;
    const int ns = batched_count(L.num_single, current_schedule_flags());
    const int nsh = batched_count(L.num_short, current_schedule_flags());
    FusedArgs a{};
    a.it = dev_items(L); a.in_pair = g->idx[RGNN_IDX_IN_PAIR]; a.in_rel = g->idx[RGNN_IDX_IN_REL]; a.in_run = g->idx[RGNN_IDX_IN_RUN];
    a.Hs = Hs; a.w_s = w_s; a.s_dst = s_dst; a.slope = slope; a.R = g->R;
    a.out = out; a.ms = reinterpret_cast<float2*>(ms); a.partial = partial; a.part_ms = reinterpret_cast<float2*>(part_ms);
    a.general_n = L.num_items - nsh - ns; a.skip_first = nsh > 0 ? L.first_short : L.first_single; a.skip_n = nsh + ns;
    a.short_first = L.first_short; a.short_n = nsh; a.single_first = L.first_single; a.single_n = ns;
    const size_t lds = (size_t)g->R * D * sizeof(float);
    const bool ldsw = sched_ws_in_lds(g->R, D);
    const size_t groups = std::max<size_t>({(size_t)a.general_n, (size_t)(nsh + 1) / 2, (size_t)(ns + 3) / 4});
    {
        KernelTimer kt(st, "aggregate_fwd");
        if (ldsw) RGNN_DISPATCH_DH(D, H, RGNN_TRY(launch_fused(rgat_aggregate_fwd_kernel<DD, LL, true>, g, lds, groups, DD / 4, a, st)));
        else RGNN_DISPATCH_DH(D, H, RGNN_TRY(launch_fused(rgat_aggregate_fwd_kernel<DD, LL, false>, g, 0, groups, DD / 4, a, st)));
    }
    if (L.num_split > 0) {
        KernelTimer kt(st, "aggregate_fwd.combine");
        RGNN_DISPATCH_DH(D, H, hipLaunchKernelGGL((rgat_combine_fwd_kernel<DD, LL>), dim3(L.num_split), dim3(1024), 0, st, L.split_row,
                                                  L.split_ptr, partial, reinterpret_cast<const float2*>(part_ms), out,
                                                  reinterpret_cast<float2*>(ms)));
        RGNN_CHECK_LAUNCH();
    }
    return RGNN_OK;
}

rgnn_status_t rgat_edge_dot_bwd(const rgnn_graph* g, int D, int H, const float* Hs, const float* w_s, const float* s_dst,
                                const float* ms, const float* dOut, const float* out, float slope, float* adz, float* G,
                                float* ds_src, float* dsy, hipStream_t st) {
    const ItemList& L = g->dst_items;
    if (L.num_items == 0 || g->E == 0) return RGNN_OK;
    FusedArgs a{};
    a.it = dev_items(L); a.in_pair = g->in_pair_tag; a.in_rel = g->idx[RGNN_IDX_IN_REL]; a.in_run = g->idx[RGNN_IDX_IN_RUN];
    a.Hs = Hs; a.w_s = w_s; a.s_dst = s_dst; a.slope = slope; a.R = g->R; a.own_singles = H == 1 || dsy != nullptr;
    a.ms = reinterpret_cast<float2*>(const_cast<float*>(ms));
    a.dOut = dOut; a.fout = out; a.adz = adz; a.G = G; a.ds_src = ds_src;
    a.dsy = reinterpret_cast<float2*>(dsy);
    const size_t lds = (size_t)g->R * D * sizeof(float);
    const bool ldsw = sched_ws_in_lds(g->R, D);
    KernelTimer kt(st, "edge_dot_bwd");
    if (ldsw) RGNN_DISPATCH_DH(D, H, RGNN_TRY(launch_fused(rgat_edge_dot_bwd_kernel<DD, LL, true>, g, lds, (size_t)L.num_items, DD / 4, a, st)));
    else RGNN_DISPATCH_DH(D, H, RGNN_TRY(launch_fused(rgat_edge_dot_bwd_kernel<DD, LL, false>, g, 0, (size_t)L.num_items, DD / 4, a, st)));
    return RGNN_OK;
}

}  // namespace rgnn
