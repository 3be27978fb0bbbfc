// Edge-traversal kernels: per-destination edge softmax, weighted gather-sum aggregation
// (forward over destination-major CSR, backward over the pair-major transpose), the
// backward per-edge dot product, and the small segment sums around them.
//
// These replace the thesis's traversal template (Ch.3 "The GEMM Template and the Traversal
// Template": one block per edge or node, partial sums per thread and warp, then atomicAdd)
// by segment walks: every output row has exactly one owner, so nothing is accumulated with
// atomics and results do not depend on scheduling.  All of them are HBM-bound: a feature
// row of D floats is read by D/4 lanes as one 16-byte load each, so a 64-lane wavefront
// has four 256-byte rows (D = 64) in flight per load instruction, and the edge loop is
// unrolled four times to keep sixteen row reads in flight per wavefront.
//
// Segments longer than kItemMax entries (hub nodes) are cut into items by the graph index;
// an item of a cut segment writes a partial row and a combine kernel sums the partial rows
// of each cut segment in order.
#include "rgnn_internal.h"
#include "traversal.h"
#include "device_utils.h"
#include "schedule.h"

namespace rgnn {

static thread_local uint32_t g_schedule_flags = 0;
uint32_t current_schedule_flags() { return g_schedule_flags; }
ScheduleFlagsScope::ScheduleFlagsScope(uint32_t flags) : prev(g_schedule_flags) { g_schedule_flags = flags; }
ScheduleFlagsScope::~ScheduleFlagsScope() { g_schedule_flags = prev; }

// ------------------------------------------------------------------ small dense helpers

// wv[r][k] = sum_n W[r][k][n] * w[r][n]      (linear operator reordering, Ch.3: x (W w) instead of (x W) w)
// for one vector per relation or two (w2 / wv2 optional) in the same pass over W.  Eight lanes per weight row,
// 16-byte loads; nd is a multiple of 32.
__global__ __launch_bounds__(256) void fold_weight_kernel(const float* __restrict__ W, const float* __restrict__ w,
                                                          const float* __restrict__ w2, int kd, int nd, int total,
                                                          float* __restrict__ wv, float* __restrict__ wv2) {
    const int i = (blockIdx.x * 256 + threadIdx.x) >> 3, l = threadIdx.x & 7;  // (r, k)
    if (i >= total) return;
    const int r = i / kd;
    const float* Wr = W + (size_t)i * nd;
    float s = 0.f, s2 = 0.f;
    for (int n = 4 * l; n < nd; n += 32) {
        const float4 x = *reinterpret_cast<const float4*>(Wr + n);
        s += dot4(x, *reinterpret_cast<const float4*>(w + (size_t)r * nd + n));
        if (w2) s2 += dot4(x, *reinterpret_cast<const float4*>(w2 + (size_t)r * nd + n));
    }
    s = group_sum<8>(s);
    s2 = group_sum<8>(s2);
    if (l == 0) {
        wv[i] = s;
        if (w2) wv2[i] = s2;
    }
}

// s_dst[q] = X[run_dst[q]] . wtp[run_rel[q]]; each lane group takes four consecutive runs so
// that four row reads are in flight per lane.
template <int D>
__global__ void run_logit_kernel(int Q, const int32_t* __restrict__ run_dst, const int32_t* __restrict__ run_rel,
                                 const float* __restrict__ X, const float* __restrict__ wtp, float* __restrict__ s_dst) {
    constexpr int LPR = D / 4;
    const int q0 = (blockIdx.x * (256 / LPR) + threadIdx.x / LPR) * 4, c4 = threadIdx.x % LPR;
    float4 x[4], w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int q = min(q0 + u, Q - 1);
        x[u] = *reinterpret_cast<const float4*>(X + (size_t)run_dst[q] * D + c4 * 4);
        w[u] = *reinterpret_cast<const float4*>(wtp + (size_t)run_rel[q] * D + c4 * 4);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const float s = group_sum<LPR>(dot4(x[u], w[u]));
        if (q0 + u < Q && c4 == 0) s_dst[q0 + u] = s;
    }
}

// out[i * ostride + h] = sum_{j in [ptr[i], ptr[i+1])} val[(via ? via[j] : j) * stride + off + h],  h < heads.
// One launch: the first n_long * heads workgroups take one (long segment, head) each (segments of more
// than kSerialMax entries, listed by the graph index; the hub runs are thousands of entries long), the
// others one lane per (segment, head) for the segments up to that length.  The long ones come first so
// that the few workgroups that walk a hub run start at once and the short segments fill the machine
// around them.
__global__ __launch_bounds__(256) void segment_scalar_sum_kernel(int n, int heads, const int32_t* __restrict__ ptr,
                                                                 const int32_t* __restrict__ via,
                                                                 const float* __restrict__ val, int stride, int off,
                                                                 int min_len, float* __restrict__ out, int n_long,
                                                                 const int32_t* __restrict__ long_ids, int ostride) {
    __shared__ float red[4];
    const int lh = 31 - __clz(heads);            // the head count is a power of two (checked by the launcher)
    const int long_blocks = n_long << lh;
    if ((int)blockIdx.x < long_blocks) {
        // four loads in flight per lane, lane sums added in lane order, then the four wavefronts' sums in order
        const int i = long_ids[blockIdx.x >> lh], h = blockIdx.x & (heads - 1);
        const int b = ptr[i], e = ptr[i + 1];
        float t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f;
        for (int j = b + (int)threadIdx.x; j < e; j += 1024) {
            const int j1 = j + 256, j2 = j + 512, j3 = j + 768;
            t0 += val[(size_t)(via ? via[j] : j) * stride + off + h];
            if (j1 < e) t1 += val[(size_t)(via ? via[j1] : j1) * stride + off + h];
            if (j2 < e) t2 += val[(size_t)(via ? via[j2] : j2) * stride + off + h];
            if (j3 < e) t3 += val[(size_t)(via ? via[j3] : j3) * stride + off + h];
        }
        const float t = group_sum<64>((t0 + t1) + (t2 + t3));
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = t;
        __syncthreads();
        if (threadIdx.x == 0) out[(size_t)i * ostride + h] = (red[0] + red[1]) + (red[2] + red[3]);
        return;
    }
    const int64_t t = (int64_t)(blockIdx.x - long_blocks) * 256 + threadIdx.x;
    if (t >= (int64_t)n * heads) return;
    const int i = (int)(t >> lh), h = (int)(t & (heads - 1));
    const int b = ptr[i], e = ptr[i + 1];
    if (e - b > kSerialMax || e - b < min_len) return;
    // four entries per step, every load unconditional (positions past the end repeat the last entry and
    // add zero), so that a lane has four values in flight instead of one; the sum keeps the entry order
    float s = 0.f;
    for (int j = b; j < e; j += 4) {
        int id[4];
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int jj = min(j + u, e - 1);
            id[u] = via ? via[jj] : jj;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = val[(size_t)id[u] * stride + off + h];
#pragma unroll
        for (int u = 0; u < 4; ++u) s += j + u < e ? v[u] : 0.f;
    }
    out[(size_t)i * ostride + h] = s;
}

// The same sums for HV = 2 or 4 heads whose values lie side by side (stride, off and ostride multiples of HV, val
// and out aligned to HV floats): one lane per segment adds all HV heads at once with vector loads, one workgroup per
// long segment.  The order of the additions per head is the one of the kernel above.
template <int HV>
__global__ __launch_bounds__(256) void segment_vec_sum_kernel(int n, const int32_t* __restrict__ ptr,
                                                              const int32_t* __restrict__ via, const float* __restrict__ val,
                                                              int stride, int off, int min_len, float* __restrict__ out,
                                                              int n_long, const int32_t* __restrict__ long_ids, int ostride) {
    struct __align__(4 * HV) Vec { float v[HV]; };
    __shared__ float red[4][HV];
    auto load = [&](int j) { return *reinterpret_cast<const Vec*>(val + (size_t)(via ? via[j] : j) * stride + off); };
    if ((int)blockIdx.x < n_long) {
        const int i = long_ids[blockIdx.x];
        const int b = ptr[i], e = ptr[i + 1];
        float t[4][HV];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int h = 0; h < HV; ++h) t[u][h] = 0.f;
        for (int j = b + (int)threadIdx.x; j < e; j += 1024) {
            Vec x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) x[u] = load(min(j + 256 * u, e - 1));
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int h = 0; h < HV; ++h) t[u][h] += j + 256 * u < e ? x[u].v[h] : 0.f;
        }
#pragma unroll
        for (int h = 0; h < HV; ++h) {
            const float w = group_sum<64>((t[0][h] + t[1][h]) + (t[2][h] + t[3][h]));
            if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6][h] = w;
        }
        __syncthreads();
        if (threadIdx.x < HV) out[(size_t)i * ostride + threadIdx.x] = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
        return;
    }
    const int64_t i = (int64_t)(blockIdx.x - n_long) * 256 + threadIdx.x;
    if (i >= n) return;
    const int b = ptr[i], e = ptr[i + 1];
    if (e - b > kSerialMax || e - b < min_len) return;
    Vec s;
#pragma unroll
    for (int h = 0; h < HV; ++h) s.v[h] = 0.f;
    for (int j = b; j < e; j += 4) {
        Vec x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u] = load(min(j + u, e - 1));
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int h = 0; h < HV; ++h) s.v[h] += j + u < e ? x[u].v[h] : 0.f;
    }
    *reinterpret_cast<Vec*>(out + (size_t)i * ostride) = s;
}

// ------------------------------------------------------------------ edge softmax (RGAT)

// Per item of the destination-major list: l_e = leakyrelu(s_src[pair] + s_dst[run]) is
// written to att, then max and sum of exp; a whole-node item normalises at once
// (att_e = +-exp(l - m)/sum, sign bit set when z_e <= 0), a piece of a cut node stores
// (m, sum) for the combine step.
struct SoftmaxArgs {
    Items it;
    const int32_t* in_pair;
    const int32_t* in_run;
    const float* s_src;
    const float* s_dst;
    float slope;
    float* att;
    float* part_m;
    float* part_s;
    float2* ms;      // optional [N]: (max, sum of exp) of every destination with edges
};

__device__ __forceinline__ float signed_att(float l, float m, float inv) {
    const float a = expf(l - m) * inv;
    return l > 0.f ? a : -a;
}

// Destinations with at most kSerialMax incoming edges: one lane per node, in node order, so
// that neighbouring lanes walk neighbouring CSR ranges.  The logits stay in registers (the loop
// over the kSerialMax slots is fully unrolled and predicated), eight index pairs and then eight
// logit gathers are in flight at a time, and att is written once.  Everything else (longer nodes
// and the pieces of cut nodes) goes through edge_softmax_long_kernel.
__global__ __launch_bounds__(256) void edge_softmax_kernel(SoftmaxArgs a, int N, const int32_t* __restrict__ in_ptr) {
    const int v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= N) return;
    const int b = in_ptr[v], len = in_ptr[v + 1] - b;
    if (len == 0 || len > kSerialMax) return;
    float l[kSerialMax];
#pragma unroll
    for (int c = 0; c < kSerialMax; c += 8) {
        if (c < len) {
            int pr[8], rn[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int j = b + min(c + u, len - 1);
                pr[u] = a.in_pair[j];
                rn[u] = a.in_run[j];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float z = a.s_src[pr[u]] + a.s_dst[rn[u]];
                l[c + u] = c + u < len ? (z > 0.f ? z : a.slope * z) : -INFINITY;
            }
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) l[c + u] = -INFINITY;
        }
    }
    float m = -INFINITY, s = 0.f;
#pragma unroll
    for (int k = 0; k < kSerialMax; ++k) m = fmaxf(m, l[k]);
#pragma unroll
    for (int k = 0; k < kSerialMax; ++k) s += expf(l[k] - m);     // the empty slots add exp(-inf) = 0
    const float inv = 1.f / s;
#pragma unroll
    for (int k = 0; k < kSerialMax; ++k)
        if (k < len) a.att[b + k] = signed_att(l[k], m, inv);
    if (a.ms) a.ms[v] = make_float2(m, s);
}

// One wavefront per item that is longer than kSerialMax or is a piece of a cut node.  An item has at
// most kItemMax entries, kItemMax / 64 per lane, which stay in registers between the passes.
__global__ __launch_bounds__(256) void edge_softmax_long_kernel(SoftmaxArgs a, int n_long, const int32_t* __restrict__ long_item) {
    constexpr int PER = kItemMax / 64;
    const int w = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (w >= n_long) return;
    const int i = long_item[w];
    const int bb = a.it.beg[i], ee = a.it.end[i], sl = a.it.slot[i];
    float l[PER];
    int pr[PER], rn[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int j = min(bb + lane + 64 * u, ee - 1);
        pr[u] = a.in_pair[j];
        rn[u] = a.in_run[j];
    }
    float m = -INFINITY, s = 0.f;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const float z = a.s_src[pr[u]] + a.s_dst[rn[u]];
        l[u] = bb + lane + 64 * u < ee ? (z > 0.f ? z : a.slope * z) : -INFINITY;
        m = fmaxf(m, l[u]);
    }
    m = wave_max(m);
#pragma unroll
    for (int u = 0; u < PER; ++u) s += expf(l[u] - m);
    s = group_sum<64>(s);
    if (sl < 0) {
        const float inv = 1.f / s;
#pragma unroll
        for (int u = 0; u < PER; ++u)
            if (bb + lane + 64 * u < ee) a.att[bb + lane + 64 * u] = signed_att(l[u], m, inv);
        if (a.ms && lane == 0) a.ms[a.it.row[i]] = make_float2(m, s);
    } else {
        // a piece of a cut node: the finish kernel normalises, from the logits
#pragma unroll
        for (int u = 0; u < PER; ++u)
            if (bb + lane + 64 * u < ee) a.att[bb + lane + 64 * u] = l[u];
        if (lane == 0) {
            a.part_m[sl] = m;
            a.part_s[sl] = s;
        }
    }
}

// Cut nodes: combine the pieces' (m, sum) in order, then normalise every piece.
// One wavefront per piece; each recomputes its node's totals (a node has few pieces).
__global__ void edge_softmax_finish_kernel(int num_partials, const int32_t* __restrict__ part_item,
                                           const int32_t* __restrict__ part_split,
                                           const int32_t* __restrict__ split_ptr, Items it,
                                           const float* __restrict__ part_m, const float* __restrict__ part_s,
                                           float* __restrict__ att, float2* __restrict__ ms) {
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (t >= num_partials) return;
    const int sp = part_split[t];
    const int p0 = split_ptr[sp], p1 = split_ptr[sp + 1];
    float m = -INFINITY;
    for (int p = p0 + lane; p < p1; p += 64) m = fmaxf(m, part_m[p]);
    m = wave_max(m);
    float s = 0.f;
    for (int p = p0 + lane; p < p1; p += 64) s += part_s[p] * expf(part_m[p] - m);
    s = group_sum<64>(s);
    const float inv = 1.f / s;
    const int item = part_item[t];
    for (int j = it.beg[item] + lane; j < it.end[item]; j += 64) att[j] = signed_att(att[j], m, inv);
    if (ms && t == p0 && lane == 0) ms[it.row[item]] = make_float2(m, s);     // the node's first piece records its totals
}

// ------------------------------------------------------------------ weighted gather-sum

// For item i with entries j in [beg, end):
//   k   = via ? via[j] : j
//   row = rowidx ? (row_by_k ? rowidx[k] : rowidx[j]) : k
//   c   = coef ? coef[k * cstride + head] : 1     (absolute value if cabs; head = which of the
//                                                  `heads` equal column groups the lane's columns lie in)
//   acc += c * src[row]
// and acc goes to out[row_i] (whole segment) or partial[slot] (piece of a cut segment).
struct GatherArgs {
    Items it;
    const int32_t* via;
    const int32_t* rowidx;
    int row_by_k;
    const float* coef;
    int cstride;
    int cabs;
    int lanes_per_head;   // lanes per row / heads
    const void* src;      // rows of TI
    void* out;            // rows of TO
    float* partial;       // fp32 rows
    int skip_first;       // items [skip_first, skip_first + skip_n) are left to the short-segment and single-entry walks
    int skip_n;
    Rank1 r1;             // optional: out[row_i] += r1.coef[row_i][head] * r1.vec[r1.seg[row_i]] (whole segments here,
                          // cut segments when their pieces are combined)
    float* sum2;          // optional (S2 kernels): sum2[row_i * sum2_stride + head] = sum_j coef[k * cstride + s2off + head]
    int sum2_stride;      // for the whole segments, added in entry order; the caller sums the cut segments itself.  With
    int s2off;            // r1.vec set, the walk also adds that sum times r1.vec[r1.seg[row_i]] to the row (r1.coef then
                          // serves only the cut segments, where their pieces are combined)
};

// the rank-1 term of a whole segment whose coefficient the walk has just summed
template <int D, int V>
__device__ __forceinline__ void add_rank1_own(const Rank1& r1, float c, size_t row, int cv, float (&acc)[V]) {
    if (!r1.vec) return;
    float t[V];
    load_cols(r1.vec + (size_t)r1.seg[row] * D + cv * V, t);
    fma_cols(acc, c, t);
}

template <int D, int V>
__device__ __forceinline__ void add_rank1(const Rank1& r1, int lanes_per_head, size_t row, int cv, float (&acc)[V]) {
    if (!r1.coef) return;
    const float c = r1.coef[row * r1.stride + cv / lanes_per_head];
    float t[V];
    load_cols(r1.vec + (size_t)r1.seg[row] * D + cv * V, t);
    fma_cols(acc, c, t);
}

// ROLE gives each use its own kernel name in profiler output (0 forward aggregation over destinations,
// 1 backward aggregation over pairs, 2 destination-side weight gradient).  The forward aggregation
// gathers rows of the large per-pair tensor, most of them once: with fp32 rows those loads carry the
// non-temporal hint (NT; it did not pay for the 2-byte rows, whose pairs are shared by more edges in the
// workloads that use them); the other two gather rows of node tensors, which are reused and stay cached.
// TI / TO: storage type of the gathered rows and of the output rows (float or bf16_t).
template <int D, typename TI, typename TO, bool R1, bool NT, bool S2 = false>
__device__ __forceinline__ void gather_general(const GatherArgs& a, int blk) {
    constexpr int V = RowT<TI>::V, LPR = D / V, IPB = 256 / LPR;
    int i = blk * IPB + threadIdx.x / LPR;
    const int cv = threadIdx.x % LPR;
    if (i >= a.it.n - a.skip_n) return;
    if (i >= a.skip_first) i += a.skip_n;      // the single-entry segments have their own kernel
    const TI* __restrict__ src = static_cast<const TI*>(a.src);
    const int b = a.it.beg[i], e = a.it.end[i];
    const int head = cv / a.lanes_per_head;
    float acc0[V], acc1[V];
    zero_cols(acc0);
    zero_cols(acc1);
    // Indices and coefficients run one batch of four ahead of the rows, so that a batch costs one
    // memory round trip instead of two.  Positions past the end repeat the last entry with a zero
    // coefficient: every load is unconditional.
    int row[4];
    float c[4], c2[S2 ? 4 : 1], s2 = 0.f;
#define RGNN_GATHER_FETCH_IDX(J)                                                                  \
    _Pragma("unroll") for (int u = 0; u < 4; ++u) {                                               \
        const int jj = min((J) + u, e - 1);                                                       \
        const int k = a.via ? a.via[jj] : jj;                                                     \
        row[u] = a.rowidx ? (a.row_by_k ? a.rowidx[k] : a.rowidx[jj]) : k;                        \
        float cc = a.coef ? a.coef[(size_t)k * a.cstride + head] : 1.f;                           \
        if (a.cabs) cc = fabsf(cc);                                                               \
        c[u] = (J) + u < e ? cc : 0.f;                                                            \
        if (S2) c2[S2 ? u : 0] = (J) + u < e ? a.coef[(size_t)k * a.cstride + a.s2off + head] : 0.f; \
    }
    if (b < e) {
        RGNN_GATHER_FETCH_IDX(b)
    }
    for (int j = b; j < e; j += 4) {
        float v[4][V];
        float cc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (NT && sizeof(TI) == 4) load_cols_nt(src + (size_t)row[u] * D + cv * V, v[u]);
            else load_cols(src + (size_t)row[u] * D + cv * V, v[u]);
            cc[u] = c[u];
            if (S2) s2 += c2[S2 ? u : 0];
        }
        if (j + 4 < e) {
            RGNN_GATHER_FETCH_IDX(j + 4)
        }
        fma_cols(acc0, cc[0], v[0]);
        fma_cols(acc1, cc[1], v[1]);
        fma_cols(acc0, cc[2], v[2]);
        fma_cols(acc1, cc[3], v[3]);
    }
#undef RGNN_GATHER_FETCH_IDX
    fma_cols(acc0, 1.f, acc1);
    const int slot = a.it.slot[i];
    if (slot < 0) {
        if (R1) add_rank1<D>(a.r1, a.lanes_per_head, (size_t)a.it.row[i], cv, acc0);
        if (S2) add_rank1_own<D>(a.r1, s2, (size_t)a.it.row[i], cv, acc0);
        store_cols(static_cast<TO*>(a.out) + (size_t)a.it.row[i] * D + cv * V, acc0);
        if (S2 && cv % a.lanes_per_head == 0) a.sum2[(size_t)a.it.row[i] * a.sum2_stride + head] = s2;
    } else {
        store_cols(a.partial + (size_t)slot * D + cv * V, acc0);
    }
}

// The whole segments with 2..kShortLen entries, items [first, first + n).  One batch of row loads covers
// such a segment, so the general kernel would spend its time on the item -> indices -> rows -> store
// chain; here a group of lanes takes two of them at a time, all loads of both independent (entries
// past a segment's end repeat its last one with a zero coefficient).
template <int D, typename TI, typename TO, bool R1, bool NT, bool S2 = false>
__device__ __forceinline__ void gather_short(const GatherArgs& a, int blk, int first, int n) {
    constexpr int V = RowT<TI>::V, LPR = D / V, GPB = 256 / LPR;
    const int g = blk * GPB + threadIdx.x / LPR, cv = threadIdx.x % LPR;
    const int i0 = 2 * g;
    if (i0 >= n) return;
    const TI* __restrict__ src = static_cast<const TI*>(a.src);
    const int head = cv / a.lanes_per_head;
    int b[2], e[2], orow[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int i = first + min(i0 + q, n - 1);
        b[q] = a.it.beg[i];
        e[q] = a.it.end[i];
        orow[q] = a.it.row[i];
    }
    int row[2][kShortLen];
    float c[2][kShortLen], s2[2] = {0.f, 0.f};
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int u = 0; u < kShortLen; ++u) {
            const int jj = min(b[q] + u, e[q] - 1);
            const int k = a.via ? a.via[jj] : jj;
            row[q][u] = a.rowidx ? (a.row_by_k ? a.rowidx[k] : a.rowidx[jj]) : k;
            float cc = a.coef ? a.coef[(size_t)k * a.cstride + head] : 1.f;
            if (a.cabs) cc = fabsf(cc);
            c[q][u] = b[q] + u < e[q] ? cc : 0.f;
            if (S2) s2[q] += b[q] + u < e[q] ? a.coef[(size_t)k * a.cstride + a.s2off + head] : 0.f;
        }
    float v[2][kShortLen][V];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int u = 0; u < kShortLen; ++u) {
            if (NT && sizeof(TI) == 4) load_cols_nt(src + (size_t)row[q][u] * D + cv * V, v[q][u]);
            else load_cols(src + (size_t)row[q][u] * D + cv * V, v[q][u]);
        }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        float acc[V];
        zero_cols(acc);
#pragma unroll
        for (int u = 0; u < kShortLen; ++u) fma_cols(acc, c[q][u], v[q][u]);
        if (i0 + q < n) {
            if (R1) add_rank1<D>(a.r1, a.lanes_per_head, (size_t)orow[q], cv, acc);
            if (S2) add_rank1_own<D>(a.r1, s2[q], (size_t)orow[q], cv, acc);
            store_cols(static_cast<TO*>(a.out) + (size_t)orow[q] * D + cv * V, acc);
            if (S2 && cv % a.lanes_per_head == 0) a.sum2[(size_t)orow[q] * a.sum2_stride + head] = s2[q];
        }
    }
}

// The whole segments with exactly one entry, items [first, first + n): out[row_i] = c * src[row].
// A group of lanes handles four of them at a time, all loads of the four independent, which keeps
// enough rows in flight where the general kernel would wait on one short dependent chain per item.
template <int D, typename TI, typename TO, bool R1, bool NT>
__device__ __forceinline__ void gather_single(const GatherArgs& a, int blk, int first, int n) {
    constexpr int V = RowT<TI>::V, LPR = D / V, GPB = 256 / LPR;
    const int g = blk * GPB + threadIdx.x / LPR, cv = threadIdx.x % LPR;
    const int i0 = 4 * g;
    if (i0 >= n) return;
    const TI* __restrict__ src = static_cast<const TI*>(a.src);
    const int head = cv / a.lanes_per_head;
    int j[4], orow[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = first + min(i0 + u, n - 1);
        j[u] = a.it.beg[i];
        orow[u] = a.it.row[i];
    }
    int row[4];
    float c[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int k = a.via ? a.via[j[u]] : j[u];
        row[u] = a.rowidx ? (a.row_by_k ? a.rowidx[k] : a.rowidx[j[u]]) : k;
        c[u] = a.coef ? a.coef[(size_t)k * a.cstride + head] : 1.f;
        if (a.cabs) c[u] = fabsf(c[u]);
    }
    float v[4][V];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        if (NT && sizeof(TI) == 4) load_cols_nt(src + (size_t)row[u] * D + cv * V, v[u]);
        else load_cols(src + (size_t)row[u] * D + cv * V, v[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        if (i0 + u < n) {
#pragma unroll
            for (int q = 0; q < V; ++q) v[u][q] *= c[u];
            if (R1) add_rank1<D>(a.r1, a.lanes_per_head, (size_t)orow[u], cv, v[u]);
            store_cols(static_cast<TO*>(a.out) + (size_t)orow[u] * D + cv * V, v[u]);
        }
    }
}

// fp32 rows: one launch for the three kinds of items: the first blocks walk the general items (longest
// first), the next ones the 2..kShortLen-entry segments, the last ones the single-entry segments, so the
// short work fills the machine while the long items drain.  bf16 rows: a launch per kind (a lane holds
// twice the columns there, and the registers of the short-segment path would cost the general walk
// its occupancy).
struct GatherRanges { int general_blocks, short_blocks, short_first, short_n, single_first, single_n; };
// R1: the rank-1 term of GatherArgs::r1 is present (fp32 rows only).
template <int D, int ROLE, typename TI, typename TO, bool R1 = false>
__global__ __launch_bounds__(256) void gather_sum_kernel(GatherArgs a, GatherRanges r) {
    const int blk = blockIdx.x;
    if (blk < r.general_blocks) gather_general<D, TI, TO, R1, ROLE == 0>(a, blk);
    else if (blk < r.general_blocks + r.short_blocks) gather_short<D, TI, TO, R1, ROLE == 0>(a, blk - r.general_blocks, r.short_first, r.short_n);
    else gather_single<D, TI, TO, R1, ROLE == 0>(a, blk - r.general_blocks - r.short_blocks, r.single_first, r.single_n);
}
// The pair-major walk that also sums the second coefficient of every entry per segment and head (GatherArgs::sum2;
// fp32 rows, lists without single-entry segments), held to the register budget of eight wavefronts per SIMD like
// the plain walk.
template <int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(8))) void gather_sum_s2_kernel(GatherArgs a, GatherRanges r) {
    const int blk = blockIdx.x;
    if (blk < r.general_blocks) gather_general<D, float, float, false, false, true>(a, blk);
    else gather_short<D, float, float, false, false, true>(a, blk - r.general_blocks, r.short_first, r.short_n);
}
template <int D, int ROLE, typename TI, typename TO>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(7))) void gather_general_kernel(GatherArgs a) { gather_general<D, TI, TO, false, ROLE == 0>(a, blockIdx.x); }
template <int D, int ROLE, typename TI, typename TO>
__global__ __launch_bounds__(256) void gather_short_kernel(GatherArgs a, int first, int n) { gather_short<D, TI, TO, false, ROLE == 0>(a, blockIdx.x, first, n); }
template <int D, int ROLE, typename TI, typename TO>
__global__ __launch_bounds__(256) void gather_single_kernel(GatherArgs a, int first, int n) { gather_single<D, TI, TO, false, ROLE == 0>(a, blockIdx.x, first, n); }

// NH weighted sums of the same rows in one walk: out[h][row_i] = sum_j coef[k][h] * src[row], k and row as
// in gather_sum_kernel (fp32 rows).  out is [NH][out_rows][D], the partial rows [NH][num_partials][D].
template <int D, int NH>
__global__ __launch_bounds__(256) void gather_heads_rows_kernel(GatherArgs a, int out_rows, int num_partials) {
    constexpr int LPR = D / 4, IPB = 256 / LPR;
    const int i = blockIdx.x * IPB + threadIdx.x / LPR, c4 = threadIdx.x % LPR;
    if (i >= a.it.n) return;
    const float* __restrict__ src = static_cast<const float*>(a.src);
    const int b = a.it.beg[i], e = a.it.end[i];
    float4 acc[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) acc[h] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = b; j < e; j += 2) {
        float4 x[2];
        float c[2][NH];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int jj = min(j + u, e - 1);
            const int k = a.via ? a.via[jj] : jj;
            const int row = a.rowidx ? (a.row_by_k ? a.rowidx[k] : a.rowidx[jj]) : k;
            x[u] = *reinterpret_cast<const float4*>(src + (size_t)row * D + c4 * 4);
#pragma unroll
            for (int h = 0; h < NH; ++h) c[u][h] = j + u < e ? a.coef[(size_t)k * NH + h] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int h = 0; h < NH; ++h) fma4(acc[h], c[u][h], x[u]);
    }
    const int slot = a.it.slot[i];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        float* o = slot < 0 ? static_cast<float*>(a.out) + ((size_t)h * out_rows + a.it.row[i]) * D
                            : a.partial + ((size_t)h * num_partials + slot) * D;
        *reinterpret_cast<float4*>(o + c4 * 4) = acc[h];
    }
}

// out[split_row[s]] = sum of partial rows [split_ptr[s], split_ptr[s+1]).  One workgroup per
// cut segment: group g of D/4 lanes sums partial rows g, g + G, g + 2G, ... (two at a time),
// then the G group sums are added in group order through LDS, so the summation order is fixed.
template <int D, typename TO>
__global__ __launch_bounds__(1024) void combine_partials_kernel(const int32_t* __restrict__ split_row,
                                                                const int32_t* __restrict__ split_ptr,
                                                                const float* __restrict__ partial,
                                                                TO* __restrict__ out, Rank1 r1, int lanes_per_head) {
    constexpr int LPR = D / 4, G = 1024 / LPR;
    __shared__ float4 red[1024];
    const int s = blockIdx.x, g = threadIdx.x / LPR, c4 = threadIdx.x % LPR;
    const int p0 = split_ptr[s], p1 = split_ptr[s + 1];
    float4 acc0 = make_float4(0.f, 0.f, 0.f, 0.f), acc1 = acc0;
    for (int p = p0 + g; p < p1; p += 2 * G) {
        fma4(acc0, 1.f, *reinterpret_cast<const float4*>(partial + (size_t)p * D + c4 * 4));
        if (p + G < p1) fma4(acc1, 1.f, *reinterpret_cast<const float4*>(partial + (size_t)(p + G) * D + c4 * 4));
    }
    fma4(acc0, 1.f, acc1);
    red[threadIdx.x] = acc0;
    __syncthreads();
    if (g == 0) {
        float4 t = red[c4];
        for (int k = 1; k < G; ++k) fma4(t, 1.f, red[k * LPR + c4]);
        float tv[4] = {t.x, t.y, t.z, t.w};
        add_rank1<D>(r1, lanes_per_head, (size_t)split_row[s], c4, tv);
        store_cols(out + (size_t)split_row[s] * D + c4 * 4, tv);
    }
}

// ------------------------------------------------------------------ edge-parallel aggregation (comparison schedule)

// out[dst_e] += |att_e| * Hs[pair_e] over equal shares of the CSR edge list: a lane group takes
// kEdgeChunk consecutive edges, sums in registers while the destination stays the same and adds the sum
// to the output row with atomic adds when it changes (the thesis' traversal template: partial
// aggregation in the thread, then atomicAdd to global memory).  Work is balanced by construction (no
// work lists), the price is the atomics.  out must be zero on entry.  The destination of a CSR edge is
// run_dst[in_run[e]].
constexpr int kEdgeChunk = 16;
template <int D>
__global__ __launch_bounds__(256) void aggregate_edge_parallel_kernel(int64_t E, const int32_t* __restrict__ in_pair,
                                                                      const int32_t* __restrict__ in_run,
                                                                      const int32_t* __restrict__ run_dst,
                                                                      const float* __restrict__ att,
                                                                      const float* __restrict__ Hs, float* __restrict__ out) {
    constexpr int LPR = D / 4, GPB = 256 / LPR;
    const int64_t e0 = ((int64_t)blockIdx.x * GPB + threadIdx.x / LPR) * kEdgeChunk;
    const int c4 = threadIdx.x % LPR;
    if (e0 >= E) return;
    const int64_t e1 = e0 + kEdgeChunk < E ? e0 + kEdgeChunk : E;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    int cur = run_dst[in_run[e0]];
    auto flush = [&](int v) {
        // the hardware's fp32 add on memory (no compare-and-swap loop); ordinary device memory
        float* o = out + (size_t)v * D + c4 * 4;
        unsafeAtomicAdd(o + 0, acc.x);
        unsafeAtomicAdd(o + 1, acc.y);
        unsafeAtomicAdd(o + 2, acc.z);
        unsafeAtomicAdd(o + 3, acc.w);
    };
    for (int64_t e = e0; e < e1; ++e) {
        const int v = run_dst[in_run[e]];
        if (v != cur) {
            flush(cur);
            acc = make_float4(0.f, 0.f, 0.f, 0.f);
            cur = v;
        }
        fma4(acc, fabsf(att[e]), *reinterpret_cast<const float4*>(Hs + (size_t)in_pair[e] * D + c4 * 4));
    }
    flush(cur);
}
__global__ void zero_f32_kernel(size_t n, float* __restrict__ x) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) x[i] = 0.f;
}

// ------------------------------------------------------------------ dX assembly

// dX[u] = sum_{p in srcpair(u)} dXp[p]  +  sum_{q in runs(u)} sum_h ds_dst[q][h] * wtp[run_rel[q]][h]  +  extra[u]
// (second and third terms optional).  The (run, head) pairs of a node are walked as one flat list.
struct NodeSumArgs {
    Items it;             // pairs by source node, ordered by length, never cut
    const int32_t* srcpair_ptr;
    const int32_t* srcpair_idx;
    const void* dXp;      // rows of TI
    const void* dXp2;     // MODE 2: a second tensor of per-pair rows, summed with the first
    const int32_t* dst_run_ptr;
    const int32_t* run_rel;
    const float* ds_dst;  // [Q][heads]
    const float* wtp;     // [R][heads][D]
    const float* extra;
    void* dX;             // rows of TO
    int heads;            // run term: sum over (run q, head h) of ds_dst[q][h] * wtp[run_rel[q]][h]
    int R;
};

// MODE 1: the destination-run term is present (RGAT); MODE 0: the kernel only sums pair rows;
// MODE 2: pair rows of two tensors (HGT: the key and the message halves of the input gradient).
template <int D, typename TI, typename TO, int MODE>
__global__ __launch_bounds__(256) void node_grad_sum_kernel(NodeSumArgs a) {
    constexpr bool RUNS = MODE == 1, TWO = MODE == 2;
    constexpr int V = RowT<TI>::V, LPR = D / V, IPB = 256 / LPR;
    const int i = blockIdx.x * IPB + threadIdx.x / LPR, cv = threadIdx.x % LPR;
    if (i >= a.it.n) return;
    const TI* __restrict__ dXp = static_cast<const TI*>(a.dXp);
    const TI* __restrict__ dXp2 = static_cast<const TI*>(a.dXp2);
    const int u = a.it.row[i];
    const int b = a.it.beg[i], e = a.it.end[i];
    const int H = a.heads, lh = 31 - __clz(H);      // the head count is a power of two
    const int qb = RUNS ? a.dst_run_ptr[u] << lh : 0, qe = RUNS ? a.dst_run_ptr[u + 1] << lh : 0;
    float acc[V], acc1[V];
    zero_cols(acc);
    zero_cols(acc1);
    // The first four pairs and the first four runs of the node are fetched together (a node has
    // about as many of either as one batch holds), so their two index -> row chains overlap.
    int pi[4], rr[4];
    float c[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        pi[t] = b + t < e ? a.srcpair_idx[b + t] : -1;
        rr[t] = -1;
        c[t] = 0.f;
        if (RUNS && qb + t < qe) {
            const int x = qb + t;
            rr[t] = (a.run_rel[x >> lh] << lh) + (x & (H - 1));
            c[t] = a.ds_dst[qb + t];
        }
    }
    if (a.extra) load_cols(a.extra + (size_t)u * D + cv * V, acc);
    {
        float v[4][V], w[4][V];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (pi[t] >= 0) load_cols_nt(dXp + (size_t)pi[t] * D + cv * V, v[t]);
            else zero_cols(v[t]);
            if (RUNS && rr[t] >= 0) load_cols(a.wtp + (size_t)rr[t] * D + cv * V, w[t]);
            else if (TWO && pi[t] >= 0) load_cols(dXp2 + (size_t)pi[t] * D + cv * V, w[t]);
            else zero_cols(w[t]);
        }
        fma_cols(acc, 1.f, v[0]);
        fma_cols(acc1, 1.f, v[1]);
        fma_cols(acc, 1.f, v[2]);
        fma_cols(acc1, 1.f, v[3]);
        if (TWO) {
            fma_cols(acc, 1.f, w[0]);
            fma_cols(acc1, 1.f, w[1]);
            fma_cols(acc, 1.f, w[2]);
            fma_cols(acc1, 1.f, w[3]);
        }
        if (RUNS) {
            fma_cols(acc, c[0], w[0]);
            fma_cols(acc1, c[1], w[1]);
            fma_cols(acc, c[2], w[2]);
            fma_cols(acc1, c[3], w[3]);
        }
    }
    for (int j = b + 4; j < e; j += 4) {
        float v[4][V], w[4][V];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            zero_cols(v[t]);
            zero_cols(w[t]);
            if (j + t < e) {
                const size_t p = (size_t)a.srcpair_idx[j + t];
                load_cols_nt(dXp + p * D + cv * V, v[t]);
                if (TWO) load_cols(dXp2 + p * D + cv * V, w[t]);
            }
        }
        fma_cols(acc, 1.f, v[0]);
        fma_cols(acc1, 1.f, v[1]);
        fma_cols(acc, 1.f, v[2]);
        fma_cols(acc1, 1.f, v[3]);
        if (TWO) {
            fma_cols(acc, 1.f, w[0]);
            fma_cols(acc1, 1.f, w[1]);
            fma_cols(acc, 1.f, w[2]);
            fma_cols(acc1, 1.f, w[3]);
        }
    }
    if (RUNS && qb + 4 < qe) {
        // row ids and coefficients of a batch are fetched while the rows of the batch before are in flight
        // (entries past the end repeat the last one with a zero coefficient)
        int rn[4];
        float cn[4];
#define RGNN_RUN_FETCH_IDX(Q0)                                                                   \
    _Pragma("unroll") for (int t = 0; t < 4; ++t) {                                              \
        const int x = min((Q0) + t, qe - 1);                                                     \
        rn[t] = (a.run_rel[x >> lh] << lh) + (x & (H - 1));                        \
        cn[t] = (Q0) + t < qe ? a.ds_dst[x] : 0.f;                                               \
    }
        RGNN_RUN_FETCH_IDX(qb + 4)
        for (int q = qb + 4; q < qe; q += 4) {
            float cq[4];
            float v[4][V];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                load_cols(a.wtp + (size_t)rn[t] * D + cv * V, v[t]);
                cq[t] = cn[t];
            }
            if (q + 4 < qe) RGNN_RUN_FETCH_IDX(q + 4)
            fma_cols(acc, cq[0], v[0]);
            fma_cols(acc1, cq[1], v[1]);
            fma_cols(acc, cq[2], v[2]);
            fma_cols(acc1, cq[3], v[3]);
        }
#undef RGNN_RUN_FETCH_IDX
    }
    fma_cols(acc, 1.f, acc1);
    store_cols(static_cast<TO*>(a.dX) + (size_t)u * D + cv * V, acc);
}

// ------------------------------------------------------------------ RGAT parameter-gradient epilogue

// Per relation r:  dw_s[r] = A[r] W[r];  dw_t[r] = U[r] W[r];  dW[r] += A[r]^T (x) w_s[r] + U[r]^T (x) w_t[r]
// where A[r] = sum_p ds_src[p] X[src_p] and U[r] = sum_q ds_dst[q] X[dst_q].  Workgroup (r, 0) forms the two
// vectors (the 256 / nd lanes of a column take the k index in turn and are added in order through LDS);
// workgroups (r, 1 + j) update 1024 consecutive elements of dW[r] each, four per lane.  nd is a power of two.
__global__ __launch_bounds__(256) void rgat_param_finish_kernel(int kd, int nd, const float* __restrict__ W,
                                                                const float* __restrict__ w_s, const float* __restrict__ w_t,
                                                                const float* __restrict__ A, const float* __restrict__ U,
                                                                float* __restrict__ dW, float* __restrict__ dw_s,
                                                                float* __restrict__ dw_t) {
    __shared__ float red[2][256];
    const int r = blockIdx.x, tid = threadIdx.x, ln = 31 - __clz(nd);
    const float* Wr = W + (size_t)r * kd * nd;
    const float* Ar = A + (size_t)r * kd;
    const float* Ur = U + (size_t)r * kd;
    if (blockIdx.y == 0) {
        const int n = tid & (nd - 1), ks = tid >> ln, KS = 256 >> ln;
        float s = 0.f, t = 0.f;
        for (int k = ks; k < kd; k += KS) {
            const float w = Wr[k * nd + n];
            s += Ar[k] * w;
            t += Ur[k] * w;
        }
        red[0][tid] = s;
        red[1][tid] = t;
        __syncthreads();
        if (ks == 0) {
            for (int q = 1; q < KS; ++q) {
                s += red[0][q * nd + n];
                t += red[1][q * nd + n];
            }
            dw_s[(size_t)r * nd + n] = s;
            dw_t[(size_t)r * nd + n] = t;
        }
        return;
    }
    const int i = ((blockIdx.y - 1) * 256 + tid) * 4;
    if (i >= kd * nd) return;
    const int k = i >> ln, n = i & (nd - 1);
    const float a = Ar[k], u = Ur[k];
    const float4 ws = *reinterpret_cast<const float4*>(w_s + (size_t)r * nd + n);
    const float4 wt = *reinterpret_cast<const float4*>(w_t + (size_t)r * nd + n);
    float4* o = reinterpret_cast<float4*>(dW + (size_t)r * kd * nd + i);
    float4 v = *o;
    v.x += a * ws.x + u * wt.x;
    v.y += a * ws.y + u * wt.y;
    v.z += a * ws.z + u * wt.z;
    v.w += a * ws.w + u * wt.w;
    *o = v;
}

// ------------------------------------------------------------------ elementwise

__global__ void relu_kernel(size_t n, float* __restrict__ x) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) x[i] = x[i] > 0.f ? x[i] : 0.f;
}
// y = (ref > 0) ? g : 0
__global__ void relu_grad_kernel(size_t n, const float* __restrict__ ref, const float* __restrict__ g,
                                 float* __restrict__ y) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) y[i] = ref[i] > 0.f ? g[i] : 0.f;
}

// same on bf16 storage (gradient in, masked gradient out); `ref` is the fp32 layer output
__global__ void relu_grad_bf16_kernel(size_t n, const float* __restrict__ ref, const bf16_t* __restrict__ g,
                                      bf16_t* __restrict__ y) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) y[i] = ref[i] > 0.f ? g[i] : (bf16_t)0;
}

// dst += src
__global__ void add_into_kernel(size_t n, const float* __restrict__ src, float* __restrict__ dst) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] += src[i];
}

// bfloat16 -> fp32 (exact: the bf16 bits are the upper half of the fp32 word)
__global__ void widen_bf16_kernel(size_t n, const uint16_t* __restrict__ src, float* __restrict__ dst) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = __uint_as_float((uint32_t)src[i] << 16);
}

// ==================================================================== host launchers


rgnn_status_t fold_weight(int R, int kd, int nd, const float* W, const float* w, float* wv, hipStream_t st, const float* w2,
                          float* wv2) {
    const int total = R * kd;
    if (nd % 32) RGNN_FAIL(RGNN_EUNSUPPORTED, "fold_weight: width %d is not a multiple of 32", nd);
    KernelTimer kt(st, "fold_weight");
    hipLaunchKernelGGL(fold_weight_kernel, dim3(blocks_for((size_t)total * 8, 256)), dim3(256), 0, st, W, w, w2, kd, nd, total, wv, wv2);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}

rgnn_status_t run_logit(const rgnn_graph* g, int D, const float* X, const float* wtp, float* s_dst, hipStream_t st) {
    if (g->Q == 0) return RGNN_OK;
    KernelTimer kt(st, "run_logit");
    RGNN_DISPATCH_D(D, hipLaunchKernelGGL(run_logit_kernel<DD>, dim3(blocks_for((size_t)((g->Q + 3) / 4) * (DD / 4), 256)), dim3(256), 0,
                                     st, (int)g->Q, g->idx[RGNN_IDX_RUN_DST], g->idx[RGNN_IDX_RUN_REL], X, wtp, s_dst));
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}

rgnn_status_t segment_scalar_sum(int n, const int32_t* ptr, const LongList& lng, const int32_t* via, const float* val,
                                 int stride, int off, float* out, hipStream_t st, const char* label, int min_len,
                                 int heads, bool long_only, int ostride) {
    if (heads < 1 || (heads & (heads - 1))) RGNN_FAIL(RGNN_EUNSUPPORTED, "segment_scalar_sum: the head count must be a power of two, got %d", heads);
    if (n == 0 || (long_only && lng.n == 0)) return RGNN_OK;
    KernelTimer kt(st, label);
    const size_t long_blocks = (size_t)lng.n * heads;
    if (ostride <= 0) ostride = heads;
    if (long_only) n = 0;   // only the first kind of workgroups: the caller has summed the segments of up to kSerialMax entries
    if ((heads == 2 || heads == 4) && stride % heads == 0 && off % heads == 0 && ostride % heads == 0) {
        const dim3 grid((unsigned)(lng.n + blocks_for((size_t)n, 256)));
        if (heads == 2) hipLaunchKernelGGL(segment_vec_sum_kernel<2>, grid, dim3(256), 0, st, n, ptr, via, val, stride, off, min_len, out, lng.n, lng.ids, ostride);
        else hipLaunchKernelGGL(segment_vec_sum_kernel<4>, grid, dim3(256), 0, st, n, ptr, via, val, stride, off, min_len, out, lng.n, lng.ids, ostride);
        RGNN_CHECK_LAUNCH();
        return RGNN_OK;
    }
    hipLaunchKernelGGL(segment_scalar_sum_kernel, dim3((unsigned)(long_blocks + blocks_for((size_t)n * heads, 256))), dim3(256), 0, st, n,
                       heads, ptr, via, val, stride, off, min_len, out, lng.n, lng.ids, ostride);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}

rgnn_status_t edge_softmax(const rgnn_graph* g, const float* s_src, const float* s_dst, float slope, float* att,
                           float* part_m, float* part_s, hipStream_t st, float* ms) {
    const ItemList& L = g->dst_items;
    if (L.num_items == 0) return RGNN_OK;
    SoftmaxArgs a{dev_items(L), g->idx[RGNN_IDX_IN_PAIR], g->idx[RGNN_IDX_IN_RUN], s_src, s_dst, slope, att, part_m, part_s,
                  reinterpret_cast<float2*>(ms)};
    {
        KernelTimer kt(st, "edge_softmax");
        hipLaunchKernelGGL(edge_softmax_kernel, dim3(blocks_for((size_t)g->N, 256)), dim3(256), 0, st, a, (int)g->N,
                           g->idx[RGNN_IDX_IN_PTR]);
        RGNN_CHECK_LAUNCH();
        if (L.num_long > 0) {
            hipLaunchKernelGGL(edge_softmax_long_kernel, dim3(blocks_for((size_t)L.num_long * 64, 256)), dim3(256), 0, st,
                               a, L.num_long, L.long_item);
            RGNN_CHECK_LAUNCH();
        }
    }
    if (L.num_partials > 0) {
        KernelTimer kt(st, "edge_softmax.finish");
        hipLaunchKernelGGL(edge_softmax_finish_kernel, dim3(blocks_for((size_t)L.num_partials * 64, 256)), dim3(256), 0,
                           st, L.num_partials, L.part_item, L.part_split, L.split_ptr, dev_items(L), part_m, part_s, att,
                           reinterpret_cast<float2*>(ms));
        RGNN_CHECK_LAUNCH();
    }
    return RGNN_OK;
}

// Launches KERNEL<DD, ..., TI, TO> for the storage types of a call.  bf16 rows exist at width 128 only.
#define RGNN_DISPATCH_ROWS(D_, IN16, OUT16, ...)                                                         \
    do {                                                                                                 \
        if (!(IN16) && !(OUT16)) { using TI = float; using TO = float; RGNN_DISPATCH_D(D_, __VA_ARGS__); }      \
        else if ((D_) != 128) RGNN_FAIL(RGNN_EUNSUPPORTED, "bf16 rows need width 128, got %d", (int)(D_)); \
        else if ((IN16) && (OUT16)) { using TI = bf16_t; using TO = bf16_t; constexpr int DD = 128; __VA_ARGS__; } \
        else if (IN16) { using TI = bf16_t; using TO = float; constexpr int DD = 128; __VA_ARGS__; }            \
        else { using TI = float; using TO = bf16_t; constexpr int DD = 128; __VA_ARGS__; }                      \
    } while (0)

rgnn_status_t gather_sum(const ItemList& L, int D, const int32_t* via, const int32_t* rowidx, int row_by_k,
                         const float* coef, int cstride, int cabs, const void* src, void* out, float* partial,
                         hipStream_t st, int role, const char* label, const char* combine_label, int heads,
                         int src_bf16, int out_bf16, const Rank1* r1, float* sum2, int sum2_stride) {
    if (L.num_items == 0) return RGNN_OK;
    const Rank1 r1v = r1 ? *r1 : Rank1{nullptr, 0, nullptr, nullptr};
    const int lpr = D / (src_bf16 ? 8 : 4);
    // enough short / single-entry segments to be worth launches of their own; the two ranges are adjacent
    const int ns = batched_count(L.num_single, current_schedule_flags());
    const int nsh = batched_count(L.num_short, current_schedule_flags());
    const int skip_first = nsh > 0 ? L.first_short : L.first_single;
    GatherArgs a{dev_items(L), via, rowidx, row_by_k, coef, cstride, cabs, lpr / heads, src, out, partial, skip_first, nsh + ns, r1v, sum2, sum2_stride, heads};
    {
        KernelTimer kt(st, label);
        GatherRanges r{};
        r.general_blocks = (int)blocks_for(L.num_items - nsh - ns, 256 / lpr);
        r.short_blocks = nsh > 0 ? (int)blocks_for((size_t)(nsh + 1) / 2, 256 / lpr) : 0;
        r.short_first = L.first_short; r.short_n = nsh; r.single_first = L.first_single; r.single_n = ns;
        const int single_blocks = ns > 0 ? (int)blocks_for((size_t)(ns + 3) / 4, 256 / lpr) : 0;
        const dim3 grid(r.general_blocks + r.short_blocks + single_blocks);
#define RGNN_LAUNCH_GATHER(KERNEL, GRID, ...)                                                                              \
    do {                                                                                                                   \
        if (role == 0) RGNN_DISPATCH_ROWS(D, src_bf16, out_bf16, hipLaunchKernelGGL((KERNEL<DD, 0, TI, TO>), GRID, dim3(256), 0, st, __VA_ARGS__)); \
        else if (role == 1) RGNN_DISPATCH_ROWS(D, src_bf16, out_bf16, hipLaunchKernelGGL((KERNEL<DD, 1, TI, TO>), GRID, dim3(256), 0, st, __VA_ARGS__)); \
        else RGNN_DISPATCH_ROWS(D, src_bf16, out_bf16, hipLaunchKernelGGL((KERNEL<DD, 2, TI, TO>), GRID, dim3(256), 0, st, __VA_ARGS__)); \
        RGNN_CHECK_LAUNCH();                                                                                               \
    } while (0)
        if (r1 && (src_bf16 || out_bf16 || role != 1)) RGNN_FAIL(RGNN_EUNSUPPORTED, "gather_sum: the rank-1 term is built for fp32 rows of the pair-major walk");
        if (sum2 && (src_bf16 || out_bf16 || role != 1 || !coef || cstride < 2 * heads || ns > 0 || L.num_single > 0))
            RGNN_FAIL(RGNN_EUNSUPPORTED, "gather_sum: the second sum is built for fp32 rows of the pair-major walk over lists without single-entry segments");
        if (r1 && !sum2) {
            if (grid.x > 0) {
                RGNN_DISPATCH_D(D, hipLaunchKernelGGL((gather_sum_kernel<DD, 1, float, float, true>), grid, dim3(256), 0, st, a, r));
                RGNN_CHECK_LAUNCH();
            }
        } else if (sum2) {
            if (grid.x > 0) {
                RGNN_DISPATCH_D(D, hipLaunchKernelGGL((gather_sum_s2_kernel<DD>), grid, dim3(256), 0, st, a, r));
                RGNN_CHECK_LAUNCH();
            }
        } else if (!src_bf16) {
            if (grid.x > 0) RGNN_LAUNCH_GATHER(gather_sum_kernel, grid, a, r);
        } else {
            if (r.general_blocks > 0) RGNN_LAUNCH_GATHER(gather_general_kernel, dim3(r.general_blocks), a);
            if (nsh > 0) RGNN_LAUNCH_GATHER(gather_short_kernel, dim3(r.short_blocks), a, L.first_short, nsh);
            if (ns > 0) RGNN_LAUNCH_GATHER(gather_single_kernel, dim3(single_blocks), a, L.first_single, ns);
        }
#undef RGNN_LAUNCH_GATHER
    }
    if (L.num_split > 0) {
        KernelTimer kt(st, combine_label);
        if (out_bf16)
            RGNN_DISPATCH_D(D, hipLaunchKernelGGL((combine_partials_kernel<DD, bf16_t>), dim3(L.num_split), dim3(1024), 0, st,
                                                  L.split_row, L.split_ptr, partial, static_cast<bf16_t*>(out), r1v, (DD / 4) / heads));
        else
            RGNN_DISPATCH_D(D, hipLaunchKernelGGL((combine_partials_kernel<DD, float>), dim3(L.num_split), dim3(1024), 0, st,
                                                  L.split_row, L.split_ptr, partial, static_cast<float*>(out), r1v, (DD / 4) / heads));
        RGNN_CHECK_LAUNCH();
    }
    return RGNN_OK;
}

rgnn_status_t gather_heads_rows(const ItemList& L, int D, int H, int out_rows, const int32_t* via, const int32_t* rowidx,
                                int row_by_k, const float* coef, const float* src, float* out, float* partial,
                                hipStream_t st, const char* label, const char* combine_label) {
    if (L.num_items == 0) return RGNN_OK;
    GatherArgs a{dev_items(L), via, rowidx, row_by_k, coef, H, 0, 1, src, out, partial, 0, 0, Rank1{nullptr, 0, nullptr, nullptr}, nullptr, 1, 1};
    {
        KernelTimer kt(st, label);
        const dim3 grid(blocks_for(L.num_items, 256 / (D / 4)));
#define RGNN_LAUNCH_NH(NH_) RGNN_DISPATCH_D(D, hipLaunchKernelGGL((gather_heads_rows_kernel<DD, NH_>), grid, dim3(256), 0, st, a, out_rows, L.num_partials))
        if (H == 2) RGNN_LAUNCH_NH(2);
        else if (H == 4) RGNN_LAUNCH_NH(4);
        else if (H == 8) RGNN_LAUNCH_NH(8);
        else RGNN_FAIL(RGNN_EUNSUPPORTED, "gather_heads_rows: %d heads not built (2, 4, 8)", H);
#undef RGNN_LAUNCH_NH
        RGNN_CHECK_LAUNCH();
    }
    if (L.num_split > 0) {
        KernelTimer kt(st, combine_label);
        for (int h = 0; h < H; ++h) {
            RGNN_DISPATCH_D(D, hipLaunchKernelGGL((combine_partials_kernel<DD, float>), dim3(L.num_split), dim3(1024), 0, st,
                                                  L.split_row, L.split_ptr, partial + (size_t)h * L.num_partials * D,
                                                  out + (size_t)h * out_rows * D, Rank1{nullptr, 0, nullptr, nullptr}, 1));
            RGNN_CHECK_LAUNCH();
        }
    }
    return RGNN_OK;
}

rgnn_status_t aggregate_edge_parallel(const rgnn_graph* g, int D, const float* att, const float* Hs, float* out,
                                      hipStream_t st) {
    if (g->N == 0) return RGNN_OK;
    KernelTimer kt(st, "aggregate_fwd_edge_parallel");
    const size_t n = (size_t)g->N * D;
    hipLaunchKernelGGL(zero_f32_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, st, n, out);   // a kernel, not a memset: callers may capture
    RGNN_CHECK_LAUNCH();
    if (g->E == 0) return RGNN_OK;
    RGNN_DISPATCH_D(D, hipLaunchKernelGGL(aggregate_edge_parallel_kernel<DD>, dim3(blocks_for(((size_t)g->E + kEdgeChunk - 1) / kEdgeChunk, 256 / (DD / 4))),
                                          dim3(256), 0, st, g->E, g->idx[RGNN_IDX_IN_PAIR], g->idx[RGNN_IDX_IN_RUN],
                                          g->idx[RGNN_IDX_RUN_DST], att, Hs, out));
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}

rgnn_status_t node_grad_sum(const rgnn_graph* g, int D, const void* dXp, const float* ds_dst, const float* wtp,
                            const float* extra, void* dX, hipStream_t st, int in_bf16, int out_bf16, int heads,
                            const void* dXp2) {
    if (g->N == 0) return RGNN_OK;
    if (ds_dst && dXp2) RGNN_FAIL(RGNN_EINVAL, "node_grad_sum: the run term and a second row tensor exclude each other");
    if (heads < 1 || (heads & (heads - 1))) RGNN_FAIL(RGNN_EUNSUPPORTED, "node_grad_sum: the head count must be a power of two, got %d", heads);
    NodeSumArgs a{dev_items(g->srcpair_items), g->idx[RGNN_IDX_SRCPAIR_PTR], g->idx[RGNN_IDX_SRCPAIR_IDX], dXp, dXp2,
                  g->idx[RGNN_IDX_DST_RUN_PTR], g->idx[RGNN_IDX_RUN_REL], ds_dst, wtp, extra, dX, heads, (int)g->R};
    KernelTimer kt(st, "node_grad_sum");
    const dim3 grid(blocks_for((size_t)g->N, 256 / (D / (in_bf16 ? 8 : 4))));
    if (ds_dst)
        RGNN_DISPATCH_ROWS(D, in_bf16, out_bf16, hipLaunchKernelGGL((node_grad_sum_kernel<DD, TI, TO, 1>), grid, dim3(256), 0, st, a));
    else if (dXp2)
        RGNN_DISPATCH_ROWS(D, in_bf16, out_bf16, hipLaunchKernelGGL((node_grad_sum_kernel<DD, TI, TO, 2>), grid, dim3(256), 0, st, a));
    else
        RGNN_DISPATCH_ROWS(D, in_bf16, out_bf16, hipLaunchKernelGGL((node_grad_sum_kernel<DD, TI, TO, 0>), grid, dim3(256), 0, st, a));
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}

rgnn_status_t rgat_param_finish(int R, int kd, int nd, const float* W, const float* w_s, const float* w_t,
                                const float* A, const float* U, float* dW, float* dw_s, float* dw_t, hipStream_t st) {
    KernelTimer kt(st, "rgat_param_finish");
    hipLaunchKernelGGL(rgat_param_finish_kernel, dim3(R, 1 + (kd * nd + 1023) / 1024), dim3(256), 0, st, kd, nd, W, w_s, w_t, A, U, dW, dw_s,
                       dw_t);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}

rgnn_status_t widen_bf16(size_t n, const uint16_t* src, float* dst, hipStream_t st) {
    if (n == 0) return RGNN_OK;
    KernelTimer kt(st, "widen_bf16");
    hipLaunchKernelGGL(widen_bf16_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, st, n, src, dst);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}
rgnn_status_t add_into(size_t n, const float* src, float* dst, hipStream_t st) {
    if (n == 0) return RGNN_OK;
    KernelTimer kt(st, "add_into");
    hipLaunchKernelGGL(add_into_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, st, n, src, dst);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}
rgnn_status_t relu_inplace(size_t n, float* x, hipStream_t st) {
    if (n == 0) return RGNN_OK;
    KernelTimer kt(st, "relu");
    hipLaunchKernelGGL(relu_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, st, n, x);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}
rgnn_status_t relu_grad(size_t n, const float* ref, const void* gin, void* y, hipStream_t st, int bf16) {
    if (n == 0) return RGNN_OK;
    KernelTimer kt(st, "relu_grad");
    if (bf16)
        hipLaunchKernelGGL(relu_grad_bf16_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, st, n, ref,
                           static_cast<const bf16_t*>(gin), static_cast<bf16_t*>(y));
    else
        hipLaunchKernelGGL(relu_grad_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, st, n, ref,
                           static_cast<const float*>(gin), static_cast<float*>(y));
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}

}  // namespace rgnn
