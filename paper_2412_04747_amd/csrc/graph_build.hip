// Device side of the graph index build: every sort, scan and scatter that produces the
// canonical index arrays runs on the GPU (rocPRIM's radix sort and scan as library
// primitives, small hand-written kernels around them).  Integer bookkeeping only.
//
// Orders (each is a total order, so the result does not depend on the input edge order):
//   CSR edges      by (dst, rel, src, input id)      one 64-bit key sort, ids as values (stable)
//   pairs          distinct (rel, src), ascending    second key sort of the CSR positions; its
//                                                    permutation is the pair-major transpose
//   runs           maximal equal (dst, rel) groups of adjacent CSR edges
//   relrun         runs by (rel, dst);  srcpair: pairs by (src, rel);  nodes by (type, id)
#include "rgnn_internal.h"

#include <cstring>
#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>

namespace rgnn {

namespace {

typedef unsigned long long u64;

// temporary device buffer, freed on scope exit
struct Tmp {
    void* p = nullptr;
    ~Tmp() { if (p) (void)hipFree(p); }
    rgnn_status_t alloc(size_t bytes) {
        hipError_t e = hipMalloc(&p, bytes ? bytes : 16);
        if (e != hipSuccess) {
            set_error("hipMalloc(%zu) failed: %s", bytes, hipGetErrorString(e));
            return e == hipErrorOutOfMemory ? RGNN_ENOMEM : RGNN_EHIP;
        }
        return RGNN_OK;
    }
    template <typename T> T* as() { return static_cast<T*>(p); }
};

template <typename T>
rgnn_status_t keep(rgnn_graph* g, size_t n, T** out) {
    void* d = nullptr;
    const size_t bytes = (n ? n : 1) * sizeof(T);
    hipError_t e = hipMalloc(&d, bytes);
    if (e != hipSuccess) {
        set_error("hipMalloc(%zu) failed: %s", bytes, hipGetErrorString(e));
        return e == hipErrorOutOfMemory ? RGNN_ENOMEM : RGNN_EHIP;
    }
    g->allocs.push_back(d);
    g->index_bytes += bytes;
    *out = static_cast<T*>(d);
    return RGNN_OK;
}
rgnn_status_t keep_idx(rgnn_graph* g, int which, size_t n) {
    g->idx_len[which] = (int64_t)n;
    return keep<int32_t>(g, n, &g->idx[which]);
}

constexpr int TPB = 256;
inline unsigned nblk(size_t n) { return (unsigned)((n + TPB - 1) / TPB); }
#define LAUNCH(kern, n, ...)                                                              \
    do {                                                                                  \
        if ((n) > 0) {                                                                    \
            hipLaunchKernelGGL(kern, dim3(nblk(n)), dim3(TPB), 0, 0, __VA_ARGS__);        \
            RGNN_HIP(hipGetLastError());                                                  \
        }                                                                                 \
    } while (0)

// err[0] = code of the first kind of problem seen, err[1] = smallest offending index
__device__ void report(int* err, int code, long long index) {
    atomicCAS(&err[0], 0, code);
    atomicMin(reinterpret_cast<unsigned int*>(&err[1]), (unsigned int)index);
}

__global__ void k_check_rowptr(long long N, long long E, const int32_t* rowptr, int* err) {
    const long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (v > N) return;
    if ((v == 0 && rowptr[0] != 0) || (v == N && rowptr[N] != E) || (v < N && rowptr[v + 1] < rowptr[v])) report(err, 4, v);
}
// destination of CSR-input edge e: the row v with rowptr[v] <= e < rowptr[v+1]
__global__ void k_csr_rows(long long N, long long E, const int32_t* rowptr, int32_t* dst) {
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    long long lo = 0, hi = N;   // largest v in [0, N) with rowptr[v] <= e
    while (hi - lo > 1) {
        const long long mid = (lo + hi) >> 1;
        if (rowptr[mid] <= e) lo = mid; else hi = mid;
    }
    dst[e] = (int32_t)lo;
}
__global__ void k_check_ntype(long long N, int T, const int32_t* ntype, int* err) {
    const long long n = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (n < N && (ntype[n] < 0 || ntype[n] >= T)) report(err, 3, n);
}
__global__ void k_key_csr(long long E, long long N, int R, const int32_t* src, const int32_t* dst, const int32_t* rel,
                          const int32_t* ntype, const int32_t* rst, const int32_t* rdt, u64* key, uint32_t* val, int* err) {
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    const int s = src[e], d = dst[e], r = rel[e];
    u64 k = 0;
    if (s < 0 || s >= N || d < 0 || d >= N || r < 0 || r >= R) report(err, 1, e);
    else {
        k = ((u64)d * (u64)R + (u64)r) * (u64)N + (u64)s;
        if (rst && (ntype[s] != rst[r] || ntype[d] != rdt[r])) report(err, 2, e);
    }
    key[e] = k;
    val[e] = (uint32_t)e;
}
__global__ void k_decode_csr(long long E, long long N, int R, const u64* key, const uint32_t* val, int32_t* in_src,
                             int32_t* in_rel, int32_t* in_dst, int32_t* in_eid) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= E) return;
    const u64 k = key[i], t = k / (u64)N;
    in_src[i] = (int32_t)(k % (u64)N);
    in_rel[i] = (int32_t)(t % (u64)R);
    in_dst[i] = (int32_t)(t / (u64)R);
    in_eid[i] = (int32_t)val[i];
}
// out[v] = first position i in the ascending array a[0..n) with a[i] >= v, for v in 0..M
__global__ void k_lower_bound(long long n, const int32_t* a, long long M, int32_t* out) {
    const long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (v > M) return;
    long long lo = 0, hi = n;
    while (lo < hi) {
        const long long mid = (lo + hi) >> 1;
        if (a[mid] < v) lo = mid + 1; else hi = mid;
    }
    out[v] = (int32_t)lo;
}
__global__ void k_key2(long long n, long long mul, const int32_t* major, const int32_t* minor, u64* key, uint32_t* val) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    key[i] = (u64)major[i] * (u64)mul + (u64)minor[i];
    val[i] = (uint32_t)i;
}
__global__ void k_flag_key(long long n, const u64* key, int32_t* flag) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) flag[i] = (i == 0 || key[i] != key[i - 1]) ? 1 : 0;
}
__global__ void k_flag_runs(long long n, const int32_t* in_dst, const int32_t* in_rel, int32_t* flag) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) flag[i] = (i == 0 || in_dst[i] != in_dst[i - 1] || in_rel[i] != in_rel[i - 1]) ? 1 : 0;
}
// sorted position i of the (rel, src) order: pair id = incl[i] - 1
__global__ void k_pairs(long long E, long long N, const u64* key, const uint32_t* pos, const int32_t* flag,
                        const int32_t* incl, const int32_t* in_dst, int32_t* in_pair, int32_t* pair_src,
                        int32_t* pair_rel, int32_t* out_ptr, int32_t* out_epos, int32_t* out_dst) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= E) return;
    const int32_t p = incl[i] - 1;
    const uint32_t c = pos[i];
    in_pair[c] = p;
    out_epos[i] = (int32_t)c;
    out_dst[i] = in_dst[c];
    if (flag[i]) {
        pair_src[p] = (int32_t)(key[i] % (u64)N);
        pair_rel[p] = (int32_t)(key[i] / (u64)N);
        out_ptr[p] = (int32_t)i;
    }
    if (i == E - 1) out_ptr[p + 1] = (int32_t)E;
}
__global__ void k_runs(long long E, const int32_t* flag, const int32_t* incl, const int32_t* in_dst,
                       const int32_t* in_rel, int32_t* in_run, int32_t* run_ptr, int32_t* run_dst, int32_t* run_rel) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= E) return;
    const int32_t q = incl[i] - 1;
    in_run[i] = q;
    if (flag[i]) { run_ptr[q] = (int32_t)i; run_dst[q] = in_dst[i]; run_rel[q] = in_rel[i]; }
    if (i == E - 1) run_ptr[q + 1] = (int32_t)E;
}
__global__ void k_cnt(long long E, const int32_t* in_run, const int32_t* run_ptr, int32_t* in_cnt, float* in_invc) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= E) return;
    const int32_t q = in_run[i], c = run_ptr[q + 1] - run_ptr[q];
    in_cnt[i] = c;
    in_invc[i] = 1.0f / (float)c;
}
__global__ void k_sorted_major(long long n, long long mul, const u64* key, const uint32_t* val, int32_t* major,
                               int32_t* perm) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    major[i] = (int32_t)(key[i] / (u64)mul);
    perm[i] = (int32_t)val[i];
}
// out_invc[j] = in_invc[out_epos[j]]: the per-edge norm coefficient in pair-major edge order
__global__ void k_permute_f32(long long n, const int32_t* idx, const float* src, float* dst) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[idx[i]];
}
__global__ void k_pair_ysel(long long P, const int32_t* out_ptr, const int32_t* out_dst, int32_t* ysel) {
    const long long p = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    const int32_t b = out_ptr[p];
    ysel[p] = (out_ptr[p + 1] - b == 1) ? (int32_t)((uint32_t)out_dst[b] | 0x80000000u) : (int32_t)p;
}
__global__ void k_pair_scale(long long P, const int32_t* out_ptr, const float* out_invc, float* scale) {
    const long long p = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    const int32_t b = out_ptr[p];
    scale[p] = (out_ptr[p + 1] - b == 1) ? out_invc[b] : 1.f;
}
__global__ void k_permute_i32(long long n, const int32_t* idx, const int32_t* src, int32_t* dst) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[idx[i]];
}
__global__ void k_tag(long long E, const int32_t* in_pair, const int32_t* out_ptr, int32_t* tag) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= E) return;
    const int32_t p = in_pair[i];
    tag[i] = (out_ptr[p + 1] - out_ptr[p] == 1) ? (int32_t)((uint32_t)p | 0x80000000u) : p;
}
// Pairs are in (relation, source) order: the first pair of a relation records its source's node type,
// and any pair whose successor in the same relation has a source of another type raises `mixed`.
__global__ void k_rel_type(long long P, const int32_t* pair_src, const int32_t* pair_rel, const int32_t* ntype,
                           int32_t* rel_type, int32_t* mixed) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= P) return;
    const int32_t r = pair_rel[i], t = ntype ? ntype[pair_src[i]] : 0;
    if (i == 0 || pair_rel[i - 1] != r) rel_type[r] = t;
    if (i + 1 < P && pair_rel[i + 1] == r && (ntype ? ntype[pair_src[i + 1]] : 0) != t) *mixed = 1;
}
__global__ void k_iota_key(long long n, const int32_t* major, u64* key, uint32_t* val) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    key[i] = (u64)(major ? major[i] : 0);
    val[i] = (uint32_t)i;
}

int bits_of(u64 max_key) {
    int b = 1;
    while (b < 64 && (max_key >> b) != 0) ++b;
    return b;
}

// stable sort of (key, val) by key over the significant bits of max_key
rgnn_status_t sort_pairs(u64* kin, u64* kout, uint32_t* vin, uint32_t* vout, size_t n, u64 max_key) {
    if (n == 0) return RGNN_OK;
    size_t bytes = 0;
    const unsigned end_bit = (unsigned)bits_of(max_key);
    RGNN_HIP(rocprim::radix_sort_pairs(nullptr, bytes, kin, kout, vin, vout, n, 0u, end_bit, (hipStream_t)0));
    Tmp t;
    RGNN_TRY(t.alloc(bytes));
    RGNN_HIP(rocprim::radix_sort_pairs(t.p, bytes, kin, kout, vin, vout, n, 0u, end_bit, (hipStream_t)0));
    RGNN_HIP(hipDeviceSynchronize());
    return RGNN_OK;
}
rgnn_status_t inclusive_scan(const int32_t* in, int32_t* out, size_t n) {
    if (n == 0) return RGNN_OK;
    size_t bytes = 0;
    RGNN_HIP(rocprim::inclusive_scan(nullptr, bytes, in, out, n, rocprim::plus<int32_t>(), (hipStream_t)0));
    Tmp t;
    RGNN_TRY(t.alloc(bytes));
    RGNN_HIP(rocprim::inclusive_scan(t.p, bytes, in, out, n, rocprim::plus<int32_t>(), (hipStream_t)0));
    RGNN_HIP(hipDeviceSynchronize());
    return RGNN_OK;
}

// device copy of an input array (uploaded when it lives on the host)
template <typename T>
rgnn_status_t input(Tmp& hold, const T* p, size_t n, int mem, const T** out) {
    if (!p || n == 0) { *out = nullptr; return RGNN_OK; }
    if (mem == RGNN_MEM_DEVICE) { *out = p; return RGNN_OK; }
    RGNN_TRY(hold.alloc(n * sizeof(T)));
    RGNN_HIP(hipMemcpy(hold.p, p, n * sizeof(T), hipMemcpyHostToDevice));
    *out = hold.as<T>();
    return RGNN_OK;
}

}  // namespace

// Fills g->idx[*], g->in_invc, g->out_invc, g->in_pair_tag, g->P, g->Q.  Synchronous.
rgnn_status_t build_index_device(rgnn_graph* g, int format, const int32_t* a, const int32_t* b, const int32_t* relp,
                                 const int32_t* ntypep, const int32_t* rstp, const int32_t* rdtp, int mem) {
    const long long N = g->N, E = g->E;
    const int R = g->R, T = g->T;
    const u64 uN = (u64)std::max<long long>(N, 1), uR = (u64)std::max(R, 1);

    Tmp h_src, h_b, h_rel, h_nt, h_rst, h_rdt, t_dst, t_err;
    const int32_t *src = nullptr, *bb = nullptr, *rel = nullptr, *ntype = nullptr, *rst = nullptr, *rdt = nullptr;
    RGNN_TRY(input(h_src, a, (size_t)E, mem, &src));
    RGNN_TRY(input(h_rel, relp, (size_t)E, mem, &rel));
    RGNN_TRY(input(h_b, b, format == RGNN_COO ? (size_t)E : (size_t)N + 1, mem, &bb));
    RGNN_TRY(input(h_nt, ntypep, (size_t)N, mem, &ntype));
    RGNN_TRY(input(h_rst, rstp, (size_t)R, mem, &rst));
    RGNN_TRY(input(h_rdt, rdtp, (size_t)R, mem, &rdt));
    RGNN_TRY(t_err.alloc(2 * sizeof(int)));
    {
        const int init[2] = {0, -1};   // code 0, index = UINT_MAX
        RGNN_HIP(hipMemcpy(t_err.p, init, sizeof(init), hipMemcpyHostToDevice));
    }
    int* err = t_err.as<int>();
    const int32_t* dst = bb;
    if (format == RGNN_CSR_DST) {
        LAUNCH(k_check_rowptr, (size_t)N + 1, N, E, bb, err);
        RGNN_TRY(t_dst.alloc((size_t)E * sizeof(int32_t)));
        int chk[2];
        RGNN_HIP(hipMemcpy(chk, err, sizeof(chk), hipMemcpyDeviceToHost));
        if (chk[0] == 4) RGNN_FAIL(RGNN_EINVAL, "CSR rowptr must start at 0, end at num_edges and be monotone (row %d)", chk[1]);
        LAUNCH(k_csr_rows, (size_t)E, N, E, bb, t_dst.as<int32_t>());
        dst = t_dst.as<int32_t>();
    }
    if (ntype) LAUNCH(k_check_ntype, (size_t)N, N, T, ntype, err);

    // ---- 1. CSR order
    Tmp k0, k1, v0, v1, flag, incl;
    const size_t maxn = (size_t)std::max<long long>(std::max<long long>(E, N), 1);
    RGNN_TRY(k0.alloc(maxn * sizeof(u64)));
    RGNN_TRY(k1.alloc(maxn * sizeof(u64)));
    RGNN_TRY(v0.alloc(maxn * sizeof(uint32_t)));
    RGNN_TRY(v1.alloc(maxn * sizeof(uint32_t)));
    RGNN_TRY(flag.alloc(maxn * sizeof(int32_t)));
    RGNN_TRY(incl.alloc(maxn * sizeof(int32_t)));
    LAUNCH(k_key_csr, (size_t)E, E, N, R, src, dst, rel, ntype, rst, rdt, k0.as<u64>(), v0.as<uint32_t>(), err);
    {
        int chk[2];
        RGNN_HIP(hipMemcpy(chk, err, sizeof(chk), hipMemcpyDeviceToHost));
        if (chk[0] == 1) RGNN_FAIL(RGNN_EINVAL, "edge %d has a node or relation id out of range (N = %lld, R = %d)", chk[1], N, R);
        if (chk[0] == 2) RGNN_FAIL(RGNN_EINVAL, "edge %d: node types do not match the types its relation is tied to", chk[1]);
        if (chk[0] == 3) RGNN_FAIL(RGNN_EINVAL, "ntype[%d] out of range [0, %d)", chk[1], T);
    }
    RGNN_TRY(sort_pairs(k0.as<u64>(), k1.as<u64>(), v0.as<uint32_t>(), v1.as<uint32_t>(), (size_t)E, uN * uR * uN));
    RGNN_TRY(keep_idx(g, RGNN_IDX_IN_PTR, (size_t)N + 1));
    RGNN_TRY(keep_idx(g, RGNN_IDX_IN_SRC, (size_t)E));
    RGNN_TRY(keep_idx(g, RGNN_IDX_IN_REL, (size_t)E));
    RGNN_TRY(keep_idx(g, RGNN_IDX_IN_EID, (size_t)E));
    Tmp in_dst_t;
    RGNN_TRY(in_dst_t.alloc((size_t)E * sizeof(int32_t)));
    int32_t* in_dst = in_dst_t.as<int32_t>();
    LAUNCH(k_decode_csr, (size_t)E, E, (long long)uN, (int)uR, k1.as<u64>(), v1.as<uint32_t>(), g->idx[RGNN_IDX_IN_SRC],
           g->idx[RGNN_IDX_IN_REL], in_dst, g->idx[RGNN_IDX_IN_EID]);
    LAUNCH(k_lower_bound, (size_t)N + 1, E, in_dst, N, g->idx[RGNN_IDX_IN_PTR]);

    // ---- 2. pairs and the pair-major transpose
    RGNN_TRY(keep_idx(g, RGNN_IDX_IN_PAIR, (size_t)E));
    RGNN_TRY(keep_idx(g, RGNN_IDX_OUT_EPOS, (size_t)E));
    RGNN_TRY(keep_idx(g, RGNN_IDX_OUT_DST, (size_t)E));
    LAUNCH(k_key2, (size_t)E, E, (long long)uN, g->idx[RGNN_IDX_IN_REL], g->idx[RGNN_IDX_IN_SRC], k0.as<u64>(), v0.as<uint32_t>());
    RGNN_TRY(sort_pairs(k0.as<u64>(), k1.as<u64>(), v0.as<uint32_t>(), v1.as<uint32_t>(), (size_t)E, uR * uN));
    LAUNCH(k_flag_key, (size_t)E, E, k1.as<u64>(), flag.as<int32_t>());
    RGNN_TRY(inclusive_scan(flag.as<int32_t>(), incl.as<int32_t>(), (size_t)E));
    int32_t P = 0;
    if (E > 0) RGNN_HIP(hipMemcpy(&P, incl.as<int32_t>() + (E - 1), sizeof(int32_t), hipMemcpyDeviceToHost));
    g->P = P;
    RGNN_TRY(keep_idx(g, RGNN_IDX_PAIR_SRC, (size_t)P));
    RGNN_TRY(keep_idx(g, RGNN_IDX_PAIR_REL, (size_t)P));
    RGNN_TRY(keep_idx(g, RGNN_IDX_OUT_PTR, (size_t)P + 1));
    RGNN_TRY(keep_idx(g, RGNN_IDX_PAIR_PTR, (size_t)R + 1));
    if (E == 0) RGNN_HIP(hipMemset(g->idx[RGNN_IDX_OUT_PTR], 0, sizeof(int32_t)));
    LAUNCH(k_pairs, (size_t)E, E, (long long)uN, k1.as<u64>(), v1.as<uint32_t>(), flag.as<int32_t>(), incl.as<int32_t>(),
           in_dst, g->idx[RGNN_IDX_IN_PAIR], g->idx[RGNN_IDX_PAIR_SRC], g->idx[RGNN_IDX_PAIR_REL],
           g->idx[RGNN_IDX_OUT_PTR], g->idx[RGNN_IDX_OUT_EPOS], g->idx[RGNN_IDX_OUT_DST]);
    LAUNCH(k_lower_bound, (size_t)R + 1, (long long)P, g->idx[RGNN_IDX_PAIR_REL], (long long)R, g->idx[RGNN_IDX_PAIR_PTR]);

    // ---- 3. runs
    RGNN_TRY(keep_idx(g, RGNN_IDX_IN_RUN, (size_t)E));
    RGNN_TRY(keep_idx(g, RGNN_IDX_IN_CNT, (size_t)E));
    RGNN_TRY(keep<float>(g, (size_t)E, &g->in_invc));
    LAUNCH(k_flag_runs, (size_t)E, E, in_dst, g->idx[RGNN_IDX_IN_REL], flag.as<int32_t>());
    RGNN_TRY(inclusive_scan(flag.as<int32_t>(), incl.as<int32_t>(), (size_t)E));
    int32_t Q = 0;
    if (E > 0) RGNN_HIP(hipMemcpy(&Q, incl.as<int32_t>() + (E - 1), sizeof(int32_t), hipMemcpyDeviceToHost));
    g->Q = Q;
    RGNN_TRY(keep_idx(g, RGNN_IDX_RUN_PTR, (size_t)Q + 1));
    RGNN_TRY(keep_idx(g, RGNN_IDX_RUN_DST, (size_t)Q));
    RGNN_TRY(keep_idx(g, RGNN_IDX_RUN_REL, (size_t)Q));
    RGNN_TRY(keep_idx(g, RGNN_IDX_DST_RUN_PTR, (size_t)N + 1));
    if (E == 0) RGNN_HIP(hipMemset(g->idx[RGNN_IDX_RUN_PTR], 0, sizeof(int32_t)));
    LAUNCH(k_runs, (size_t)E, E, flag.as<int32_t>(), incl.as<int32_t>(), in_dst, g->idx[RGNN_IDX_IN_REL],
           g->idx[RGNN_IDX_IN_RUN], g->idx[RGNN_IDX_RUN_PTR], g->idx[RGNN_IDX_RUN_DST], g->idx[RGNN_IDX_RUN_REL]);
    LAUNCH(k_cnt, (size_t)E, E, g->idx[RGNN_IDX_IN_RUN], g->idx[RGNN_IDX_RUN_PTR], g->idx[RGNN_IDX_IN_CNT], g->in_invc);
    LAUNCH(k_lower_bound, (size_t)N + 1, (long long)Q, g->idx[RGNN_IDX_RUN_DST], N, g->idx[RGNN_IDX_DST_RUN_PTR]);

    // ---- 4. runs by (rel, dst)
    RGNN_TRY(keep_idx(g, RGNN_IDX_RELRUN_IDX, (size_t)Q));
    RGNN_TRY(keep_idx(g, RGNN_IDX_RELRUN_PTR, (size_t)R + 1));
    LAUNCH(k_key2, (size_t)Q, (long long)Q, (long long)uN, g->idx[RGNN_IDX_RUN_REL], g->idx[RGNN_IDX_RUN_DST], k0.as<u64>(), v0.as<uint32_t>());
    RGNN_TRY(sort_pairs(k0.as<u64>(), k1.as<u64>(), v0.as<uint32_t>(), v1.as<uint32_t>(), (size_t)Q, uR * uN));
    LAUNCH(k_sorted_major, (size_t)Q, (long long)Q, (long long)uN, k1.as<u64>(), v1.as<uint32_t>(), flag.as<int32_t>(), g->idx[RGNN_IDX_RELRUN_IDX]);
    LAUNCH(k_lower_bound, (size_t)R + 1, (long long)Q, flag.as<int32_t>(), (long long)R, g->idx[RGNN_IDX_RELRUN_PTR]);
    RGNN_TRY(keep<int32_t>(g, (size_t)Q, &g->relrun_dst));
    LAUNCH(k_permute_i32, (size_t)Q, (long long)Q, g->idx[RGNN_IDX_RELRUN_IDX], g->idx[RGNN_IDX_RUN_DST], g->relrun_dst);
    g->idx[RGNN_IDX_RELRUN_DST] = g->relrun_dst; g->idx_len[RGNN_IDX_RELRUN_DST] = Q;

    // ---- 5. pairs by (src, rel)
    RGNN_TRY(keep_idx(g, RGNN_IDX_SRCPAIR_IDX, (size_t)P));
    RGNN_TRY(keep_idx(g, RGNN_IDX_SRCPAIR_PTR, (size_t)N + 1));
    LAUNCH(k_key2, (size_t)P, (long long)P, (long long)uR, g->idx[RGNN_IDX_PAIR_SRC], g->idx[RGNN_IDX_PAIR_REL], k0.as<u64>(), v0.as<uint32_t>());
    RGNN_TRY(sort_pairs(k0.as<u64>(), k1.as<u64>(), v0.as<uint32_t>(), v1.as<uint32_t>(), (size_t)P, uN * uR));
    LAUNCH(k_sorted_major, (size_t)P, (long long)P, (long long)uR, k1.as<u64>(), v1.as<uint32_t>(), flag.as<int32_t>(), g->idx[RGNN_IDX_SRCPAIR_IDX]);
    LAUNCH(k_lower_bound, (size_t)N + 1, (long long)P, flag.as<int32_t>(), N, g->idx[RGNN_IDX_SRCPAIR_PTR]);

    // ---- 6. nodes by (type, id)
    RGNN_TRY(keep_idx(g, RGNN_IDX_NTYPE_PERM, (size_t)N));
    RGNN_TRY(keep_idx(g, RGNN_IDX_NTYPE_PTR, (size_t)T + 1));
    LAUNCH(k_iota_key, (size_t)N, N, ntype, k0.as<u64>(), v0.as<uint32_t>());
    RGNN_TRY(sort_pairs(k0.as<u64>(), k1.as<u64>(), v0.as<uint32_t>(), v1.as<uint32_t>(), (size_t)N, (u64)std::max(T, 1)));
    LAUNCH(k_sorted_major, (size_t)N, N, 1LL, k1.as<u64>(), v1.as<uint32_t>(), flag.as<int32_t>(), g->idx[RGNN_IDX_NTYPE_PERM]);
    LAUNCH(k_lower_bound, (size_t)T + 1, N, flag.as<int32_t>(), (long long)T, g->idx[RGNN_IDX_NTYPE_PTR]);

    // ---- 7. pair ids tagged with "single edge"
    RGNN_TRY(keep<int32_t>(g, (size_t)E, &g->in_pair_tag));
    LAUNCH(k_tag, (size_t)E, E, g->idx[RGNN_IDX_IN_PAIR], g->idx[RGNN_IDX_OUT_PTR], g->in_pair_tag);
    g->idx[RGNN_IDX_IN_PAIR_TAG] = g->in_pair_tag; g->idx_len[RGNN_IDX_IN_PAIR_TAG] = E;
    RGNN_TRY(keep<float>(g, (size_t)E, &g->out_invc));
    LAUNCH(k_permute_f32, (size_t)E, E, g->idx[RGNN_IDX_OUT_EPOS], g->in_invc, g->out_invc);
    RGNN_TRY(keep<int32_t>(g, (size_t)P, &g->pair_ysel));
    LAUNCH(k_pair_ysel, (size_t)P, (long long)P, g->idx[RGNN_IDX_OUT_PTR], g->idx[RGNN_IDX_OUT_DST], g->pair_ysel);
    g->idx[RGNN_IDX_PAIR_SEL_DST] = g->pair_ysel; g->idx_len[RGNN_IDX_PAIR_SEL_DST] = P;
    RGNN_TRY(keep<float>(g, (size_t)P, &g->pair_scale));
    LAUNCH(k_pair_scale, (size_t)P, (long long)P, g->idx[RGNN_IDX_OUT_PTR], g->out_invc, g->pair_scale);

    // ---- 8. node type of each relation's sources, if it is a single one
    RGNN_TRY(keep<int32_t>(g, (size_t)R, &g->rel_src_type));
    Tmp mixed_t;
    RGNN_TRY(mixed_t.alloc(sizeof(int32_t)));
    RGNN_HIP(hipMemset(g->rel_src_type, 0, (size_t)R * sizeof(int32_t)));
    RGNN_HIP(hipMemset(mixed_t.as<int32_t>(), 0, sizeof(int32_t)));
    LAUNCH(k_rel_type, (size_t)P, (long long)P, g->idx[RGNN_IDX_PAIR_SRC], g->idx[RGNN_IDX_PAIR_REL], ntype, g->rel_src_type,
           mixed_t.as<int32_t>());
    int32_t mixed = 0;
    RGNN_HIP(hipMemcpy(&mixed, mixed_t.as<int32_t>(), sizeof(int32_t), hipMemcpyDeviceToHost));
    g->rel_src_tied = mixed == 0;
    g->idx[RGNN_IDX_REL_SRC_TYPE] = g->rel_src_type; g->idx_len[RGNN_IDX_REL_SRC_TYPE] = R;
    RGNN_HIP(hipDeviceSynchronize());
    return RGNN_OK;
}

}  // namespace rgnn
