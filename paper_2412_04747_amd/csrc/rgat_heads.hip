// Pieces of multi-head RGAT that the single-head path does not have.  With H heads the d_out
// columns split into H slices of d_out / H; head h of an edge uses the slices of hs, ht, w_s[r]
// and w_t[r] (the single-head formulas of the thesis' RGAT listing, applied per slice, outputs
// concatenated).  The rest of the multi-head path reuses the typed-linear kernels, the per-head
// softmax / edge-dot kernels of the HGT layer and the gather-sum with one coefficient per head.
#include "rgnn_internal.h"
#include "traversal.h"
#include "device_utils.h"

namespace rgnn {

// wv[r][h][k] = sum_{n in head h} W[r][k][n] * w[r][n]   (linear operator reordering, per head; the H vectors
// of a relation are adjacent, so the walks that need all of them touch one short block)
__global__ void fold_weight_heads_kernel(const float* __restrict__ W, const float* __restrict__ w, int R, int kd, int nd,
                                         int H, float* __restrict__ wv) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;   // (r, h, k)
    if (i >= H * R * kd) return;
    const int dh = nd / H;
    const int r = i / (H * kd), h = i / kd % H, k = i % kd;
    const float* Wr = W + ((size_t)r * kd + k) * nd + h * dh;
    const float* wr = w + (size_t)r * nd + h * dh;
    float s = 0.f;
    for (int n = 0; n < dh; ++n) s += Wr[n] * wr[n];
    wv[i] = s;
}

// s_dst[q][h] = X[run_dst[q]] . wtp[run_rel[q]][h]: the run's X row is read once, one full-width dot per head; a lane
// group takes four consecutive runs so that four row reads (and the heads' folded vectors) are in flight per lane
template <int D>
__global__ __launch_bounds__(256) void run_logit_heads_kernel(int Q, int R, int H, const int32_t* __restrict__ run_dst,
                                                              const int32_t* __restrict__ run_rel,
                                                              const float* __restrict__ X, const float* __restrict__ wtp,
                                                              float* __restrict__ s_dst) {
    constexpr int LPR = D / 4;
    const int q0 = (blockIdx.x * (256 / LPR) + threadIdx.x / LPR) * 4, c4 = threadIdx.x % LPR;
    if (q0 >= Q) return;
    float4 x[4];
    int r[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int q = min(q0 + u, Q - 1);
        x[u] = *reinterpret_cast<const float4*>(X + (size_t)run_dst[q] * D + c4 * 4);
        r[u] = run_rel[q];
    }
    for (int h = 0; h < H; ++h) {
        float4 w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) w[u] = *reinterpret_cast<const float4*>(wtp + ((size_t)r[u] * H + h) * D + c4 * 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float t = group_sum<LPR>(dot4(x[u], w[u]));
            if (c4 == 0 && q0 + u < Q) s_dst[(size_t)(q0 + u) * H + h] = t;
        }
    }
}

// Per relation r, with U[h][r] = sum_q ds_dst[q][h] X[dst_q] and h(n) the head of column n:
//   dw_t[r][n] = sum_k U[h(n)][r][k] W[r][k][n];   dW[r][k][n] += U[h(n)][r][k] * w_t[r][n]
// and, where A[r][h] = sum_p ds_src[p][h] X[src_p] is given (otherwise the caller forms dw_s from the message rows),
//   dw_s[r][n] = sum_k A[r][h(n)][k] W[r][k][n]
__global__ void rgat_heads_param_finish_kernel(int R, int kd, int nd, int H, const float* __restrict__ W,
                                               const float* __restrict__ w_t, const float* __restrict__ U,
                                               const float* __restrict__ A, float* __restrict__ dW,
                                               float* __restrict__ dw_s, float* __restrict__ dw_t) {
    const int r = blockIdx.x, dh = nd / H;
    const float* Wr = W + (size_t)r * kd * nd;
    for (int n = threadIdx.x; n < nd; n += blockDim.x) {
        const float* Ur = U + ((size_t)(n / dh) * R + r) * kd;
        float t = 0.f;
        for (int k = 0; k < kd; ++k) t += Ur[k] * Wr[k * nd + n];
        dw_t[(size_t)r * nd + n] = t;
        if (A) {
            const float* Ar = A + ((size_t)r * H + n / dh) * kd;
            float s = 0.f;
            for (int k = 0; k < kd; ++k) s += Ar[k] * Wr[k * nd + n];
            dw_s[(size_t)r * nd + n] = s;
        }
    }
    for (int i = threadIdx.x; i < kd * nd; i += blockDim.x) {
        const int k = i / nd, n = i % nd;
        dW[(size_t)r * kd * nd + i] += U[((size_t)(n / dh) * R + r) * kd + k] * w_t[(size_t)r * nd + n];
    }
}

// ---------------------------------------------------------------------------------------- launchers

rgnn_status_t fold_weight_heads(int R, int kd, int nd, int H, const float* W, const float* w, float* wv, hipStream_t st) {
    KernelTimer kt(st, "fold_weight");
    hipLaunchKernelGGL(fold_weight_heads_kernel, dim3(blocks_for((size_t)H * R * kd, 256)), dim3(256), 0, st, W, w, R, kd,
                       nd, H, wv);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}

rgnn_status_t run_logit_heads(const rgnn_graph* g, int D, int H, const float* X, const float* wtp, float* s_dst,
                              hipStream_t st) {
    if (g->Q == 0) return RGNN_OK;
    KernelTimer kt(st, "run_logit");
    RGNN_DISPATCH_D(D, hipLaunchKernelGGL(run_logit_heads_kernel<DD>, dim3(blocks_for((size_t)((g->Q + 3) / 4) * (DD / 4), 256)), dim3(256),
                                          0, st, (int)g->Q, (int)g->R, H, g->idx[RGNN_IDX_RUN_DST], g->idx[RGNN_IDX_RUN_REL], X,
                                          wtp, s_dst));
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}

rgnn_status_t rgat_heads_param_finish(int R, int kd, int nd, int H, const float* W, const float* w_t, const float* U,
                                      const float* A, float* dW, float* dw_s, float* dw_t, hipStream_t st) {
    KernelTimer kt(st, "rgat_param_finish");
    hipLaunchKernelGGL(rgat_heads_param_finish_kernel, dim3(R), dim3(256), 0, st, R, kd, nd, H, W, w_t, U, A, dW, dw_s, dw_t);
    RGNN_CHECK_LAUNCH();
    return RGNN_OK;
}

}  // namespace rgnn
