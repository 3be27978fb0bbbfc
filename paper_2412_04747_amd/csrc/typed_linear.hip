// Relation-segmented typed linear layer on the CDNA4 matrix cores, fp32.
//
// Forward   Y[i] = X[gather[i]] W[seg(i)]          (thesis Ch.3: segment MM, Y[S] = X[G] x W[T];
//                                                   rows are presorted by type so one weight serves a segment)
// Backward  dXrow[i] = dY[i] W[seg(i)]^T,  dW[s] = sum_{i in s} X[gather[i]]^T dY[i]
//
// Rows are cut into 64-row tiles that never straddle a segment; a persistent workgroup of
// four wavefronts walks a contiguous chunk of tiles and keeps the current segment's weight
// in LDS, reloading it only when the segment changes.  The 64x64-wide products run on
// v_mfma_f32_32x32x2_f32.  The K index of the MFMA is a free permutation, so each lane
// reads its A operand as 16-byte LDS vectors: lane (m, half) owns k = half*K/2 + 0..K/2-1.
#include "rgnn_internal.h"

#include <algorithm>

namespace rgnn {

typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ v16f mfma32(float a, float b, v16f c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Row of the 32x32 accumulator held in register v of a lane in half `h` (lane / 32);
// the column is lane % 32.
__device__ __forceinline__ int acc_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

struct TileArgs {
    const int32_t* tile_seg;
    const int32_t* tile_row0;
    const int32_t* tile_row1;
    const int32_t* chunk_tile;
    const int32_t* chunk_slot;
};

constexpr int TM = kTileRows;

// ---------------------------------------------------------------------------------------
// Forward.  Software pipeline per workgroup: the rows of tile t+1 are fetched from HBM
// into registers while tile t is multiplied out of LDS, so the gather latency (index, then
// row) hides behind the MFMAs and the epilogue.  Two barriers per tile: one after the
// input tile is written to LDS, one after the accumulators are staged for the coalesced
// 16-byte row stores.
template <int KD, int ND>
__global__ __launch_bounds__(256) void typed_linear_fwd_kernel(TileArgs t, const float* __restrict__ X,
                                                               const int32_t* __restrict__ gather,
                                                               const float* __restrict__ W, float* __restrict__ Y,
                                                               int scatter_out, int accumulate,
                                                               const float* __restrict__ vec, float* __restrict__ s_out) {
    constexpr int XS = KD + 4, YS = ND + 4;
    constexpr int CB = ND / 32, NBLK = 2 * CB, NBW = (NBLK + 3) / 4;
    constexpr int LPRI = KD / 4, RPPI = 256 / LPRI, NX = TM / RPPI;   // input rows: lanes per row, rows per pass, passes
    constexpr int LPRO = ND / 4, RPPO = 256 / LPRO;
    extern __shared__ __align__(16) float smem[];
    float* Ws = smem;                 // [KD][ND]
    float* Xs = Ws + KD * ND;         // [TM][XS]
    float* Ys = Xs + TM * XS;         // [TM][YS]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 31, kh = lane >> 5, rb = wave & 1;
    const int ci = tid % LPRI, ri = tid / LPRI;
    const int t0 = t.chunk_tile[blockIdx.x], t1 = t.chunk_tile[blockIdx.x + 1];
    float4 xr[NX];
    auto fetch = [&](int ti) {
        const int row0 = t.tile_row0[ti], row1 = t.tile_row1[ti];
#pragma unroll
        for (int it = 0; it < NX; ++it) {
            const int row = row0 + ri + it * RPPI;
            xr[it] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < row1) {
                const size_t s = gather ? (size_t)gather[row] : (size_t)row;
                xr[it] = *reinterpret_cast<const float4*>(X + s * KD + ci * 4);
            }
        }
    };
    if (t0 < t1) fetch(t0);
    int cur_seg = -1;
    for (int ti = t0; ti < t1; ++ti) {
        const int seg = t.tile_seg[ti], row0 = t.tile_row0[ti], row1 = t.tile_row1[ti];
        if (seg != cur_seg) {
            const float4* Wg = reinterpret_cast<const float4*>(W + (size_t)seg * KD * ND);
            for (int i = tid; i < KD * ND / 4; i += 256) reinterpret_cast<float4*>(Ws)[i] = Wg[i];
            cur_seg = seg;
        }
#pragma unroll
        for (int it = 0; it < NX; ++it)
            *reinterpret_cast<float4*>(Xs + (ri + it * RPPI) * XS + ci * 4) = xr[it];
        __syncthreads();
        if (ti + 1 < t1) fetch(ti + 1);
        v16f acc[NBW];
#pragma unroll
        for (int b = 0; b < NBW; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
        if (wave < NBLK) {
#pragma unroll 2
            for (int tt = 0; tt < KD / 8; ++tt) {
                const int k0 = kh * (KD / 2) + 4 * tt;
                const float4 a4 = *reinterpret_cast<const float4*>(Xs + (rb * 32 + m) * XS + k0);
                const float av[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int b = 0; b < NBW; ++b) {
                        const int cb = (wave >> 1) + 2 * b;
                        acc[b] = mfma32(av[i], Ws[(k0 + i) * ND + cb * 32 + m], acc[b]);
                    }
            }
#pragma unroll
            for (int b = 0; b < NBW; ++b) {
                const int cb = (wave >> 1) + 2 * b;
#pragma unroll
                for (int v = 0; v < 16; ++v) Ys[(rb * 32 + acc_row(v, kh)) * YS + cb * 32 + m] = acc[b][v];
            }
        }
        __syncthreads();
        {
            const int c4 = tid % LPRO;
            float4 wv = make_float4(0.f, 0.f, 0.f, 0.f);
            if (vec) wv = *reinterpret_cast<const float4*>(vec + (size_t)seg * ND + c4 * 4);
            for (int r = tid / LPRO; r < TM; r += RPPO) {
                const int row = row0 + r;
                const bool ok = row < row1;
                float4 y = *reinterpret_cast<const float4*>(Ys + r * YS + c4 * 4);
                if (ok) {
                    const size_t d = (scatter_out && gather) ? (size_t)gather[row] : (size_t)row;
                    float4* yp = reinterpret_cast<float4*>(Y + d * ND + c4 * 4);
                    if (accumulate) {
                        const float4 o = *yp;
                        y.x += o.x; y.y += o.y; y.z += o.z; y.w += o.w;
                    }
                    *yp = y;
                }
                if (vec) {
                    float s = y.x * wv.x + y.y * wv.y + y.z * wv.z + y.w * wv.w;
#pragma unroll
                    for (int o = LPRO / 2; o > 0; o >>= 1) s += __shfl_xor(s, o);
                    if (ok && c4 == 0) s_out[row] = s;
                }
            }
        }
        // no barrier here: the next iteration's writes go to Xs (all MFMA reads of it are
        // behind the barrier above) and Ys is rewritten only after the next barrier.
    }
}

// ---------------------------------------------------------------------------------------
// Backward tile: dY_eff[i] = dY[i] + rowscale[i] * vec[seg]   (the rank-1 term lets the caller
// fold d(row . vec)/d row into the same pass), then
//   dXrow[i]  = dY_eff[i] W^T                      (MFMA, contraction over the output features)
//   dW[seg]  += X_tile^T dY_eff                    (MFMA, contraction over the tile's rows)
//   Avec[seg]+= sum_i rowscale[i] X_tile[i]        (vector ALU)
// dW and Avec stay in registers while consecutive tiles share a segment and are flushed to
// the chunk's partial slot when the segment changes; a second kernel sums the slots of each
// segment in slot order, so the result does not depend on scheduling.
template <int KD, int ND>
__global__ __launch_bounds__(256) void typed_linear_bwd_kernel(TileArgs t, const float* __restrict__ X,
                                                               const int32_t* __restrict__ gather,
                                                               const float* __restrict__ W,
                                                               const float* __restrict__ dY, int dy_gathered,
                                                               float* __restrict__ dXrow, int scatter_dx,
                                                               const float* __restrict__ rowscale,
                                                               const float* __restrict__ vec,
                                                               float* __restrict__ part) {
    constexpr int XS = KD + 4, YS = ND + 4, WS = ND + 1;
    constexpr int STG = (XS > YS ? XS : YS);
    constexpr int KB = KD / 32, NB = ND / 32;
    constexpr int DBLK = 2 * KB, DBW = (DBLK + 3) / 4;   // dXrow blocks (row block, k block) per wave
    constexpr int WBLK = KB * NB, WBW = (WBLK + 3) / 4;  // dW blocks (k block, n block) per wave
    constexpr int AG = 256 / KD;                         // row groups of the Avec accumulation
    constexpr int SLOT = KD * ND + KD;
    extern __shared__ __align__(16) float smem[];
    float* Ws = smem;                 // [KD][WS]
    float* dYs = Ws + KD * WS;        // [TM][STG]  (also the dXrow stage)
    float* Xs = dYs + TM * STG;       // [TM][XS]
    float* dss = Xs + TM * XS;        // [TM]
    float* red = dss + TM;            // [256]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 31, kh = lane >> 5, rb = wave & 1;
    v16f accw[WBW];
#pragma unroll
    for (int b = 0; b < WBW; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) accw[b][v] = 0.f;
    float acca = 0.f;
    int cur_seg = -1;
    int slot = t.chunk_slot[blockIdx.x] - 1;
    const int t0 = t.chunk_tile[blockIdx.x], t1 = t.chunk_tile[blockIdx.x + 1];
    for (int ti = t0; ti <= t1; ++ti) {
        const int seg = (ti < t1) ? t.tile_seg[ti] : -2;
        if (seg != cur_seg) {
            if (cur_seg >= 0) {  // flush the finished segment's partial sums
                float* ps = part + (size_t)slot * SLOT;
                if (wave < WBLK) {
#pragma unroll
                    for (int b = 0; b < WBW; ++b) {
                        const int blk = wave + 4 * b, kb = blk % KB, nb = blk / KB;
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            ps[(kb * 32 + acc_row(v, kh)) * ND + nb * 32 + m] = accw[b][v];
                            accw[b][v] = 0.f;
                        }
                    }
                }
                red[tid] = acca;
                acca = 0.f;
                __syncthreads();
                if (tid < KD) {
                    float s = 0.f;
#pragma unroll
                    for (int g2 = 0; g2 < AG; ++g2) s += red[g2 * KD + tid];
                    ps[KD * ND + tid] = s;
                }
                __syncthreads();
            }
            if (ti == t1) break;
            ++slot;
            const float* Wg = W + (size_t)seg * KD * ND;
            for (int i = tid; i < KD * ND; i += 256) Ws[(i / ND) * WS + (i % ND)] = Wg[i];
            cur_seg = seg;
        }
        const int row0 = t.tile_row0[ti], row1 = t.tile_row1[ti];
        if (tid < TM) dss[tid] = (rowscale && row0 + tid < row1) ? rowscale[row0 + tid] : 0.f;
        {
            constexpr int LPR = KD / 4, RPP = 256 / LPR;
            const int c4 = tid % LPR;
            for (int r = tid / LPR; r < TM; r += RPP) {
                const int row = row0 + r;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (row < row1) {
                    const size_t s = gather ? (size_t)gather[row] : (size_t)row;
                    v = *reinterpret_cast<const float4*>(X + s * KD + c4 * 4);
                }
                *reinterpret_cast<float4*>(Xs + r * XS + c4 * 4) = v;
            }
        }
        {
            constexpr int LPR = ND / 4, RPP = 256 / LPR;
            const int c4 = tid % LPR;
            float4 wv = make_float4(0.f, 0.f, 0.f, 0.f);
            if (vec) wv = *reinterpret_cast<const float4*>(vec + (size_t)seg * ND + c4 * 4);
            for (int r = tid / LPR; r < TM; r += RPP) {
                const int row = row0 + r;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (row < row1) {
                    const size_t s = (dy_gathered && gather) ? (size_t)gather[row] : (size_t)row;
                    v = *reinterpret_cast<const float4*>(dY + s * ND + c4 * 4);
                    if (rowscale && vec) {
                        const float sc = rowscale[row];
                        v.x += sc * wv.x; v.y += sc * wv.y; v.z += sc * wv.z; v.w += sc * wv.w;
                    }
                }
                *reinterpret_cast<float4*>(dYs + r * STG + c4 * 4) = v;
            }
        }
        __syncthreads();
        // dXrow tile: rows x KD, contraction over n
        v16f accx[DBW];
#pragma unroll
        for (int b = 0; b < DBW; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) accx[b][v] = 0.f;
        if (wave < DBLK) {
#pragma unroll 2
            for (int tt = 0; tt < ND / 8; ++tt) {
                const int n0 = kh * (ND / 2) + 4 * tt;
                const float4 a4 = *reinterpret_cast<const float4*>(dYs + (rb * 32 + m) * STG + n0);
                const float av[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int b = 0; b < DBW; ++b) {
                        const int cb = (wave >> 1) + 2 * b;
                        accx[b] = mfma32(av[i], Ws[(cb * 32 + m) * WS + n0 + i], accx[b]);
                    }
            }
        }
        // dW blocks: KD x ND, contraction over the tile's rows (two rows per MFMA)
        if (wave < WBLK) {
#pragma unroll 4
            for (int s = 0; s < TM / 2; ++s) {
                const int r = 2 * s + kh;
#pragma unroll
                for (int b = 0; b < WBW; ++b) {
                    const int blk = wave + 4 * b, kb = blk % KB, nb = blk / KB;
                    accw[b] = mfma32(Xs[r * XS + kb * 32 + m], dYs[r * STG + nb * 32 + m], accw[b]);
                }
            }
        }
        if (rowscale) {
            const int k = tid % KD;
            for (int r = tid / KD; r < TM; r += AG) acca += dss[r] * Xs[r * XS + k];
        }
        __syncthreads();  // all reads of dYs done; reuse it to stage dXrow
        if (wave < DBLK) {
#pragma unroll
            for (int b = 0; b < DBW; ++b) {
                const int cb = (wave >> 1) + 2 * b;
#pragma unroll
                for (int v = 0; v < 16; ++v) dYs[(rb * 32 + acc_row(v, kh)) * STG + cb * 32 + m] = accx[b][v];
            }
        }
        __syncthreads();
        {
            constexpr int LPR = KD / 4, RPP = 256 / LPR;
            const int c4 = tid % LPR;
            for (int r = tid / LPR; r < TM; r += RPP) {
                const int row = row0 + r;
                if (row < row1) {
                    const size_t d = (scatter_dx && gather) ? (size_t)gather[row] : (size_t)row;
                    *reinterpret_cast<float4*>(dXrow + d * KD + c4 * 4) =
                        *reinterpret_cast<const float4*>(dYs + r * STG + c4 * 4);
                }
            }
        }
        __syncthreads();
    }
}

// Pipelined variant of the backward tile kernel for feature widths up to 64: the X and dY
// rows of tile t+1 are fetched into registers while tile t is processed, and dXrow is staged
// in its own LDS buffer so that two barriers per tile suffice.
template <int KD, int ND>
__global__ __launch_bounds__(256) void typed_linear_bwd_pipe_kernel(TileArgs t, const float* __restrict__ X,
                                                                    const int32_t* __restrict__ gather,
                                                                    const float* __restrict__ W,
                                                                    const float* __restrict__ dY, int dy_gathered,
                                                                    float* __restrict__ dXrow, int scatter_dx,
                                                                    const float* __restrict__ rowscale,
                                                                    const float* __restrict__ vec,
                                                                    float* __restrict__ part) {
    constexpr int XS = KD + 4, YS = ND + 4, WS = ND + 1;
    constexpr int KB = KD / 32, NB = ND / 32;
    constexpr int DBLK = 2 * KB, DBW = (DBLK + 3) / 4;
    constexpr int WBLK = KB * NB, WBW = (WBLK + 3) / 4;
    constexpr int AG = 256 / KD;
    constexpr int SLOT = KD * ND + KD;
    constexpr int LPRX = KD / 4, RPPX = 256 / LPRX, NXR = TM / RPPX;
    constexpr int LPRY = ND / 4, RPPY = 256 / LPRY, NYR = TM / RPPY;
    extern __shared__ __align__(16) float smem[];
    float* Ws = smem;                 // [KD][WS]
    float* dYs = Ws + KD * WS;        // [TM][YS]
    float* Xs = dYs + TM * YS;        // [TM][XS]
    float* DXs = Xs + TM * XS;        // [TM][XS]  dXrow stage
    float* dss = DXs + TM * XS;       // [TM]
    float* red = dss + TM;            // [256]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 31, kh = lane >> 5, rb = wave & 1;
    const int cx = tid % LPRX, rx = tid / LPRX, cy = tid % LPRY, ry = tid / LPRY;
    v16f accw[WBW];
#pragma unroll
    for (int b = 0; b < WBW; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) accw[b][v] = 0.f;
    float acca = 0.f;
    const int t0 = t.chunk_tile[blockIdx.x], t1 = t.chunk_tile[blockIdx.x + 1];
    float4 xr[NXR], yr[NYR];
    float sr[NYR];
    float dsr = 0.f;
    auto fetch = [&](int ti) {
        const int row0 = t.tile_row0[ti], row1 = t.tile_row1[ti];
#pragma unroll
        for (int it = 0; it < NXR; ++it) {
            const int row = row0 + rx + it * RPPX;
            xr[it] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < row1) {
                const size_t s = gather ? (size_t)gather[row] : (size_t)row;
                xr[it] = *reinterpret_cast<const float4*>(X + s * KD + cx * 4);
            }
        }
#pragma unroll
        for (int it = 0; it < NYR; ++it) {
            const int row = row0 + ry + it * RPPY;
            yr[it] = make_float4(0.f, 0.f, 0.f, 0.f);
            sr[it] = 0.f;
            if (row < row1) {
                const size_t s = (dy_gathered && gather) ? (size_t)gather[row] : (size_t)row;
                yr[it] = *reinterpret_cast<const float4*>(dY + s * ND + cy * 4);
                if (rowscale) sr[it] = rowscale[row];
            }
        }
        dsr = (rowscale && tid < TM && row0 + tid < row1) ? rowscale[row0 + tid] : 0.f;
    };
    if (t0 < t1) fetch(t0);
    int cur_seg = -1;
    int slot = t.chunk_slot[blockIdx.x] - 1;
    for (int ti = t0; ti <= t1; ++ti) {
        const int seg = (ti < t1) ? t.tile_seg[ti] : -2;
        if (seg != cur_seg) {
            if (cur_seg >= 0) {  // flush the finished segment's partial sums
                float* ps = part + (size_t)slot * SLOT;
                if (wave < WBLK) {
#pragma unroll
                    for (int b = 0; b < WBW; ++b) {
                        const int blk = wave + 4 * b, kb = blk % KB, nb = blk / KB;
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            ps[(kb * 32 + acc_row(v, kh)) * ND + nb * 32 + m] = accw[b][v];
                            accw[b][v] = 0.f;
                        }
                    }
                }
                __syncthreads();   // earlier readers of red are done
                red[tid] = acca;
                acca = 0.f;
                __syncthreads();
                if (tid < KD) {
                    float s = 0.f;
#pragma unroll
                    for (int g2 = 0; g2 < AG; ++g2) s += red[g2 * KD + tid];
                    ps[KD * ND + tid] = s;
                }
            }
            if (ti == t1) break;
            ++slot;
            // every wave is past the previous tile's second barrier, so Ws is free
            const float* Wg = W + (size_t)seg * KD * ND;
            for (int i = tid; i < KD * ND; i += 256) Ws[(i / ND) * WS + (i % ND)] = Wg[i];
            cur_seg = seg;
        }
        const int row0 = t.tile_row0[ti], row1 = t.tile_row1[ti];
        {
            float4 wv = make_float4(0.f, 0.f, 0.f, 0.f);
            if (vec && rowscale) wv = *reinterpret_cast<const float4*>(vec + (size_t)seg * ND + cy * 4);
#pragma unroll
            for (int it = 0; it < NXR; ++it)
                *reinterpret_cast<float4*>(Xs + (rx + it * RPPX) * XS + cx * 4) = xr[it];
#pragma unroll
            for (int it = 0; it < NYR; ++it) {
                float4 v = yr[it];
                v.x += sr[it] * wv.x; v.y += sr[it] * wv.y; v.z += sr[it] * wv.z; v.w += sr[it] * wv.w;
                *reinterpret_cast<float4*>(dYs + (ry + it * RPPY) * YS + cy * 4) = v;
            }
            if (tid < TM) dss[tid] = dsr;
        }
        __syncthreads();
        if (ti + 1 < t1) fetch(ti + 1);
        v16f accx[DBW];
#pragma unroll
        for (int b = 0; b < DBW; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) accx[b][v] = 0.f;
        if (wave < DBLK) {
#pragma unroll 2
            for (int tt = 0; tt < ND / 8; ++tt) {
                const int n0 = kh * (ND / 2) + 4 * tt;
                const float4 a4 = *reinterpret_cast<const float4*>(dYs + (rb * 32 + m) * YS + n0);
                const float av[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int b = 0; b < DBW; ++b) {
                        const int cb = (wave >> 1) + 2 * b;
                        accx[b] = mfma32(av[i], Ws[(cb * 32 + m) * WS + n0 + i], accx[b]);
                    }
            }
#pragma unroll
            for (int b = 0; b < DBW; ++b) {
                const int cb = (wave >> 1) + 2 * b;
#pragma unroll
                for (int v = 0; v < 16; ++v) DXs[(rb * 32 + acc_row(v, kh)) * XS + cb * 32 + m] = accx[b][v];
            }
        }
        if (wave < WBLK) {
#pragma unroll 4
            for (int s = 0; s < TM / 2; ++s) {
                const int r = 2 * s + kh;
#pragma unroll
                for (int b = 0; b < WBW; ++b) {
                    const int blk = wave + 4 * b, kb = blk % KB, nb = blk / KB;
                    accw[b] = mfma32(Xs[r * XS + kb * 32 + m], dYs[r * YS + nb * 32 + m], accw[b]);
                }
            }
        }
        if (rowscale) {
            const int k = tid % KD;
            for (int r = tid / KD; r < TM; r += AG) acca += dss[r] * Xs[r * XS + k];
        }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < NXR; ++it) {
            const int r = rx + it * RPPX, row = row0 + r;
            if (row < row1) {
                const size_t d = (scatter_dx && gather) ? (size_t)gather[row] : (size_t)row;
                *reinterpret_cast<float4*>(dXrow + d * KD + cx * 4) =
                    *reinterpret_cast<const float4*>(DXs + r * XS + cx * 4);
            }
        }
    }
}

// dW[s] (and Avec[s]) = sum of the partial slots of segment s, in slot order.
__global__ void slot_reduce_kernel(const float* __restrict__ part, const int32_t* __restrict__ seg_slot_ptr,
                                   int kn, int kd, float* __restrict__ dW, float* __restrict__ Avec) {
    const int seg = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int slot_sz = kn + kd;
    if (i >= slot_sz) return;
    float s = 0.f;
    for (int sl = seg_slot_ptr[seg]; sl < seg_slot_ptr[seg + 1]; ++sl) s += part[(size_t)sl * slot_sz + i];
    if (i < kn) dW[(size_t)seg * kn + i] = s;
    else if (Avec) Avec[(size_t)seg * kd + (i - kn)] = s;
}

// ---------------------------------------------------------------------------------------
static TileArgs tile_args(const TileList& t) {
    return TileArgs{t.tile_seg, t.tile_row0, t.tile_row1, t.chunk_tile, t.chunk_slot};
}

template <int KD, int ND>
static rgnn_status_t launch_fwd(const TypedLinearArgs& a, hipStream_t st) {
    const size_t lds = sizeof(float) * (KD * ND + TM * (KD + 4) + TM * (ND + 4));
    auto kern = typed_linear_fwd_kernel<KD, ND>;
    RGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    KernelTimer kt(st, a.label ? a.label : "typed_linear_fwd");
    hipLaunchKernelGGL(kern, dim3(a.tiles->num_chunks), dim3(256), lds, st, tile_args(*a.tiles), a.X, a.gather, a.W,
                       a.Y, a.scatter_out, a.accumulate, a.vec, a.s_out);
    RGNN_HIP(hipGetLastError());
    return RGNN_OK;
}

rgnn_status_t typed_linear_fwd(int d_in, int d_out, const TypedLinearArgs& a, hipStream_t st) {
    if (a.tiles->num_tiles == 0) return RGNN_OK;
    if (d_in == 64 && d_out == 64) return launch_fwd<64, 64>(a, st);
    if (d_in == 32 && d_out == 32) return launch_fwd<32, 32>(a, st);
    if (d_in == 128 && d_out == 128) return launch_fwd<128, 128>(a, st);
    RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear: d_in = %d, d_out = %d not supported (need equal, 32/64/128)", d_in, d_out);
}

size_t typed_linear_bwd_scratch_floats(int d_in, int d_out, const TileList& t) {
    return (size_t)std::max(t.num_slots, 1) * ((size_t)d_in * d_out + d_in);
}

template <int KD, int ND>
static rgnn_status_t launch_bwd(const TypedLinearBwdArgs& a, hipStream_t st) {
    constexpr int STG = (KD > ND ? KD : ND) + 4;
    constexpr bool PIPE = (KD <= 64 && ND <= 64);
    const size_t lds = PIPE ? sizeof(float) * (KD * (ND + 1) + TM * (ND + 4) + 2 * TM * (KD + 4) + TM + 256)
                            : sizeof(float) * (KD * (ND + 1) + TM * STG + TM * (KD + 4) + TM + 256);
    auto kern = PIPE ? typed_linear_bwd_pipe_kernel<KD, ND> : typed_linear_bwd_kernel<KD, ND>;
    if (a.tiles->num_tiles > 0) {
        RGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        KernelTimer kt(st, a.label ? a.label : "typed_linear_bwd");
        hipLaunchKernelGGL(kern, dim3(a.tiles->num_chunks), dim3(256), lds, st, tile_args(*a.tiles), a.X, a.gather, a.W,
                           a.dY, a.dy_gathered, a.dXrow, a.scatter_dx, a.rowscale, a.vec, a.part);
        RGNN_HIP(hipGetLastError());
    }
    const int kn = KD * ND;
    KernelTimer kt(st, "typed_linear_bwd.reduce");
    hipLaunchKernelGGL(slot_reduce_kernel, dim3((kn + KD + 255) / 256, a.tiles->num_segs), dim3(256), 0, st, a.part,
                       a.tiles->seg_slot_ptr, kn, KD, a.dW, a.Avec);
    RGNN_HIP(hipGetLastError());
    return RGNN_OK;
}

rgnn_status_t typed_linear_bwd(int d_in, int d_out, const TypedLinearBwdArgs& a, hipStream_t st) {
    if (d_in == 64 && d_out == 64) return launch_bwd<64, 64>(a, st);
    if (d_in == 32 && d_out == 32) return launch_bwd<32, 32>(a, st);
    if (d_in == 128 && d_out == 128) return launch_bwd<128, 128>(a, st);
    RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear backward: d_in = %d, d_out = %d not supported (need equal, 32/64/128)", d_in, d_out);
}

}  // namespace rgnn
