// Relation-segmented typed linear layer on the CDNA4 matrix cores, fp32.
//
// Forward   Y[i] = X[gather[i]] W[seg(i)]          (thesis Ch.3: segment MM, Y[S] = X[G] x W[T];
//                                                   rows are presorted by type so one weight serves a segment)
// Backward  dXrow[i] = dY[i] W[seg(i)]^T,  dW[s] = sum_{i in s} X[gather[i]]^T dY[i]
//
// Rows are cut into 64-row tiles that never straddle a segment; a persistent workgroup
// walks a contiguous chunk of tiles and keeps the current segment's weight in LDS,
// reloading it only when the segment changes.  The products run on v_mfma_f32_32x32x2_f32.  The K index of the MFMA is a free permutation, so each lane
// reads its A operand as 16-byte LDS vectors: lane (m, half) owns k = half*K/2 + 0..K/2-1.
#include "rgnn_internal.h"

#include <algorithm>

namespace rgnn {

typedef float v16f __attribute__((ext_vector_type(16)));
// Native 4-float vector for the register prefetch buffers: unlike HIP's float4 struct it is
// copied with plain vector loads and stores, so arrays of it stay in registers.
typedef float v4f __attribute__((ext_vector_type(4)));

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

// ---------------------------------------------------------------------------------------
// Wave-independent kernels (feature widths up to 64).
//
// Within a run of tiles that share a segment, the wavefronts of a workgroup do not
// synchronise with each other: wavefront w owns the 32-row units w, w + NW, ... of the run,
// stages them in its private LDS region and keeps the rows of its next unit in flight in
// registers (the gather indices one unit further ahead).  Workgroup barriers are needed only
// when the segment changes (reload of the shared weight tile, flush of the weight-gradient
// partial sums).  This keeps 8 KB (forward) / 16 KB (backward) of HBM reads in flight per
// wavefront at all times, which is what the random row gather needs.
//
// LDS accesses of one wavefront are executed in issue order, so inside a wavefront a store
// followed by a load of another lane's data needs no barrier; wave_lds_fence() only stops
// the compiler from moving LDS accesses across it and waits for outstanding LDS operations.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// First tile index >= ti whose segment differs from tile ti's (or t1).
__device__ __forceinline__ int run_end(const int32_t* __restrict__ tile_seg, int ti, int t1) {
    const int seg = tile_seg[ti];
    int e = ti + 1;
    while (e < t1 && tile_seg[e] == seg) ++e;
    return e;
}

// Compile-time switches of the wave kernels.  They are template parameters rather than
// run-time flags so that the unit loop holds no conditional global load: with one, the
// compiler has to wait for every outstanding memory operation (the prefetched rows and the
// previous unit's stores) at each use.
//   GATHER   rows are read through the gather list        SCATTER  outputs are written through it as well
//   ACCUM    forward: Y += result                         VEC      forward: s_out = Y_row . vec[seg], per head:
//                                                                  s_out[row][h] over the h-th of s_heads column slices
//   DYG      backward: dY rows are read through the list  RS       backward: rowscale / Avec / xvec in use
//   WT       multiply by W[seg]^T (W stored [ND][KD]): the input-gradient product dY W^T
//   ADDV     Y_row += rowscale[row] * vec[seg]  (the rank-1 part of single-head RGAT's input gradient)
template <int KD, int ND, bool GATHER, bool SCATTER, bool ACCUM, bool VEC, bool WT = false, bool ADDV = false>
__global__ __launch_bounds__(256) void typed_linear_fwd_wave_kernel(TileArgs t, const float* __restrict__ X,
                                                                    const int32_t* __restrict__ gather,
                                                                    const float* __restrict__ W, float* __restrict__ Y,
                                                                    const float* __restrict__ vec,
                                                                    float* __restrict__ s_out,
                                                                    const float* __restrict__ rowscale, int s_heads) {
    constexpr int NW = 4;                                   // wavefronts per workgroup
    constexpr int XS = (KD > ND ? KD : ND) + 4;             // row stride of the per-wave stage
    constexpr int CB = ND / 32;
    constexpr int LPRI = KD / 4, RPI = 64 / LPRI, NX = 32 / RPI;   // input: lanes per row, rows per load, loads per unit
    constexpr int LPRO = ND / 4, RPO = 64 / LPRO, NO = 32 / RPO;
    static_assert(!SCATTER || KD == ND, "scattered output reuses the input rows' lane mapping");
    extern __shared__ __align__(16) float smem[];
    float* Ws = smem;                                       // [KD][ND]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float* Xw = smem + KD * ND + wave * 32 * XS;            // [32][XS] private to this wavefront
    const int m = lane & 31, kh = lane >> 5;
    const int ci = lane % LPRI, ri = lane / LPRI, co = lane % LPRO, ro = lane / LPRO;
    const int t0 = t.chunk_tile[blockIdx.x], t1 = t.chunk_tile[blockIdx.x + 1];
    for (int ta = t0; ta < t1;) {
        const int tb = run_end(t.tile_seg, ta, t1);
        const int seg = t.tile_seg[ta];
        const int ra = t.tile_row0[ta], rbnd = t.tile_row1[tb - 1];   // rows [ra, rbnd) of this segment
        const int nu = (rbnd - ra + 31) / 32;
        __syncthreads();                                    // every wavefront is done with the previous weight
        if (!WT) {
            const float4* Wg = reinterpret_cast<const float4*>(W + (size_t)seg * KD * ND);
            for (int i = tid; i < KD * ND / 4; i += 64 * NW) reinterpret_cast<float4*>(Ws)[i] = Wg[i];
        } else {
            // Ws[k][n] = W[n][k]: neighbouring lanes take neighbouring n, so the LDS writes of a
            // wavefront fall on different banks (the strided global reads hit the cache)
            const float* Wg = W + (size_t)seg * KD * ND;
            for (int i = tid; i < ND * (KD / 4); i += 64 * NW) {
                const int n = i % ND, k4 = i / ND;
                const float4 w4 = *reinterpret_cast<const float4*>(Wg + (size_t)n * KD + k4 * 4);
                Ws[(k4 * 4 + 0) * ND + n] = w4.x;
                Ws[(k4 * 4 + 1) * ND + n] = w4.y;
                Ws[(k4 * 4 + 2) * ND + n] = w4.z;
                Ws[(k4 * 4 + 3) * ND + n] = w4.w;
            }
        }
        __syncthreads();
        float4 wv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (VEC || ADDV) wv = *reinterpret_cast<const float4*>(vec + (size_t)seg * ND + co * 4);
        // lanes per head of an output row (a power of two, like the head count), and its log2
        const int lls = (31 - __clz(LPRO)) - (VEC ? 31 - __clz(s_heads) : 0), lph = 1 << lls;
        // Rows past the end of the run are clamped to its last row, so every load below is
        // unconditional; what they bring in is never stored.
        v4f xr[NX];
        int gi[NX], gcur[NX];
#define RGNN_FETCH_IDX(U)                                                           \
    _Pragma("unroll") for (int it = 0; it < NX; ++it) {                             \
        const int row_ = min(ra + (U) * 32 + ri + it * RPI, rbnd - 1);              \
        gi[it] = GATHER ? gather[row_] : row_;                                      \
    }
#define RGNN_FETCH_ROWS()                                                           \
    _Pragma("unroll") for (int it = 0; it < NX; ++it) {                             \
        xr[it] = *reinterpret_cast<const v4f*>(X + (size_t)gi[it] * KD + ci * 4); \
        gcur[it] = gi[it];                                                          \
    }
        RGNN_FETCH_IDX(wave)
        RGNN_FETCH_ROWS()
        RGNN_FETCH_IDX(wave + NW)
        for (int u = wave; u < nu; u += NW) {
            int gout[NX];
#pragma unroll
            for (int it = 0; it < NX; ++it) {
                *reinterpret_cast<v4f*>(Xw + (ri + it * RPI) * XS + ci * 4) = xr[it];
                gout[it] = gcur[it];
            }
            wave_lds_fence();
            RGNN_FETCH_ROWS()             // unit u + NW
            RGNN_FETCH_IDX(u + 2 * NW)
            v16f acc[CB];
#pragma unroll
            for (int b = 0; b < CB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
#pragma unroll 2
            for (int tt = 0; tt < KD / 8; ++tt) {
                const int k0 = kh * (KD / 2) + 4 * tt;
                const float4 a4 = *reinterpret_cast<const float4*>(Xw + m * XS + k0);
                const float av[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int b = 0; b < CB; ++b) acc[b] = mfma32(av[i], Ws[(k0 + i) * ND + b * 32 + m], acc[b]);
            }
            wave_lds_fence();             // all reads of the input rows are done before the stage is overwritten
#pragma unroll
            for (int b = 0; b < CB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) Xw[acc_row(v, kh) * XS + b * 32 + m] = acc[b][v];
            wave_lds_fence();
#pragma unroll
            for (int it = 0; it < NO; ++it) {
                const int r = ro + it * RPO, row = ra + u * 32 + r;
                const bool ok = row < rbnd;
                float4 y = *reinterpret_cast<const float4*>(Xw + r * XS + co * 4);
                const size_t d = SCATTER ? (size_t)gout[it] : (size_t)min(row, rbnd - 1);
                float4* yp = reinterpret_cast<float4*>(Y + d * ND + co * 4);
                if (ACCUM) {
                    const float4 o = *yp;
                    y.x += o.x; y.y += o.y; y.z += o.z; y.w += o.w;
                }
                if (ADDV) {
                    const float sc = rowscale[min(row, rbnd - 1)];
                    y.x += sc * wv.x; y.y += sc * wv.y; y.z += sc * wv.z; y.w += sc * wv.w;
                }
                if (ok) {   // rows of a large tensor that is read again only after it has left the caches: non-temporal
                    const v4f yv = {y.x, y.y, y.z, y.w};
                    __builtin_nontemporal_store(yv, reinterpret_cast<v4f*>(yp));
                }
                if (VEC) {
                    // the lanes of a head's column slice are added (the slices are aligned groups of lph lanes)
                    float sdot = y.x * wv.x + y.y * wv.y + y.z * wv.z + y.w * wv.w;
#pragma unroll
                    for (int o = LPRO / 2; o > 0; o >>= 1) {
                        const float other = __shfl_xor(sdot, o);
                        if (o < lph) sdot += other;
                    }
                    if (ok && (co & (lph - 1)) == 0) s_out[(size_t)row * s_heads + (co >> lls)] = sdot;
                }
            }
            wave_lds_fence();             // the stage is read out before the next unit's rows overwrite it
        }
#undef RGNN_FETCH_IDX
#undef RGNN_FETCH_ROWS
        ta = tb;
    }
}

// Backward of a segment's rows:
//   dXrow[i]  = dY[i] W^T + rowscale[i] * xvec[seg]   (MFMA, contraction over the output features;
//                                                     the rank-1 term is added when the row is stored)
//   dW[seg]   = sum_i X[g(i)]^T dY[i]                 (MFMA, contraction over the rows)
//   Avec[seg] = sum_i rowscale[i] X[g(i)]             (vector ALU)
// With dY_eff = dY + rowscale (x) v, xvec = W v gives dXrow = dY_eff W^T exactly, and the caller
// completes dW = X^T dY_eff by adding Avec^T (x) v; dY_eff itself is never formed.
//
// Backward, wave-independent: eight wavefronts per workgroup, each owning 32-row units of
// the run.  Per unit a wavefront forms dXrow = dY W^T (+ rowscale (x) xvec) and adds its
// rows' contribution to the full KD x ND weight gradient (KB*NB blocks, kept in registers
// for the whole run) and to Avec.  At the end of a run the eight wavefronts' partial weight
// gradients are summed in wavefront order through LDS and written to the chunk's slot.
//
// SEL (row selector): row i of dY is either dY[ysel[i]] or, when the top bit of ysel[i] is set, row
// ysel[i] & 0x7FFFFFFF of a second tensor times a per-row scale; rowscale[i] and that scale come as one
// (rowscale, scale) pair per row.  (RGAT: the gradient row of a (source,
// relation) pair with a single edge is att_e * dOut[dst_e]; it is read from dOut here instead of
// being written out per pair first.)  A lane keeps the selector and the scale of one row of the unit
// and hands them to the lanes that load or store that row with a cross-lane read.
//
// HS > 0 (row selector with HS heads, instead of RS): the columns form HS equal slices; a selected row is
//   dY_alt[row] * a[h] + b[h] * wvec[seg]   on the columns of slice h,
// with (b[0..HS), a[0..HS)) = hcoef[i] per row i.  (Multi-head RGAT: the complete gradient row of a single-edge
// pair, att_e^h dOut[dst_e] + dz_e^h w_s[r] per head, is formed while the row is staged; rows that are not
// selected come from dY as they are.)  The slot's vector part then holds HS vectors, sum over the rows of
// b[h] * X[g(i)] for h < HS (selected or not: b is the row's rowscale per head).
struct RowSelect { const int32_t* sel; const float* alt; const float2* ds_scale; const float* hcoef; const float* wvec; };
template <int KD, int ND, bool GATHER, bool DYG, bool SCATTER, bool RS, bool SEL = false, int HS = 0>
__global__ __launch_bounds__(512) void typed_linear_bwd_wave_kernel(TileArgs t, const float* __restrict__ X,
                                                                    const int32_t* __restrict__ gather,
                                                                    const float* __restrict__ W,
                                                                    const float* __restrict__ dY,
                                                                    float* __restrict__ dXrow,
                                                                    const float* __restrict__ rowscale,
                                                                    const float* __restrict__ vec,
                                                                    float* __restrict__ part, RowSelect ys) {
    static_assert(!SEL || !DYG, "the row selector replaces the dY gather");
    static_assert(HS == 0 || (SEL && !RS && (HS == 2 || HS == 4)), "per-head row selector: two or four heads, no rowscale");
    constexpr int NW = 8;
    constexpr int XS = KD + 4, YS = (ND > KD ? ND : KD) + 4, WS = ND + 1;
    constexpr int KB = KD / 32, NB = ND / 32, WB = KB * NB;
    constexpr int NA = HS ? HS : 1;                         // vectors in a slot's vector part
    constexpr int SLOT = KD * ND + NA * KD;
    constexpr int LPRX = KD / 4, RPX = 64 / LPRX, NXR = 32 / RPX;
    constexpr int LPRY = ND / 4, RPY = 64 / LPRY, NYR = 32 / RPY;
    constexpr int WREG = 32 * XS + 32 * YS + 32;            // floats of LDS per wavefront
    static_assert(!(DYG || SCATTER) || KD == ND, "gathered dY / scattered dXrow reuse the X rows' lane mapping");
    extern __shared__ __align__(16) float smem[];
    float* Ws = smem;                                       // [KD][WS]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float* Xw = smem + KD * WS + wave * WREG;               // [32][XS]  gathered input rows
    float* Yw = Xw + 32 * XS;                               // [32][YS]  dY rows, then the dXrow stage
    float* dsw = Yw + 32 * YS;                              // [32]      rowscale of the unit's rows
    const int m = lane & 31, kh = lane >> 5;
    const int cx = lane % LPRX, rx = lane / LPRX, cy = lane % LPRY, ry = lane / LPRY;
    const int t0 = t.chunk_tile[blockIdx.x], t1 = t.chunk_tile[blockIdx.x + 1];
    int slot = t.chunk_slot[blockIdx.x];
    for (int ta = t0; ta < t1; ++slot) {
        const int tb = run_end(t.tile_seg, ta, t1);
        const int seg = t.tile_seg[ta];
        const int ra = t.tile_row0[ta], rbnd = t.tile_row1[tb - 1];
        const int nu = (rbnd - ra + 31) / 32;
        __syncthreads();                                    // previous run's flush has read the LDS regions
        {
            const float* Wg = W + (size_t)seg * KD * ND;
            for (int i = tid; i < KD * ND; i += 64 * NW) Ws[(i / ND) * WS + (i % ND)] = Wg[i];
        }
        __syncthreads();
        float4 xv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (RS && vec) xv = *reinterpret_cast<const float4*>(vec + (size_t)seg * KD + cx * 4);
        if (HS) xv = *reinterpret_cast<const float4*>(ys.wvec + (size_t)seg * ND + cy * 4);   // this lane's columns of wvec[seg]
        v16f accw[WB];
#pragma unroll
        for (int b = 0; b < WB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) accw[b][v] = 0.f;
        float pa[KB];                                       // partial of Avec[kb * 32 + m] over the rows of parity kh
        v4f pah[HS ? KB : 1];                               // HS: the same for heads 0..3 (element h)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            pa[kb] = 0.f;
            pah[HS ? kb : 0] = v4f{0.f, 0.f, 0.f, 0.f};
        }
        // Rows past the end of the run are clamped to its last row (loads stay unconditional)
        // and zeroed when they are written to LDS, so they add nothing to the weight gradient.
        v4f xr[NXR], yr[NYR];
        float dsr = 0.f;
        int gi[NXR], gcur[NXR];
        int ysn = 0;          // SEL: selector of row (lane & 31) of the unit whose rows are fetched next
        float alr = 1.f;      // SEL: scale of row (lane & 31) of the unit whose rows are in yr
        // HS: (b[h0], b[h0 + 1], a[h0], a[h0 + 1]) of row (lane & 31) of the unit whose rows are in yr, a = 1 for a row
        // that is not selected (hon false); with four heads the upper half of the wavefront keeps heads 2 and 3 (h0 = 2)
        float hcf[4] = {0.f, 0.f, 1.f, 1.f};
        bool hon = false;
        const int h0 = HS == 4 ? 2 * (lane >> 5) : 0;
        // LANEIDX: the gather index of row (lane & 31) is kept by that lane and handed to the lanes that
        // load the row with a cross-lane read (one register instead of NXR); the variants that reuse the
        // indices for dY or for the scattered store keep them per load.
        constexpr bool LANEIDX = GATHER && !DYG && !SCATTER;
        int gsn = 0;
        auto fetch_idx = [&](int u) {
            if (LANEIDX) {
                gsn = gather[min(ra + u * 32 + (lane & 31), rbnd - 1)];
            } else {
#pragma unroll
                for (int it = 0; it < NXR; ++it) {
                    const int row = min(ra + u * 32 + rx + it * RPX, rbnd - 1);
                    gi[it] = GATHER ? gather[row] : row;
                }
            }
            if (SEL) ysn = ys.sel[min(ra + u * 32 + (lane & 31), rbnd - 1)];
        };
        auto fetch = [&](int u) {
#pragma unroll
            for (int it = 0; it < NXR; ++it) {
                const int gx = LANEIDX ? __shfl(gsn, rx + it * RPX) : gi[it];
                xr[it] = *reinterpret_cast<const v4f*>(X + (size_t)gx * KD + cx * 4);
                gcur[it] = gx;
            }
#pragma unroll
            for (int it = 0; it < NYR; ++it) {
                if (SEL) {
                    const int sl = __shfl(ysn, ry + it * RPY);
                    const float* base = sl < 0 ? ys.alt : dY;
                    yr[it] = *reinterpret_cast<const v4f*>(base + (size_t)(sl & 0x7FFFFFFF) * ND + cy * 4);
                } else {
                    const size_t s2 = DYG ? (size_t)gi[it] : (size_t)min(ra + u * 32 + ry + it * RPY, rbnd - 1);
                    yr[it] = *reinterpret_cast<const v4f*>(dY + s2 * ND + cy * 4);
                }
            }
            if (HS) {
                const float* hp = ys.hcoef + (size_t)min(ra + u * 32 + (lane & 31), rbnd - 1) * 2 * HS + h0;
                const float2 bb = *reinterpret_cast<const float2*>(hp), aa = *reinterpret_cast<const float2*>(hp + HS);
                hon = ysn < 0;
                hcf[0] = bb.x; hcf[1] = bb.y;
                hcf[2] = hon ? aa.x : 1.f; hcf[3] = hon ? aa.y : 1.f;
            } else if (SEL) {
                const float2 pr = ys.ds_scale[min(ra + u * 32 + (lane & 31), rbnd - 1)];
                dsr = pr.x;
                alr = ysn < 0 ? pr.y : 1.f;
            } else if (RS) {
                dsr = rowscale[min(ra + u * 32 + (lane & 31), rbnd - 1)];
            }
        };
        fetch_idx(wave);
        fetch(wave);
        fetch_idx(wave + NW);
        for (int u = wave; u < nu; u += NW) {
            const int rows_left = rbnd - (ra + u * 32);      // rows of this unit that exist (may exceed 32)
            int gout[NXR];
#pragma unroll
            for (int it = 0; it < NXR; ++it) {
                const bool ok = rx + it * RPX < rows_left;
                v4f v = xr[it];
                if (!ok) v = v4f{0.f, 0.f, 0.f, 0.f};
                *reinterpret_cast<v4f*>(Xw + (rx + it * RPX) * XS + cx * 4) = v;
                gout[it] = gcur[it];
            }
#pragma unroll
            for (int it = 0; it < NYR; ++it) {
                const bool ok = ry + it * RPY < rows_left;
                v4f v = yr[it];
                if (HS) {
                    // coefficients of this lane's head from the lane that keeps them for the row
                    const int hd = cy / (LPRY / HS);
                    const int from = ry + it * RPY + (HS == 4 ? 32 * (hd >> 1) : 0);
                    const float b0 = __shfl(hon ? hcf[0] : 0.f, from), b1 = __shfl(hon ? hcf[1] : 0.f, from);
                    const float a0 = __shfl(hcf[2], from), a1 = __shfl(hcf[3], from);
                    const float bq = hd & 1 ? b1 : b0, aq = hd & 1 ? a1 : a0;
                    v = v4f{v[0] * aq + bq * xv.x, v[1] * aq + bq * xv.y, v[2] * aq + bq * xv.z, v[3] * aq + bq * xv.w};
                } else if (SEL) {
                    const float sc = __shfl(alr, ry + it * RPY);
                    v = v4f{v[0] * sc, v[1] * sc, v[2] * sc, v[3] * sc};
                }
                if (!ok) v = v4f{0.f, 0.f, 0.f, 0.f};
                *reinterpret_cast<v4f*>(Yw + (ry + it * RPY) * YS + cy * 4) = v;
            }
            const float dsc = RS && (lane & 31) < rows_left ? dsr : 0.f;   // rowscale of row (lane & 31), zero past the end
            if (RS && lane < 32) dsw[lane] = dsc;
            if (HS) {
                // the row's rowscale per head goes into the four spare floats that end its row of Xw (zero past the end);
                // the weight-gradient section reads them back row by row
                static_assert(XS - KD == 4, "the spare floats of an X row hold the per-head rowscale");
                const bool ok = (lane & 31) < rows_left;
                if (HS == 4 || lane < 32)
                    *reinterpret_cast<float2*>(Xw + (lane & 31) * XS + KD + h0) = make_float2(ok ? hcf[0] : 0.f, ok ? hcf[1] : 0.f);
            }
            wave_lds_fence();
            fetch(u + NW);
            fetch_idx(u + 2 * NW);
            // The wavefront that is in its MFMA section goes first at instruction issue: the other wavefront
            // of the SIMD then fills the gaps with its loads and stores instead of interleaving its own MFMAs.
            __builtin_amdgcn_s_setprio(2);
            // dXrow unit: 32 x KD, contraction over the output features.  The LDS operands of both MFMA
            // sections are read ahead of the MFMAs that use them (a ring of B operands two steps deep here,
            // one step in the weight-gradient section), so a wavefront alone on its SIMD keeps the pipe fed.
            v16f accx[KB];
#pragma unroll
            for (int b = 0; b < KB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) accx[b][v] = 0.f;
            {
                const float* yrow = Yw + m * YS + kh * (ND / 2);
                const float* wcol = Ws + m * WS + kh * (ND / 2);
                float bq[3][KB];
                float4 a4 = *reinterpret_cast<const float4*>(yrow), a4n = a4;
#pragma unroll
                for (int b = 0; b < KB; ++b) {
                    bq[0][b] = wcol[b * 32 * WS];
                    bq[1][b] = wcol[b * 32 * WS + 1];
                }
#pragma unroll
                for (int s2 = 0; s2 < ND / 2; ++s2) {
                    if (s2 + 2 < ND / 2) {
#pragma unroll
                        for (int b = 0; b < KB; ++b) bq[(s2 + 2) % 3][b] = wcol[b * 32 * WS + s2 + 2];
                    }
                    if (s2 % 4 == 0 && s2 + 4 < ND / 2) a4n = *reinterpret_cast<const float4*>(yrow + s2 + 4);
                    __builtin_amdgcn_sched_barrier(0);
                    const float av = s2 % 4 == 0 ? a4.x : s2 % 4 == 1 ? a4.y : s2 % 4 == 2 ? a4.z : a4.w;
#pragma unroll
                    for (int b = 0; b < KB; ++b) accx[b] = mfma32(av, bq[s2 % 3][b], accx[b]);
                    if (s2 % 4 == 3) a4 = a4n;
                }
            }
            // weight gradient: KD x ND, contraction over the unit's 32 rows (two rows per MFMA).  The rows'
            // contribution to Avec rides along: lane (m, kh) holds X[2 s + kh][kb * 32 + m] as its A operand
            // and adds rowscale[2 s + kh] times it to its partial of column kb * 32 + m.  With heads, a 4x4x1 MFMA
            // does that for four heads at once: each group of four lanes forms the outer product of the rowscale of
            // its row for heads 0..3 (lane j of the group brings head j's) with the group's four X values, and lane
            // (m, kh) gets the four heads' partials of its column.
            {
                float av[KB], bv[NB];
                float c1 = 0.f, c1n = 0.f;
                if (HS) c1 = Xw[kh * XS + KD + (lane & (HS - 1))];
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) av[kb] = Xw[kh * XS + kb * 32 + m];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) bv[nb] = Yw[kh * YS + nb * 32 + m];
#pragma unroll
                for (int s2 = 0; s2 < 16; ++s2) {
                    float an[KB], bn[NB];
                    if (s2 + 1 < 16) {
                        const int r = 2 * (s2 + 1) + kh;
#pragma unroll
                        for (int kb = 0; kb < KB; ++kb) an[kb] = Xw[r * XS + kb * 32 + m];
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) bn[nb] = Yw[r * YS + nb * 32 + m];
                        if (HS) c1n = Xw[r * XS + KD + (lane & (HS - 1))];
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    if (RS) {
                        const float w0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, dsc), 2 * s2));
                        const float w1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, dsc), 2 * s2 + 1));
                        const float w = kh ? w1 : w0;
#pragma unroll
                        for (int kb = 0; kb < KB; ++kb) pa[kb] += w * av[kb];
                    }
                    if (HS) {
#pragma unroll
                        for (int kb = 0; kb < KB; ++kb) pah[HS ? kb : 0] = __builtin_amdgcn_mfma_f32_4x4x1f32(c1, av[kb], pah[HS ? kb : 0], 0, 0, 0);
                        c1 = c1n;
                    }
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                        for (int kb = 0; kb < KB; ++kb) accw[nb * KB + kb] = mfma32(av[kb], bv[nb], accw[nb * KB + kb]);

                    if (s2 + 1 < 16) {
#pragma unroll
                        for (int kb = 0; kb < KB; ++kb) av[kb] = an[kb];
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) bv[nb] = bn[nb];
                    }
                }
            }
            __builtin_amdgcn_s_setprio(0);
            wave_lds_fence();             // all reads of Yw are done before it becomes the dXrow stage
#pragma unroll
            for (int b = 0; b < KB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) Yw[acc_row(v, kh) * YS + b * 32 + m] = accx[b][v];
            wave_lds_fence();
#pragma unroll
            for (int it = 0; it < NXR; ++it) {
                const int r = rx + it * RPX;
                float4 o = *reinterpret_cast<const float4*>(Yw + r * YS + cx * 4);
                if (RS) {
                    const float sc = dsw[r];
                    o.x += sc * xv.x; o.y += sc * xv.y; o.z += sc * xv.z; o.w += sc * xv.w;
                }
                const size_t d = SCATTER ? (size_t)gout[it] : (size_t)(ra + u * 32 + r);
                if (r < rows_left) {
                    const v4f ov = {o.x, o.y, o.z, o.w};
                    __builtin_nontemporal_store(ov, reinterpret_cast<v4f*>(dXrow + d * KD + cx * 4));
                }
            }
            wave_lds_fence();
        }
        // flush: every wavefront parks its partial weight gradient in its own LDS region, then
        // all threads add the eight copies in wavefront order.
        __syncthreads();
        {
            float* mine = smem + KD * WS + wave * WREG;      // holds a slot's floats (checked on the host)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        mine[(kb * 32 + acc_row(v, kh)) * ND + nb * 32 + m] = accw[nb * KB + kb][v];
#pragma unroll
            for (int h = 0; h < NA; ++h) {
                float acca = 0.f;                           // Avec[h][k = lane] (lanes < KD): both row parities added
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) {
                    const float mine_p = HS ? pah[HS ? kb : 0][h & 3] : pa[kb];
                    const float both = mine_p + __shfl_xor(mine_p, 32);
                    if (kh == kb) acca = both;
                }
                if (lane < KD) mine[KD * ND + h * KD + lane] = acca;
            }
        }
        __syncthreads();
        {
            float* ps = part + (size_t)slot * SLOT;
            for (int i = tid; i < SLOT; i += 64 * NW) {
                float sum = 0.f;
#pragma unroll
                for (int w2 = 0; w2 < NW; ++w2) sum += smem[KD * WS + w2 * WREG + i];
                ps[i] = sum;
            }
        }
        ta = tb;
    }
}

// dW[s] (and Avec[s]) = sum of the partial slots of segment s, in slot order; kd = floats of a slot's vector part.
__global__ void slot_reduce_kernel(const float* __restrict__ part, const int32_t* __restrict__ seg_slot_ptr,
                                   int kn, int kd, float* __restrict__ dW, float* __restrict__ Avec) {
    const int seg = blockIdx.x;                 // segments on the x dimension: their count has no 65535 limit there
    const int i = blockIdx.y * blockDim.x + threadIdx.x;
    const int slot_sz = kn + kd;
    if (i >= slot_sz) return;
    // four partial sums keep four loads in flight; they are combined in a fixed order
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    const int b = seg_slot_ptr[seg], e = seg_slot_ptr[seg + 1];
    int sl = b;
    for (; sl + 3 < e; sl += 4) {
        s0 += part[(size_t)sl * slot_sz + i];
        s1 += part[(size_t)(sl + 1) * slot_sz + i];
        s2 += part[(size_t)(sl + 2) * slot_sz + i];
        s3 += part[(size_t)(sl + 3) * slot_sz + i];
    }
    for (; sl < e; ++sl) s0 += part[(size_t)sl * slot_sz + i];
    const float s = (s0 + s1) + (s2 + s3);
    if (i < kn) dW[(size_t)seg * kn + i] = s;
    else if (Avec) Avec[(size_t)seg * kd + (i - kn)] = s;
}

// ---------------------------------------------------------------------------------------
// Weight gradient alone, fp32, for width 128, where the fused backward kernel above no longer fits
// (a wavefront cannot hold a 128 x 128 gradient):  part[slot] = sum over the chunk's rows of
// X[g(i)]^T dY[i].  Four wavefronts; each owns a 32-feature band of X and all four 32-column blocks
// of dY (64 accumulator registers), kept across the tiles of a segment.  The 64-row tile of X and of
// dY sits row-major in LDS: the MFMA contracts over rows two at a time, so a lane's A operand is
// X[row 2s + kh][band + m] and its B operand dY[row 2s + kh][block + m], both conflict-free 4-byte
// reads.  The next tile's rows are in flight in registers while the current one is multiplied.
// RS: the slot's vector part gets sum over the rows of rowscale[i] * X[g(i)] (otherwise zeros).
template <int D, bool GATHER, bool DYG, bool RS>
__global__ __launch_bounds__(256) void typed_linear_wgrad_f32_kernel(TileArgs t, const float* __restrict__ X,
                                                                     const int32_t* __restrict__ gather,
                                                                     const float* __restrict__ dY,
                                                                     const float* __restrict__ rowscale,
                                                                     float* __restrict__ part) {
    static_assert(D == 128, "four wavefronts x four 32-column blocks");
    constexpr int XS = D + 4;                              // LDS row stride
    constexpr int LPR = D / 4, RPP = 256 / LPR, NL = 64 / RPP;   // lanes per row, rows per pass, passes per tile
    constexpr int SLOT = D * D + D;
    extern __shared__ __align__(16) float smem[];
    float* Xt = smem;                                      // [64][XS]
    float* Yt = smem + 64 * XS;                            // [64][XS]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 31, kh = lane >> 5;
    const int cx = tid % LPR, rx = tid / LPR;
    v16f acc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
    const int t0 = t.chunk_tile[blockIdx.x], t1 = t.chunk_tile[blockIdx.x + 1];
    v4f xr[NL], yr[NL];
    int gi[NL];
    float rs[NL];
    v4f avec = {0.f, 0.f, 0.f, 0.f};                      // this thread's share of the vector part (columns 4 cx ..)
#define RGNN_WF_FETCH_IDX(TI)                                                       \
    {                                                                               \
        const int row0_ = t.tile_row0[TI], row1_ = t.tile_row1[TI];                 \
        _Pragma("unroll") for (int it = 0; it < NL; ++it) {                         \
            const int row_ = min(row0_ + rx + it * RPP, row1_ - 1);                 \
            gi[it] = GATHER ? gather[row_] : row_;                                  \
        }                                                                           \
    }
#define RGNN_WF_FETCH(TI)                                                           \
    {                                                                               \
        const int row0_ = t.tile_row0[TI], row1_ = t.tile_row1[TI];                 \
        _Pragma("unroll") for (int it = 0; it < NL; ++it) {                         \
            xr[it] = *reinterpret_cast<const v4f*>(X + (size_t)gi[it] * D + cx * 4); \
            const int row_ = min(row0_ + rx + it * RPP, row1_ - 1);                 \
            const size_t s_ = (DYG && GATHER) ? (size_t)gi[it] : (size_t)row_;      \
            yr[it] = *reinterpret_cast<const v4f*>(dY + s_ * D + cx * 4);           \
            if (RS) rs[it] = rowscale[row_];                                        \
        }                                                                           \
    }
    if (t0 < t1) {
        RGNN_WF_FETCH_IDX(t0)
        RGNN_WF_FETCH(t0)
    }
    if (t0 + 1 < t1) RGNN_WF_FETCH_IDX(t0 + 1)
    int cur_seg = -1;
    int slot = t.chunk_slot[blockIdx.x] - 1;
    for (int ti = t0; ti <= t1; ++ti) {
        const int seg = (ti < t1) ? t.tile_seg[ti] : -2;
        if (seg != cur_seg) {
            if (cur_seg >= 0) {   // flush: band `wave` of the gradient, four column blocks
                float* ps = part + (size_t)slot * SLOT;
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        ps[(wave * 32 + acc_row(v, kh)) * D + b * 32 + m] = acc[b][v];
                        acc[b][v] = 0.f;
                    }
                if (RS) {   // the eight threads sharing a column group add their shares in order, through LDS
                    __syncthreads();
                    *reinterpret_cast<v4f*>(Xt + rx * XS + cx * 4) = avec;
                    avec = v4f{0.f, 0.f, 0.f, 0.f};
                    __syncthreads();
                    if (tid < D) {
                        float sum = 0.f;
#pragma unroll
                        for (int r = 0; r < RPP; ++r) sum += Xt[r * XS + tid];
                        ps[D * D + tid] = sum;
                    }
                    __syncthreads();
                } else if (tid < D) {
                    ps[D * D + tid] = 0.f;
                }
            }
            if (ti == t1) break;
            ++slot;
            cur_seg = seg;
        }
        const int rows = t.tile_row1[ti] - t.tile_row0[ti];
#pragma unroll
        for (int it = 0; it < NL; ++it) {
            const int r = rx + it * RPP;
            const bool ok = r < rows;                      // rows past the end of the tile count as zeros
            const v4f z = {0.f, 0.f, 0.f, 0.f};
            *reinterpret_cast<v4f*>(Xt + r * XS + cx * 4) = ok ? xr[it] : z;
            *reinterpret_cast<v4f*>(Yt + r * XS + cx * 4) = ok ? yr[it] : z;
            if (RS && ok) avec += rs[it] * xr[it];
        }
        __syncthreads();
        if (ti + 1 < t1) RGNN_WF_FETCH(ti + 1)
        if (ti + 2 < t1) RGNN_WF_FETCH_IDX(ti + 2)
#pragma unroll 4
        for (int s = 0; s < 32; ++s) {
            const int r = 2 * s + kh;
            const float a = Xt[r * XS + wave * 32 + m];
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[b] = mfma32(a, Yt[r * XS + b * 32 + m], acc[b]);
        }
        __syncthreads();   // operand reads are done before the next tile is written
    }
#undef RGNN_WF_FETCH_IDX
#undef RGNN_WF_FETCH
}

// ---------------------------------------------------------------------------------------
static TileArgs tile_args(const TileList& t) {
    return TileArgs{t.tile_seg, t.tile_row0, t.tile_row1, t.chunk_tile, t.chunk_slot};
}

template <int KD, int ND, bool GATHER, bool SCATTER, bool ACCUM, bool VEC, bool WT = false, bool ADDV = false>
static rgnn_status_t launch_fwd_wave(const TypedLinearArgs& a, hipStream_t st, const float* rowscale = nullptr) {
    const size_t lds = sizeof(float) * (KD * ND + 4 * 32 * ((KD > ND ? KD : ND) + 4));
    auto kern = typed_linear_fwd_wave_kernel<KD, ND, GATHER, SCATTER, ACCUM, VEC, WT, ADDV>;
    RGNN_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds));
    KernelTimer kt(st, a.label ? a.label : "typed_linear_fwd");
    hipLaunchKernelGGL(kern, dim3(a.tiles->num_chunks), dim3(256), lds, st, tile_args(*a.tiles), a.X, a.gather, a.W, a.Y,
                       a.vec, a.s_out, rowscale, a.s_heads);
    RGNN_HIP(hipGetLastError());
    return RGNN_OK;
}

template <int KD, int ND>
static rgnn_status_t launch_fwd(const TypedLinearArgs& a, hipStream_t st) {
    // the combinations the layers use
    const bool g = a.gather != nullptr, sc = g && a.scatter_out, ac = a.accumulate != 0, v = a.vec != nullptr;
    if (v && (a.s_heads < 1 || (a.s_heads & (a.s_heads - 1)) || a.s_heads > ND / 4))
        RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear: %d heads for the row-vector products at width %d", a.s_heads, ND);
    if (g && !sc && !ac && v) return launch_fwd_wave<KD, ND, true, false, false, true>(a, st);
    if (g && !sc && !ac && !v) return launch_fwd_wave<KD, ND, true, false, false, false>(a, st);
    if constexpr (KD == ND) {
        if (g && sc && !ac && !v) return launch_fwd_wave<KD, ND, true, true, false, false>(a, st);
    }
    if (!g && !ac && !v) return launch_fwd_wave<KD, ND, false, false, false, false>(a, st);
    if (!g && ac && !v) return launch_fwd_wave<KD, ND, false, false, true, false>(a, st);
    RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear forward: this combination of gather / scatter / accumulate / vec is not built");
}

rgnn_status_t typed_linear_fwd(int d_in, int d_out, const TypedLinearArgs& a, hipStream_t st) {
    if (a.tiles->num_tiles == 0) return RGNN_OK;
    if (d_in == 64 && d_out == 64) return launch_fwd<64, 64>(a, st);
    if (d_in == 32 && d_out == 32) return launch_fwd<32, 32>(a, st);
    if (d_in == 128 && d_out == 128) return launch_fwd<128, 128>(a, st);
    if (d_in == 32 && d_out == 64) return launch_fwd<32, 64>(a, st);
    if (d_in == 64 && d_out == 32) return launch_fwd<64, 32>(a, st);
    RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear: d_in = %d, d_out = %d not supported (need 32 / 64 / 128, different widths only among 32 and 64)", d_in, d_out);
}

size_t typed_linear_bwd_scratch_floats(int d_in, int d_out, const TileList& t, int vectors) {
    return (size_t)std::max(t.num_slots, 1) * ((size_t)d_in * d_out + (size_t)std::max(vectors, 1) * d_in);
}

static rgnn_status_t launch_slot_reduce(int kd, int nd, const TypedLinearBwdArgs& a, hipStream_t st, int vectors = 1) {
    const int kn = kd * nd, kv = kd * vectors;
    KernelTimer kt(st, "typed_linear_bwd.reduce");
    hipLaunchKernelGGL(slot_reduce_kernel, dim3(a.tiles->num_segs, (kn + kv + 255) / 256), dim3(256), 0, st, a.part,
                       a.tiles->seg_slot_ptr, kn, kv, a.dW, a.Avec);
    RGNN_HIP(hipGetLastError());
    return RGNN_OK;
}

template <int KD, int ND, bool GATHER, bool DYG, bool SCATTER, bool RS, bool SEL = false, int HS = 0>
static rgnn_status_t launch_bwd_wave(const TypedLinearBwdArgs& a, hipStream_t st) {
    constexpr int WREG = 32 * (KD + 4) + 32 * ((ND > KD ? ND : KD) + 4) + 32;
    static_assert(WREG >= KD * ND + (HS ? HS : 1) * KD, "per-wavefront LDS region must hold a weight-gradient copy");
    const size_t lds = sizeof(float) * (KD * (ND + 1) + 8 * WREG);
    auto kern = typed_linear_bwd_wave_kernel<KD, ND, GATHER, DYG, SCATTER, RS, SEL, HS>;
    RGNN_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds));
    KernelTimer kt(st, a.label ? a.label : "typed_linear_bwd");
    hipLaunchKernelGGL(kern, dim3(a.tiles->num_chunks), dim3(512), lds, st, tile_args(*a.tiles), a.X, a.gather, a.W,
                       a.dY, a.dXrow, a.rowscale, a.vec, a.part, RowSelect{a.ysel, a.dY_alt, a.ds_yscale, a.hcoef, a.wvec});
    RGNN_HIP(hipGetLastError());
    return RGNN_OK;
}

// Width 128: dXrow = dY W^T (+ rowscale (x) vec) with the forward wave kernel on the transposed weight,
// then the weight-gradient kernel; two passes over dY, but both near the matrix cores' rate.
template <int D>
static rgnn_status_t launch_bwd_split(const TypedLinearBwdArgs& a, hipStream_t st) {
    const bool g = a.gather != nullptr, dg = g && a.dy_gathered, sc = g && a.scatter_dx, rs = a.rowscale != nullptr;
    TypedLinearArgs f{};
    f.tiles = a.tiles; f.X = a.dY; f.gather = dg ? a.gather : nullptr; f.W = a.W; f.Y = a.dXrow;
    f.scatter_out = sc; f.vec = a.vec; f.label = a.label ? a.label : "typed_linear_bwd";
    if (dg != sc) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear backward: dY gathered and dXrow scattered must go together");
    if (rs && (dg || !a.vec)) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear backward: rowscale needs vec and ungathered dY");
    if (rs) RGNN_TRY((launch_fwd_wave<D, D, false, false, false, false, true, true>(f, st, a.rowscale)));
    else if (dg) RGNN_TRY((launch_fwd_wave<D, D, true, true, false, false, true>(f, st)));
    else RGNN_TRY((launch_fwd_wave<D, D, false, false, false, false, true>(f, st)));
    const size_t lds = sizeof(float) * 2 * 64 * (D + 4);
    KernelTimer kt(st, wgrad_label(f.label));
#define RGNN_LAUNCH_WGRAD(G_, DG_, RS_)                                                                              \
    {                                                                                                                \
        auto kern = typed_linear_wgrad_f32_kernel<D, G_, DG_, RS_>;                                                  \
        RGNN_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds));                                       \
        hipLaunchKernelGGL(kern, dim3(a.tiles->num_chunks), dim3(256), lds, st, tile_args(*a.tiles), a.X, a.gather, \
                           a.dY, a.rowscale, a.part);                                                                \
    }
    if (g && dg) RGNN_LAUNCH_WGRAD(true, true, false)
    else if (g && rs) RGNN_LAUNCH_WGRAD(true, false, true)
    else if (g) RGNN_LAUNCH_WGRAD(true, false, false)
    else if (!rs) RGNN_LAUNCH_WGRAD(false, false, false)
    else RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear backward: rowscale needs gathered X");
#undef RGNN_LAUNCH_WGRAD
    RGNN_HIP(hipGetLastError());
    return RGNN_OK;
}

template <int KD, int ND>
static rgnn_status_t launch_bwd(const TypedLinearBwdArgs& a, hipStream_t st) {
    if (a.tiles->num_tiles > 0) {
        bool done = false;
        if constexpr (KD == 128 && ND == 128) {
            if (a.ysel) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear backward: no row selector at width 128");
            RGNN_TRY(launch_bwd_split<128>(a, st));
            done = true;
        }
        if constexpr (KD <= 64 && ND <= 64) {
            const bool g = a.gather != nullptr, dg = g && a.dy_gathered, sc = g && a.scatter_dx, rs = a.rowscale != nullptr;
            done = true;
            if (a.ysel && a.hcoef) {
                if (!(g && !dg && !sc && !rs && a.dY_alt && a.wvec) || (a.sel_heads != 2 && a.sel_heads != 4) || ND % (4 * a.sel_heads))
                    RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear backward: the per-head row selector needs gathered X, ungathered dY, no rowscale, 2 or 4 heads of a multiple of 4 columns");
                if (a.sel_heads == 2) RGNN_TRY((launch_bwd_wave<KD, ND, true, false, false, false, true, 2>(a, st)));
                else RGNN_TRY((launch_bwd_wave<KD, ND, true, false, false, false, true, 4>(a, st)));
            } else if (a.ysel && !(g && !dg && !sc && !rs && a.vec && a.dY_alt && a.ds_yscale))
                RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear backward: the row selector needs gathered X, ungathered dY, vec and the (rowscale, scale) pairs");
            else if (a.ysel) RGNN_TRY((launch_bwd_wave<KD, ND, true, false, false, true, true>(a, st)));
            else if (g && !dg && !sc && rs) RGNN_TRY((launch_bwd_wave<KD, ND, true, false, false, true>(a, st)));
            else if (g && !dg && !sc && !rs) RGNN_TRY((launch_bwd_wave<KD, ND, true, false, false, false>(a, st)));
            else if (KD == ND && g && dg && sc && !rs) {
                if constexpr (KD == ND) RGNN_TRY((launch_bwd_wave<KD, ND, true, true, true, false>(a, st)));
            } else if (!g && !rs) RGNN_TRY((launch_bwd_wave<KD, ND, false, false, false, false>(a, st)));
            else done = false;
        }
        if (!done) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear backward: this combination of gather / scatter / rowscale is not built");
    }
    return launch_slot_reduce(KD, ND, a, st, KD <= 64 && a.ysel && a.hcoef ? a.sel_heads : 1);
}

rgnn_status_t typed_linear_slot_reduce(int d_in, int d_out, const TileList& tiles, const float* part, float* dW,
                                       float* Avec, hipStream_t st) {
    const int kn = d_in * d_out;
    KernelTimer kt(st, "typed_linear_bwd.reduce");
    hipLaunchKernelGGL(slot_reduce_kernel, dim3(tiles.num_segs, (kn + d_in + 255) / 256), dim3(256), 0, st, part,
                       tiles.seg_slot_ptr, kn, d_in, dW, Avec);
    RGNN_HIP(hipGetLastError());
    return RGNN_OK;
}

rgnn_status_t typed_linear_bwd(int d_in, int d_out, const TypedLinearBwdArgs& a, hipStream_t st) {
    if (d_in == 64 && d_out == 64) return launch_bwd<64, 64>(a, st);
    if (d_in == 32 && d_out == 32) return launch_bwd<32, 32>(a, st);
    if (d_in == 128 && d_out == 128) return launch_bwd<128, 128>(a, st);
    if (d_in == 32 && d_out == 64) return launch_bwd<32, 64>(a, st);
    if (d_in == 64 && d_out == 32) return launch_bwd<64, 32>(a, st);
    RGNN_FAIL(RGNN_EUNSUPPORTED, "typed linear backward: d_in = %d, d_out = %d not supported (need 32 / 64 / 128, different widths only among 32 and 64)", d_in, d_out);
}

}  // namespace rgnn
