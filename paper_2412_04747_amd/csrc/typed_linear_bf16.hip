// Typed linear layer on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation,
// for the bfloat16-input workloads:   Y[i] = A[g(i)] W[seg(i)]   or   Y[i] = A[g(i)] W[seg(i)]^T.
//
// Operands that are bf16 at the boundary (X, the given weights) go to the MFMA as they are,
// so their products are exact.  Operands that only exist in fp32 (intermediate rows such as
// K, V, Z and incoming gradients; the block-diagonal attention weights with mu/sqrt(dh)
// folded in) are split on the fly into two bf16 planes, x = hi + lo, and multiplied with two
// MFMAs, which keeps about 16 mantissa bits: the results stay within ~1e-5 of the fp32 path
// while the contraction runs at bf16 rate.  At these widths the kernel is bound by HBM
// traffic, not by the matrix cores, so the extra MFMAs are free.
//
// Same wave-independent structure as the fp32 kernels: a workgroup keeps the segment's weight
// in LDS (as W_l[out column][contraction index], so a lane reads its B operand, eight
// consecutive contraction indices of one output column, as one 16-byte vector); each
// wavefront owns 32-row units, keeps the next unit's rows in flight in registers, and writes
// its accumulators straight to HBM (two full 128-byte lines per store instruction).
#include "rgnn_internal.h"

namespace rgnn {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ int acc_row16(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

__device__ __forceinline__ void wave_lds_fence_b() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// fp32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ unsigned bf16_rne(float x) {
    unsigned u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
// x = hi + lo (+ ~2^-17 |x|): both as bf16 bits
__device__ __forceinline__ void bf16_split(float x, unsigned& hi, unsigned& lo) {
    hi = bf16_rne(x);
    lo = bf16_rne(x - __uint_as_float(hi << 16));
}

struct TileArgsB {
    const int32_t* tile_seg;
    const int32_t* tile_row0;
    const int32_t* tile_row1;
    const int32_t* chunk_tile;
};

__device__ __forceinline__ int run_end_b(const int32_t* __restrict__ tile_seg, int ti, int t1) {
    const int seg = tile_seg[ti];
    int e = ti + 1;
    while (e < t1 && tile_seg[e] == seg) ++e;
    return e;
}

//   CD     contraction width, OD output width (both multiples of 32, CD a multiple of 16)
//   A_BF16 A rows are bf16 (exact) / fp32 (split)       W_BF16 weights are bf16 (exact) / fp32 (split)
//   WT     false: Y = A W  (W stored [CD][OD])          true: Y = A W^T  (W stored [OD][CD])
//   GATHER rows are read through the gather list        SCATTER outputs are written through it as well
template <int CD, int OD, bool A_BF16, bool W_BF16, bool WT, bool GATHER, bool SCATTER>
__global__ __launch_bounds__(256) void typed_linear_bf16_kernel(TileArgsB t, const void* __restrict__ Av,
                                                                const int32_t* __restrict__ gather,
                                                                const void* __restrict__ Wv, float* __restrict__ Y) {
    constexpr int NW = 4;
    constexpr int LS = CD + 8;                                // LDS row stride in bf16 elements (16-byte aligned rows)
    constexpr int OB = OD / 32;
    constexpr int APL = A_BF16 ? 1 : 2, WPL = W_BF16 ? 1 : 2; // planes (hi [, lo])
    constexpr int LPR = A_BF16 ? CD / 8 : CD / 4;             // lanes per A row (16-byte loads)
    constexpr int RPI = 64 / LPR, NX = 32 / RPI;
    extern __shared__ __align__(16) unsigned short lds[];
    unsigned short* Wl = lds;                                 // [WPL][OD][LS]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    unsigned short* Aw = lds + WPL * OD * LS + wave * (APL * 32 * LS + 64);   // [APL][32][LS] + 32 ints
    int* gidx = reinterpret_cast<int*>(Aw + APL * 32 * LS);
    const int m = lane & 31, kh = lane >> 5;
    const int ci = lane % LPR, ri = lane / LPR;
    const int t0 = t.chunk_tile[blockIdx.x], t1 = t.chunk_tile[blockIdx.x + 1];
    for (int ta = t0; ta < t1;) {
        const int tb = run_end_b(t.tile_seg, ta, t1);
        const int seg = t.tile_seg[ta];
        const int ra = t.tile_row0[ta], rbnd = t.tile_row1[tb - 1];
        const int nu = (rbnd - ra + 31) / 32;
        __syncthreads();                                      // every wavefront is done with the previous weight
        // weight of this segment into LDS as Wl[out column][contraction index]
        for (int i = tid; i < CD * OD; i += 64 * NW) {
            // source element i of the row-major weight: (a, b) = (i / inner, i % inner)
            const int a = WT ? i / CD : i / OD, b = WT ? i % CD : i % OD;
            const int o = WT ? a : b, c = WT ? b : a;         // output column, contraction index
            if (W_BF16) {
                Wl[o * LS + c] = static_cast<const unsigned short*>(Wv)[(size_t)seg * CD * OD + i];
            } else {
                unsigned hi, lo;
                bf16_split(static_cast<const float*>(Wv)[(size_t)seg * CD * OD + i], hi, lo);
                Wl[o * LS + c] = (unsigned short)hi;
                Wl[OD * LS + o * LS + c] = (unsigned short)lo;
            }
        }
        __syncthreads();
        v4u xr[NX];                                           // 16 bytes per load: 8 bf16 or 4 floats
        int gi[NX], gcur[NX];
#define RGNN_FETCH_IDX(U)                                                       \
    _Pragma("unroll") for (int it = 0; it < NX; ++it) {                         \
        const int row_ = min(ra + (U) * 32 + ri + it * RPI, rbnd - 1);          \
        gi[it] = GATHER ? gather[row_] : row_;                                  \
    }
#define RGNN_FETCH_ROWS()                                                       \
    _Pragma("unroll") for (int it = 0; it < NX; ++it) {                         \
        const char* p_ = static_cast<const char*>(Av) + (size_t)gi[it] * CD * (A_BF16 ? 2 : 4) + ci * 16; \
        xr[it] = *reinterpret_cast<const v4u*>(p_);                             \
        gcur[it] = gi[it];                                                      \
    }
        RGNN_FETCH_IDX(wave)
        RGNN_FETCH_ROWS()
        RGNN_FETCH_IDX(wave + NW)
        for (int u = wave; u < nu; u += NW) {
#pragma unroll
            for (int it = 0; it < NX; ++it) {
                const int r = ri + it * RPI;
                if (A_BF16) {
                    *reinterpret_cast<v4u*>(Aw + r * LS + ci * 8) = xr[it];
                } else {
                    unsigned h[4], l[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) bf16_split(__uint_as_float(xr[it][e]), h[e], l[e]);
                    uint2 hv = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
                    uint2 lv = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
                    *reinterpret_cast<uint2*>(Aw + r * LS + ci * 4) = hv;
                    *reinterpret_cast<uint2*>(Aw + 32 * LS + r * LS + ci * 4) = lv;
                }
                if (SCATTER && ci == 0) gidx[r] = gcur[it];
            }
            wave_lds_fence_b();
            RGNN_FETCH_ROWS()             // unit u + NW
            RGNN_FETCH_IDX(u + 2 * NW)
            v16f acc[OB];
#pragma unroll
            for (int b = 0; b < OB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
#pragma unroll 2
            for (int s = 0; s < CD / 16; ++s) {
                const int c0 = 16 * s + 8 * kh;
                const bf16x8 ah = *reinterpret_cast<const bf16x8*>(Aw + m * LS + c0);
                bf16x8 al;
                if (!A_BF16) al = *reinterpret_cast<const bf16x8*>(Aw + 32 * LS + m * LS + c0);
#pragma unroll
                for (int b = 0; b < OB; ++b) {
                    const bf16x8 bh = *reinterpret_cast<const bf16x8*>(Wl + (b * 32 + m) * LS + c0);
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc[b], 0, 0, 0);
                    if (!A_BF16) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc[b], 0, 0, 0);
                    if (!W_BF16) {
                        const bf16x8 bl = *reinterpret_cast<const bf16x8*>(Wl + OD * LS + (b * 32 + m) * LS + c0);
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc[b], 0, 0, 0);
                    }
                }
            }
            // accumulators straight to HBM: lanes 0..31 and 32..63 each write one 128-byte line
            const int rows_left = rbnd - (ra + u * 32);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = acc_row16(v, kh);
                if (r < rows_left) {
                    const size_t d = SCATTER ? (size_t)gidx[r] : (size_t)(ra + u * 32 + r);
#pragma unroll
                    for (int b = 0; b < OB; ++b) Y[d * OD + b * 32 + m] = acc[b][v];
                }
            }
            wave_lds_fence_b();           // operand reads (and gidx reads) are done before the next unit's rows land
        }
#undef RGNN_FETCH_IDX
#undef RGNN_FETCH_ROWS
        ta = tb;
    }
}

// ---------------------------------------------------------------------------------------
// Weight gradient on the bf16 matrix cores:  dW[seg] = sum_{i in seg} X[g(i)]^T dY[i],  D x D.
// The contraction runs over rows, so the MFMA operands are "eight consecutive rows of one
// feature": the 64-row tile is stored feature-major in LDS (T[f][row]), transposed while it is
// written.  Feature row f keeps its eight 16-byte row groups at positions g ^ ((f ^ (f >> 3)) & 7):
// the 16-byte operand reads of 8 neighbouring features then fall on 8 different bank groups, and
// the 2-byte transposing writes of the 16 (or 32) lanes sharing a row spread over 8 banks as well.
// X is used as is when its bf16 original exists, otherwise it and dY are split into hi + lo planes.
// Each of the four wavefronts owns one 32-feature band of X and all four 32-column blocks of dY
// (64 accumulator registers), kept across the tiles of a segment and flushed to the chunk's slot.
__device__ __forceinline__ int tswz(int f, int row) {
    return f * 64 + ((((row >> 3) ^ (f ^ (f >> 3))) & 7) << 3) + (row & 7);
}

template <int D, bool X_BF16, bool GATHER, bool DYG>
__global__ __launch_bounds__(256) void typed_linear_wgrad_bf16_kernel(TileArgsB t, const int32_t* __restrict__ chunk_slot,
                                                                      const void* __restrict__ Xv,
                                                                      const int32_t* __restrict__ gather,
                                                                      const float* __restrict__ dY,
                                                                      float* __restrict__ part) {
    static_assert(D == 128, "four wavefronts x four 32-column blocks");
    constexpr int TMW = 64;
    constexpr int XPL = X_BF16 ? 1 : 2;
    constexpr int LPX = X_BF16 ? D / 8 : D / 4, RPX = 256 / LPX, NXL = TMW / RPX;   // X: lanes/row, rows/pass, passes
    constexpr int LPY = D / 4, RPY = 256 / LPY, NYL = TMW / RPY;
    constexpr int SLOT = D * D + D;
    extern __shared__ __align__(16) unsigned short lds[];
    unsigned short* Xt = lds;                         // [XPL][D][64]
    unsigned short* Yt = lds + XPL * D * 64;          // [2][D][64]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 31, kh = lane >> 5;
    const int cx = tid % LPX, rx = tid / LPX, cy = tid % LPY, ry = tid / LPY;
    v16f acc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
    const int t0 = t.chunk_tile[blockIdx.x], t1 = t.chunk_tile[blockIdx.x + 1];
    v4u xr[NXL], yr[NYL];
    int gi[NXL];
#define RGNN_W_FETCH_IDX(TI)                                                        \
    {                                                                               \
        const int row0_ = t.tile_row0[TI], row1_ = t.tile_row1[TI];                 \
        _Pragma("unroll") for (int it = 0; it < NXL; ++it) {                        \
            const int row_ = min(row0_ + rx + it * RPX, row1_ - 1);                 \
            gi[it] = GATHER ? gather[row_] : row_;                                  \
        }                                                                           \
    }
#define RGNN_W_FETCH(TI)                                                            \
    {                                                                               \
        const int row0_ = t.tile_row0[TI], row1_ = t.tile_row1[TI];                 \
        _Pragma("unroll") for (int it = 0; it < NXL; ++it)                          \
            xr[it] = *reinterpret_cast<const v4u*>(static_cast<const char*>(Xv) +   \
                                                   (size_t)gi[it] * D * (X_BF16 ? 2 : 4) + cx * 16); \
        _Pragma("unroll") for (int it = 0; it < NYL; ++it) {                        \
            const int row_ = min(row0_ + ry + it * RPY, row1_ - 1);                 \
            const size_t s_ = (DYG && GATHER) ? (size_t)gather[row_] : (size_t)row_; \
            yr[it] = *reinterpret_cast<const v4u*>(dY + s_ * D + cy * 4);           \
        }                                                                           \
    }
    if (t0 < t1) {
        RGNN_W_FETCH_IDX(t0)
        RGNN_W_FETCH(t0)
    }
    if (t0 + 1 < t1) RGNN_W_FETCH_IDX(t0 + 1)
    int cur_seg = -1;
    int slot = chunk_slot[blockIdx.x] - 1;
    for (int ti = t0; ti <= t1; ++ti) {
        const int seg = (ti < t1) ? t.tile_seg[ti] : -2;
        if (seg != cur_seg) {
            if (cur_seg >= 0) {   // flush: band `wave` of the gradient, four column blocks
                float* ps = part + (size_t)slot * SLOT;
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        ps[(wave * 32 + acc_row16(v, kh)) * D + b * 32 + m] = acc[b][v];
                        acc[b][v] = 0.f;
                    }
            }
            if (ti == t1) break;
            ++slot;
            cur_seg = seg;
        }
        const int rows = t.tile_row1[ti] - t.tile_row0[ti];
        // transpose the prefetched rows into LDS (rows past the end of the tile as zeros)
#pragma unroll
        for (int it = 0; it < NXL; ++it) {
            const int r = rx + it * RPX;
            const bool ok = r < rows;
            if (X_BF16) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const unsigned w = xr[it][e >> 1];
                    const unsigned short v = ok ? (unsigned short)((e & 1) ? (w >> 16) : (w & 0xFFFFu)) : (unsigned short)0;
                    Xt[tswz(cx * 8 + e, r)] = v;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    unsigned h, l;
                    bf16_split(ok ? __uint_as_float(xr[it][e]) : 0.f, h, l);
                    Xt[tswz(cx * 4 + e, r)] = (unsigned short)h;
                    Xt[D * 64 + tswz(cx * 4 + e, r)] = (unsigned short)l;
                }
            }
        }
#pragma unroll
        for (int it = 0; it < NYL; ++it) {
            const int r = ry + it * RPY;
            const bool ok = r < rows;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                unsigned h, l;
                bf16_split(ok ? __uint_as_float(yr[it][e]) : 0.f, h, l);
                Yt[tswz(cy * 4 + e, r)] = (unsigned short)h;
                Yt[D * 64 + tswz(cy * 4 + e, r)] = (unsigned short)l;
            }
        }
        __syncthreads();
        if (ti + 1 < t1) RGNN_W_FETCH(ti + 1)
        if (ti + 2 < t1) RGNN_W_FETCH_IDX(ti + 2)
#pragma unroll
        for (int s = 0; s < TMW / 16; ++s) {
            const int r0 = 16 * s + 8 * kh;
            const int fa = wave * 32 + m;
            const bf16x8 ah = *reinterpret_cast<const bf16x8*>(Xt + tswz(fa, r0));
            bf16x8 al;
            if (!X_BF16) al = *reinterpret_cast<const bf16x8*>(Xt + D * 64 + tswz(fa, r0));
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int fb = b * 32 + m;
                const bf16x8 bh = *reinterpret_cast<const bf16x8*>(Yt + tswz(fb, r0));
                const bf16x8 bl = *reinterpret_cast<const bf16x8*>(Yt + D * 64 + tswz(fb, r0));
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc[b], 0, 0, 0);
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc[b], 0, 0, 0);
                if (!X_BF16) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc[b], 0, 0, 0);
            }
        }
        __syncthreads();   // operand reads are done before the next tile is transposed in
    }
#undef RGNN_W_FETCH_IDX
#undef RGNN_W_FETCH
}

template <bool X_BF16, bool GATHER, bool DYG>
static rgnn_status_t launch_wgrad(const TypedLinearWgradBf16Args& a, hipStream_t st) {
    constexpr int D = 128;
    const size_t lds = sizeof(unsigned short) * ((X_BF16 ? 1 : 2) + 2) * D * 64;
    auto kern = typed_linear_wgrad_bf16_kernel<D, X_BF16, GATHER, DYG>;
    RGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    KernelTimer kt(st, a.label ? a.label : "typed_linear_wgrad");
    TileArgsB t{a.tiles->tile_seg, a.tiles->tile_row0, a.tiles->tile_row1, a.tiles->chunk_tile};
    hipLaunchKernelGGL(kern, dim3(a.tiles->num_chunks), dim3(256), lds, st, t, a.tiles->chunk_slot, a.X, a.gather, a.dY,
                       a.part);
    RGNN_HIP(hipGetLastError());
    return RGNN_OK;
}

// Fills the partial slots only; the caller sums them with the slot reduction of typed_linear.hip.
rgnn_status_t typed_linear_wgrad_bf16(int d, const TypedLinearWgradBf16Args& a, hipStream_t st) {
    if (d != 128) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed_linear_wgrad_bf16: width %d not supported (128)", d);
    if (a.tiles->num_tiles == 0) return RGNN_OK;
    const bool g = a.gather != nullptr, dg = g && a.dy_gathered;
    if (a.x_bf16) {
        if (g && dg) return launch_wgrad<true, true, true>(a, st);
        if (g) return launch_wgrad<true, true, false>(a, st);
        return launch_wgrad<true, false, false>(a, st);
    }
    if (g && dg) return launch_wgrad<false, true, true>(a, st);
    if (g) return launch_wgrad<false, true, false>(a, st);
    return launch_wgrad<false, false, false>(a, st);
}

template <int CD, int OD, bool A_BF16, bool W_BF16, bool WT, bool GATHER, bool SCATTER>
static rgnn_status_t launch(const TypedLinearBf16Args& a, hipStream_t st) {
    constexpr int LS = CD + 8, APL = A_BF16 ? 1 : 2, WPL = W_BF16 ? 1 : 2;
    const size_t lds = sizeof(unsigned short) * ((size_t)WPL * OD * LS + 4 * (APL * 32 * LS + 64));
    auto kern = typed_linear_bf16_kernel<CD, OD, A_BF16, W_BF16, WT, GATHER, SCATTER>;
    RGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    KernelTimer kt(st, a.label ? a.label : "typed_linear_bf16");
    TileArgsB t{a.tiles->tile_seg, a.tiles->tile_row0, a.tiles->tile_row1, a.tiles->chunk_tile};
    hipLaunchKernelGGL(kern, dim3(a.tiles->num_chunks), dim3(256), lds, st, t, a.A, a.gather, a.W, a.Y);
    RGNN_HIP(hipGetLastError());
    return RGNN_OK;
}

template <int D, bool A_BF16, bool W_BF16, bool WT>
static rgnn_status_t launch_gs(const TypedLinearBf16Args& a, hipStream_t st) {
    const bool g = a.gather != nullptr, sc = g && a.scatter_out;
    if (g && sc) return launch<D, D, A_BF16, W_BF16, WT, true, true>(a, st);
    if (g) return launch<D, D, A_BF16, W_BF16, WT, true, false>(a, st);
    return launch<D, D, A_BF16, W_BF16, WT, false, false>(a, st);
}

template <int D>
static rgnn_status_t launch_d(const TypedLinearBf16Args& a, hipStream_t st) {
    // the combinations the layers use
    if (a.a_bf16 && a.w_bf16 && !a.transpose_w) return launch_gs<D, true, true, false>(a, st);    // X W
    if (!a.a_bf16 && a.w_bf16 && !a.transpose_w) return launch_gs<D, false, true, false>(a, st);  // Z Wo
    if (!a.a_bf16 && a.w_bf16 && a.transpose_w) return launch_gs<D, false, true, true>(a, st);    // dY W^T
    if (!a.a_bf16 && !a.w_bf16 && !a.transpose_w) return launch_gs<D, false, false, false>(a, st); // K Watt_bd
    if (!a.a_bf16 && !a.w_bf16 && a.transpose_w) return launch_gs<D, false, false, true>(a, st);  // dKa Watt_bd^T
    RGNN_FAIL(RGNN_EUNSUPPORTED, "typed_linear_bf16: operand combination not built");
}

rgnn_status_t typed_linear_bf16(int d, const TypedLinearBf16Args& a, hipStream_t st) {
    if (a.tiles->num_tiles == 0) return RGNN_OK;
    if (d == 128) return launch_d<128>(a, st);
    if (d == 64) return launch_d<64>(a, st);
    if (d == 32) return launch_d<32>(a, st);
    RGNN_FAIL(RGNN_EUNSUPPORTED, "typed_linear_bf16: width %d not supported (32/64/128)", d);
}

}  // namespace rgnn
