// Typed linear layer on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation,
// for the bfloat16-input workloads:   Y[i] = A[g(i)] W[seg(i)]   or   Y[i] = A[g(i)] W[seg(i)]^T.
//
// Operands stored as bf16 (X, the given weights, and at width 128 every intermediate row
// tensor) go to the MFMA as they are, so their products are exact.  Operands that only exist
// in fp32 (the block-diagonal attention weights with mu/sqrt(dh) folded in; at widths below 128
// the intermediate rows) are split on the fly into two bf16 planes, x = hi + lo, and multiplied
// with two MFMAs, which keeps about 16 mantissa bits.  At these widths the kernel is bound by
// HBM traffic, not by the matrix cores, so the extra MFMAs are free.  The output rows are
// written as fp32 or rounded to bf16 (nearest even).
//
// Same wave-independent structure as the fp32 kernels: a workgroup keeps the segment's weight
// in LDS (as W_l[out column][contraction index], so a lane reads its B operand, eight
// consecutive contraction indices of one output column, as one 16-byte vector); each
// wavefront owns 32-row units, keeps the next unit's rows in flight in registers, and writes
// its accumulators straight to HBM.
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
// two fp32 -> packed bf16 pair (lo in bits 0..15), round to nearest even, one v_cvt_pk_bf16_f32
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned bf16_pack_rne(float lo, float hi) {
    const v2f v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}
// x = hi + lo (+ ~2^-17 |x|): both as bf16 bits
__device__ __forceinline__ void bf16_split(float x, unsigned& hi, unsigned& lo) {
    hi = bf16_rne(x);
    lo = bf16_rne(x - __uint_as_float(hi << 16));
}

// eight bf16 (four packed pairs) times s, rounded to nearest even again
__device__ __forceinline__ v4u bf16x8_scale(v4u x, float s) {
    v4u y;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        y[e] = bf16_pack_rne(__uint_as_float(x[e] << 16) * s, __uint_as_float(x[e] & 0xFFFF0000u) * s);
    return y;
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
//   Y_BF16 output rows are stored as bf16 / fp32        ACC    (fp32 output only) Y += result
// A gather entry with the top bit set reads row (entry & 0x7FFFFFFF) of Alt instead of A (not with SCATTER).
// rowscale (optional, bf16 A only): row i of the tiles is multiplied by rowscale[i] (and rounded to bf16
// again) on its way into LDS; the lane that holds a row's factor hands it to the lanes that store the row.
template <int CD, int OD, bool A_BF16, bool W_BF16, bool WT, bool GATHER, bool SCATTER, bool Y_BF16, bool ACC>
__global__ __launch_bounds__(256) void typed_linear_bf16_kernel(TileArgsB t, const void* __restrict__ Av,
                                                                const int32_t* __restrict__ gather,
                                                                const void* __restrict__ Wv, void* __restrict__ Yv,
                                                                const void* __restrict__ Alt,
                                                                const float* __restrict__ rowscale) {
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
        float scn = 1.f, sc = 1.f;                            // rowscale of row (lane & 31): next unit's, and of the rows in xr
#define RGNN_FETCH_IDX(U)                                                       \
    _Pragma("unroll") for (int it = 0; it < NX; ++it) {                         \
        const int row_ = min(ra + (U) * 32 + ri + it * RPI, rbnd - 1);          \
        gi[it] = GATHER ? gather[row_] : row_;                                  \
    }                                                                           \
    if (A_BF16 && rowscale) scn = rowscale[min(ra + (U) * 32 + (lane & 31), rbnd - 1)];
#define RGNN_FETCH_ROWS()                                                       \
    _Pragma("unroll") for (int it = 0; it < NX; ++it) {                         \
        const char* b_ = static_cast<const char*>(GATHER && !SCATTER && gi[it] < 0 ? Alt : Av); \
        const char* p_ = b_ + (size_t)(GATHER && !SCATTER ? gi[it] & 0x7FFFFFFF : gi[it]) * CD * (A_BF16 ? 2 : 4) + ci * 16; \
        xr[it] = *reinterpret_cast<const v4u*>(p_);                             \
        gcur[it] = gi[it];                                                      \
    }                                                                           \
    sc = scn;
        RGNN_FETCH_IDX(wave)
        RGNN_FETCH_ROWS()
        RGNN_FETCH_IDX(wave + NW)
        for (int u = wave; u < nu; u += NW) {
#pragma unroll
            for (int it = 0; it < NX; ++it) {
                const int r = ri + it * RPI;
                if (A_BF16) {
                    v4u x = xr[it];
                    if (rowscale) x = bf16x8_scale(x, __shfl(sc, r));
                    *reinterpret_cast<v4u*>(Aw + r * LS + ci * 8) = x;
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
            const int rows_left = rbnd - (ra + u * 32);
            if (!Y_BF16) {
                // accumulators straight to HBM: lanes 0..31 and 32..63 each write one 128-byte line
                float* __restrict__ Y = static_cast<float*>(Yv);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = acc_row16(v, kh);
                    if (r < rows_left) {
                        const size_t d = SCATTER ? (size_t)gidx[r] : (size_t)(ra + u * 32 + r);
#pragma unroll
                            for (int b = 0; b < OB; ++b) {
                            if (ACC) Y[d * OD + b * 32 + m] += acc[b][v];
                            else Y[d * OD + b * 32 + m] = acc[b][v];
                        }
                    }
                }
            } else {
                // bf16 rows go through the wavefront's A area of LDS (free once the operand reads are
                // done), so that HBM sees whole rows: registers v and v + 1 hold rows r and r + 1 of
                // column m; neighbouring lanes swap one of the two, an even lane then owns (row r;
                // columns m, m + 1), an odd lane (row r + 1; columns m - 1, m), and each writes one
                // packed pair.  Then 16-byte pieces of whole rows are copied out, OD / 8 lanes per row.
                static_assert(!Y_BF16 || (A_BF16 && OD <= CD), "the output tile is staged in the A area");
                unsigned short* __restrict__ Y = static_cast<unsigned short*>(Yv);
                const bool odd = m & 1;
                wave_lds_fence_b();
#pragma unroll
                for (int v = 0; v < 16; v += 2) {
                    const int r = acc_row16(v, kh) + (odd ? 1 : 0);
#pragma unroll
                    for (int b = 0; b < OB; ++b) {
                        // quad_perm [1, 0, 3, 2]: the neighbouring lane's two values
                        const float a0 = acc[b][v], a1 = acc[b][v + 1];
                        const float n0 = __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(a0), 0xB1, 0xF, 0xF, true));
                        const float n1 = __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(a1), 0xB1, 0xF, 0xF, true));
                        const unsigned w = bf16_pack_rne(odd ? n1 : a0, odd ? a1 : n0);
                        *reinterpret_cast<unsigned*>(Aw + r * LS + b * 32 + (m & ~1)) = w;
                    }
                }
                wave_lds_fence_b();
                constexpr int LPO = OD / 8, RPP = 64 / LPO;       // lanes per output row, rows per pass
                const int oc = lane % LPO, orow = lane / LPO;
#pragma unroll
                for (int pass = 0; pass < 32 / RPP; ++pass) {
                    const int r = orow + pass * RPP;
                    if (r < rows_left) {
                        const size_t d = SCATTER ? (size_t)gidx[r] : (size_t)(ra + u * 32 + r);
                        __builtin_nontemporal_store(*reinterpret_cast<const v4u*>(Aw + r * LS + oc * 8), reinterpret_cast<v4u*>(Y + d * OD + oc * 8));
                    }
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
// Weight gradient on the bf16 matrix cores:  dW[seg] = sum_{i in seg} X[g(i)]^T dY[i],  D x D,
// X and dY rows stored as bf16.
// The contraction runs over rows, so the MFMA operands are "eight consecutive rows of one
// feature": the 64-row tile is stored feature-major in LDS (T[f][row]), transposed while it is
// written.  A lane loads the same eight features of four consecutive rows, packs the four
// values of each feature into one 8-byte word and writes eight such words.  Feature row f keeps
// its eight 16-byte row groups at positions g ^ ((f ^ (f >> 3)) & 7): the 16-byte operand reads
// of 8 neighbouring features then fall on 8 different bank groups, and so do the transposing
// writes of the 16 lanes sharing a row group.  Each of the four wavefronts owns one 32-feature
// band of X and all four 32-column blocks of dY (64 accumulator registers), kept across the tiles
// of a segment and flushed to the chunk's slot.  The kernel is bound by how many row loads are in
// flight, so registers are budgeted for three wavefronts per SIMD and one 32 KB tile buffer is
// used (NBUF = 2 alternates two buffers and saves a barrier per tile, but halves the occupancy).
__device__ __forceinline__ int tswz(int f, int row) {
    return f * 64 + ((((row >> 3) ^ (f ^ (f >> 3))) & 7) << 3) + (row & 7);
}

// rows[k] = eight bf16 of row k (k = 0..3) of features f0 .. f0 + 7 (f0 a multiple of 8); writes
// T[f0 + e][row0 .. row0 + 3] for e = 0..7.  `at` = tswz(f0, row0) and `g8` = 8 * (its row-group
// position): feature f0 + e sits 64 e further with the group position XOR e.
__device__ __forceinline__ void transpose4_to_lds(unsigned short* __restrict__ T, int at, int g8, const v4u (&rows)[4]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const unsigned a0 = rows[0][e >> 1], a1 = rows[1][e >> 1], a2 = rows[2][e >> 1], a3 = rows[3][e >> 1];
        const unsigned w01 = (e & 1) ? ((a0 >> 16) | (a1 & 0xFFFF0000u)) : ((a0 & 0xFFFFu) | (a1 << 16));
        const unsigned w23 = (e & 1) ? ((a2 >> 16) | (a3 & 0xFFFF0000u)) : ((a2 & 0xFFFFu) | (a3 << 16));
        *reinterpret_cast<uint2*>(T + at - g8 + e * 64 + (g8 ^ (e * 8))) = make_uint2(w01, w23);
    }
}

// SEL: row i of dY is dY[ysel[i]], or dYalt[ysel[i] & 0x7FFFFFFF] when the top bit of ysel[i] is set; with
// yscale the row is also multiplied by yscale[i] (rounded to bf16 again) before it enters the tile.
template <int D, bool GATHER, bool DYG, int NBUF, bool SEL = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void typed_linear_wgrad_bf16_kernel(TileArgsB t, const int32_t* __restrict__ chunk_slot,
                                                                      const unsigned short* __restrict__ X,
                                                                      const int32_t* __restrict__ gather,
                                                                      const unsigned short* __restrict__ dY,
                                                                      float* __restrict__ part,
                                                                      const int32_t* __restrict__ ysel,
                                                                      const unsigned short* __restrict__ dYalt,
                                                                      const float* __restrict__ yscale) {
    static_assert(D == 128, "four wavefronts x four 32-column blocks");
    static_assert(!(SEL && DYG), "the row selector replaces the dY gather");
    constexpr int TMW = 64;
    constexpr int LPX = D / 8;                        // lanes per row (16-byte loads)
    constexpr int SLOT = D * D + D;
    constexpr int BUF = 2 * D * 64;                   // one buffer: X tile and dY tile, feature-major
    extern __shared__ __align__(16) unsigned short lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 31, kh = lane >> 5;
    const int cx = tid % LPX, rq = tid / LPX;         // features 8 cx .. 8 cx + 7 of rows 4 rq .. 4 rq + 3
    v16f acc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
    const int t0 = t.chunk_tile[blockIdx.x], t1 = t.chunk_tile[blockIdx.x + 1];
    // writes: tswz(8 cx, 4 rq) = wat + 8 * (group position);  reads: tswz(32 j + m, 16 s + 8 kh) =
    // (32 j + m) * 64 + (8 * ((kh ^ m ^ (m >> 3)) & 7) ^ 32 (j & 1) ^ 16 s)
    const int wat = cx * 512 + 4 * (rq & 1), wg8_0 = (((rq >> 1) ^ cx) & 7) * 8;
    const int rg8_0 = ((kh ^ m ^ (m >> 3)) & 7) * 8;
    v4u xr[4], yr[4];
    int gi[4], gy[SEL ? 4 : 1];
    float ysn = 1.f, ysc = 1.f;   // yscale of row 16 * wave + (lane & 15): next tile's, and of the rows in yr
#define RGNN_W_FETCH_IDX(TI)                                                        \
    {                                                                               \
        const int row0_ = t.tile_row0[TI], row1_ = t.tile_row1[TI];                 \
        _Pragma("unroll") for (int k = 0; k < 4; ++k) {                             \
            const int row_ = min(row0_ + 4 * rq + k, row1_ - 1);                    \
            gi[k] = GATHER ? gather[row_] : row_;                                   \
            if (SEL) gy[SEL ? k : 0] = ysel[row_];                                  \
        }                                                                           \
        if (SEL && yscale) ysn = yscale[min(row0_ + 16 * wave + (lane & 15), row1_ - 1)]; \
    }
#define RGNN_W_FETCH(TI)                                                            \
    {                                                                               \
        const int row0_ = t.tile_row0[TI], row1_ = t.tile_row1[TI];                 \
        _Pragma("unroll") for (int k = 0; k < 4; ++k) {                             \
            xr[k] = *reinterpret_cast<const v4u*>(X + (size_t)gi[k] * D + cx * 8);  \
            const int row_ = min(row0_ + 4 * rq + k, row1_ - 1);                    \
            if (SEL) {                                                              \
                const int y_ = gy[SEL ? k : 0];                                     \
                yr[k] = *reinterpret_cast<const v4u*>((y_ < 0 ? dYalt : dY) + (size_t)(y_ & 0x7FFFFFFF) * D + cx * 8); \
            } else {                                                                \
                const size_t s_ = (DYG && GATHER) ? (size_t)gi[k] : (size_t)row_;   \
                yr[k] = *reinterpret_cast<const v4u*>(dY + s_ * D + cx * 8);        \
            }                                                                       \
        }                                                                           \
        ysc = ysn;                                                                  \
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
        unsigned short* Xt = lds + ((ti - t0) % NBUF) * BUF;   // [D][64]
        unsigned short* Yt = Xt + D * 64;                   // [D][64]
        // rows past the end of the tile count as zeros
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (4 * rq + k >= rows) {
                xr[k] = v4u{0u, 0u, 0u, 0u};
                yr[k] = v4u{0u, 0u, 0u, 0u};
            }
        // The swizzled LDS positions differ from a per-lane base only by XORs with constants; the
        // bases are made opaque once per tile so that the 36 positions are recomputed (one XOR each)
        // rather than kept in registers across the loop.
        int wg8 = wg8_0, rg8 = rg8_0;
        asm volatile("" : "+v"(wg8), "+v"(rg8));
        transpose4_to_lds(Xt, wat + wg8, wg8, xr);
        if (SEL && yscale) {
#pragma unroll
            for (int k = 0; k < 4; ++k) yr[k] = bf16x8_scale(yr[k], __shfl(ysc, 4 * ((lane >> 4) & 3) + k));
        }
        transpose4_to_lds(Yt, wat + wg8, wg8, yr);
        __syncthreads();   // the tile is complete; the other buffer is free once every wavefront is here
        if (ti + 1 < t1) RGNN_W_FETCH(ti + 1)
        if (ti + 2 < t1) RGNN_W_FETCH_IDX(ti + 2)
#pragma unroll
        for (int s = 0; s < TMW / 16; ++s) {
            const bf16x8 ah = *reinterpret_cast<const bf16x8*>(Xt + (wave * 32 + m) * 64 + (rg8 ^ (32 * (wave & 1)) ^ (16 * s)));
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const bf16x8 bh = *reinterpret_cast<const bf16x8*>(Yt + (b * 32 + m) * 64 + (rg8 ^ (32 * (b & 1)) ^ (16 * s)));
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc[b], 0, 0, 0);
            }
        }
        if (NBUF == 1) __syncthreads();   // operand reads are done before the next tile is transposed in
    }
#undef RGNN_W_FETCH_IDX
#undef RGNN_W_FETCH
}

template <bool GATHER, bool DYG, bool SEL = false>
static rgnn_status_t launch_wgrad(const TypedLinearWgradBf16Args& a, hipStream_t st) {
    constexpr int D = 128, NBUF = 1;
    const size_t lds = sizeof(unsigned short) * NBUF * (2 * D * 64);
    auto kern = typed_linear_wgrad_bf16_kernel<D, GATHER, DYG, NBUF, SEL>;
    RGNN_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds));
    KernelTimer kt(st, a.label ? a.label : "typed_linear_wgrad");
    TileArgsB t{a.tiles->tile_seg, a.tiles->tile_row0, a.tiles->tile_row1, a.tiles->chunk_tile};
    hipLaunchKernelGGL(kern, dim3(a.tiles->num_chunks), dim3(256), lds, st, t, a.tiles->chunk_slot,
                       static_cast<const unsigned short*>(a.X), a.gather, static_cast<const unsigned short*>(a.dY), a.part,
                       a.ysel, static_cast<const unsigned short*>(a.dY_alt), a.yscale);
    RGNN_HIP(hipGetLastError());
    return RGNN_OK;
}

// Fills the partial slots only; the caller sums them with the slot reduction of typed_linear.hip.
rgnn_status_t typed_linear_wgrad_bf16(int d, const TypedLinearWgradBf16Args& a, hipStream_t st) {
    if (d != 128) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed_linear_wgrad_bf16: width %d not supported (128)", d);
    if (a.tiles->num_tiles == 0) return RGNN_OK;
    const bool g = a.gather != nullptr, dg = g && a.dy_gathered;
    if (a.ysel) {
        if (!g || dg || !a.dY_alt) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed_linear_wgrad_bf16: the row selector needs gathered X and ungathered dY");
        return launch_wgrad<true, false, true>(a, st);
    }
    if (g && dg) return launch_wgrad<true, true>(a, st);
    if (g) return launch_wgrad<true, false>(a, st);
    return launch_wgrad<false, false>(a, st);
}

template <int CD, int OD, bool A_BF16, bool W_BF16, bool WT, bool GATHER, bool SCATTER, bool Y_BF16, bool ACC>
static rgnn_status_t launch(const TypedLinearBf16Args& a, hipStream_t st) {
    constexpr int LS = CD + 8, APL = A_BF16 ? 1 : 2, WPL = W_BF16 ? 1 : 2;
    const size_t lds = sizeof(unsigned short) * ((size_t)WPL * OD * LS + 4 * (APL * 32 * LS + 64));
    auto kern = typed_linear_bf16_kernel<CD, OD, A_BF16, W_BF16, WT, GATHER, SCATTER, Y_BF16, ACC>;
    RGNN_TRY(allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds));
    KernelTimer kt(st, a.label ? a.label : "typed_linear_bf16");
    TileArgsB t{a.tiles->tile_seg, a.tiles->tile_row0, a.tiles->tile_row1, a.tiles->chunk_tile};
    hipLaunchKernelGGL(kern, dim3(a.tiles->num_chunks), dim3(256), lds, st, t, a.A, a.gather, a.W, a.Y, a.A_alt, a.rowscale);
    RGNN_HIP(hipGetLastError());
    return RGNN_OK;
}

template <int D, bool A_BF16, bool W_BF16, bool WT, bool Y_BF16, bool ACC = false>
static rgnn_status_t launch_gs(const TypedLinearBf16Args& a, hipStream_t st) {
    const bool g = a.gather != nullptr, sc = g && a.scatter_out;
    if (a.A_alt && !(g && !sc)) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed_linear_bf16: a second row tensor needs gathered, unscattered rows");
    if (a.rowscale && !A_BF16) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed_linear_bf16: the row scale is built for bf16 rows");
    if (g && sc) return launch<D, D, A_BF16, W_BF16, WT, true, true, Y_BF16, ACC>(a, st);
    if constexpr (ACC) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed_linear_bf16: accumulation is built for gathered + scattered rows only");
    if (g) return launch<D, D, A_BF16, W_BF16, WT, true, false, Y_BF16, false>(a, st);
    return launch<D, D, A_BF16, W_BF16, WT, false, false, Y_BF16, false>(a, st);
}

// The combinations the layers use.  Below width 128 only forward products with fp32 results occur
// (intermediate rows are fp32 there); at width 128 every row operand is bf16.
template <int D>
static rgnn_status_t launch_d(const TypedLinearBf16Args& a, hipStream_t st) {
    if constexpr (D < 128) {
        if (a.y_bf16 || a.transpose_w || a.accumulate) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed_linear_bf16: combination needs width 128");
        if (a.a_bf16 && a.w_bf16) return launch_gs<D, true, true, false, false>(a, st);      // X W
        if (!a.a_bf16 && a.w_bf16) return launch_gs<D, false, true, false, false>(a, st);    // Z Wo
        if (!a.a_bf16 && !a.w_bf16) return launch_gs<D, false, false, false, false>(a, st);  // K Watt_bd
    } else {
        if (!a.a_bf16) RGNN_FAIL(RGNN_EUNSUPPORTED, "typed_linear_bf16: width 128 takes bf16 rows");
        if (a.accumulate) {
            if (a.w_bf16 && a.transpose_w && !a.y_bf16) return launch_gs<D, true, true, true, false, true>(a, st);  // dX += dQ Wq^T
            RGNN_FAIL(RGNN_EUNSUPPORTED, "typed_linear_bf16: accumulation is built for fp32 results of bf16 W^T only");
        }
        if (a.w_bf16 && !a.transpose_w && a.y_bf16) return launch_gs<D, true, true, false, true>(a, st);    // X W -> Hs, K, Q, V
        if (a.w_bf16 && !a.transpose_w && !a.y_bf16) return launch_gs<D, true, true, false, false>(a, st);  // Z Wo -> out
        if (!a.w_bf16 && !a.transpose_w && a.y_bf16) return launch_gs<D, true, false, false, true>(a, st);  // K Watt_bd -> Ka
        if (a.w_bf16 && a.transpose_w && a.y_bf16) return launch_gs<D, true, true, true, true>(a, st);      // dY W^T -> bf16 rows
        if (a.w_bf16 && a.transpose_w && !a.y_bf16) return launch_gs<D, true, true, true, false>(a, st);    // dK Wk^T -> fp32 dX part
        if (!a.w_bf16 && a.transpose_w && a.y_bf16) return launch_gs<D, true, false, true, true>(a, st);    // dKa Watt_bd^T
    }
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
