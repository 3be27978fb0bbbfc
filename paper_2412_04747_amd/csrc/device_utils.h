// Device helpers shared by the traversal and HGT kernels.  Internal.
#pragma once
#include "rgnn_internal.h"

namespace rgnn {

// Device view of an ItemList: item i covers entries [beg[i], end[i]) of a CSR-like list, belongs to
// segment row[i], and writes to the segment's own output row (slot < 0) or to partial row `slot`.
struct Items {
    int n;
    const int32_t* beg;
    const int32_t* end;
    const int32_t* row;
    const int32_t* slot;
};
inline Items dev_items(const ItemList& L) { return Items{L.num_items, L.beg, L.end, L.row, L.slot}; }

// Cross-lane moves inside a row of 16 lanes on the VALU (DPP), no LDS traffic.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm:[1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm:[2,3,0,1]
constexpr int kDppHalfMirror = 0x141;    // lane i <-> 7 - i within each 8 lanes
constexpr int kDppMirror = 0x140;        // lane i <-> 15 - i within each 16 lanes
constexpr int kDppRowBcast0 = 0x150;     // + n: every lane of a row reads the row's lane n

// sum over an aligned group of W lanes (W a power of two, at most 64); every lane of the group gets the
// same bits.  Up to 16 lanes the exchange partners are chosen so that each step is one DPP add: after
// the two quad steps a quad holds one value, so mirroring a half row (then the row) pairs different
// quads (halves) just as a butterfly would.
template <int W>
__device__ __forceinline__ float group_sum(float v) {
    if (W >= 2) v += dpp_move<kDppQuadSwap1>(v);
    if (W >= 4) v += dpp_move<kDppQuadSwap2>(v);
    if (W >= 8) v += dpp_move<kDppHalfMirror>(v);
    if (W >= 16) v += dpp_move<kDppMirror>(v);
    if (W >= 32) v += __shfl_xor(v, 16);
    if (W >= 64) v += __shfl_xor(v, 32);
    return v;
}
// value held by lane `lane` of the caller's aligned group of W lanes; with W == 16 and a `lane` the compiler
// can fold to a constant this is one DPP move
template <int W, typename Tv>
__device__ __forceinline__ Tv group_lane(Tv v, int lane) {
    if constexpr (W == 16) {
        switch (lane) {
            case 0: return dpp_move<kDppRowBcast0 + 0>(v);
            case 1: return dpp_move<kDppRowBcast0 + 1>(v);
            case 2: return dpp_move<kDppRowBcast0 + 2>(v);
            case 3: return dpp_move<kDppRowBcast0 + 3>(v);
            case 4: return dpp_move<kDppRowBcast0 + 4>(v);
            case 5: return dpp_move<kDppRowBcast0 + 5>(v);
            case 6: return dpp_move<kDppRowBcast0 + 6>(v);
            case 7: return dpp_move<kDppRowBcast0 + 7>(v);
            case 8: return dpp_move<kDppRowBcast0 + 8>(v);
            case 9: return dpp_move<kDppRowBcast0 + 9>(v);
            case 10: return dpp_move<kDppRowBcast0 + 10>(v);
            case 11: return dpp_move<kDppRowBcast0 + 11>(v);
            case 12: return dpp_move<kDppRowBcast0 + 12>(v);
            case 13: return dpp_move<kDppRowBcast0 + 13>(v);
            case 14: return dpp_move<kDppRowBcast0 + 14>(v);
            default: return dpp_move<kDppRowBcast0 + 15>(v);
        }
    }
    return __shfl(v, lane, W);
}
__device__ __forceinline__ float group_sum_dyn(float v, int w) {
    for (int o = w / 2; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float dot4(const float4& a, const float4& b) {
    return a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
}
__device__ __forceinline__ void fma4(float4& acc, float c, const float4& v) {
    acc.x += c * v.x; acc.y += c * v.y; acc.z += c * v.z; acc.w += c * v.w;
}

// ---- feature rows in fp32 or bf16 storage --------------------------------------------------------
// A lane owns the columns one 16-byte load brings in: 4 of an fp32 row, 8 of a bf16 row.  All
// arithmetic is fp32; bf16 is a storage format only (widening is exact, narrowing rounds to
// nearest even).
typedef unsigned short bf16_t;   // bit pattern of a bfloat16

template <typename T> struct RowT;
template <> struct RowT<float> { static constexpr int V = 4; };
template <> struct RowT<bf16_t> { static constexpr int V = 8; };

// two fp32 -> packed bf16 pair (lo in bits 0..15), round to nearest even, one v_cvt_pk_bf16_f32
typedef float rgnn_v2f __attribute__((ext_vector_type(2)));
typedef __bf16 rgnn_bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned bf16_pack2(float lo, float hi) {
    const rgnn_v2f v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, rgnn_bf16x2));
}

// v[0..V) = p[0..V), p 16-byte aligned for V * sizeof(T) == 16 (8-byte aligned for four bf16)
template <int V>
__device__ __forceinline__ void load_cols(const float* __restrict__ p, float (&v)[V]) {
#pragma unroll
    for (int q = 0; q < V / 4; ++q) {
        const float4 t = reinterpret_cast<const float4*>(p)[q];
        v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
    }
}
// the same with a non-temporal hint: rows that are gathered once and not read again soon
typedef float rgnn_v4f __attribute__((ext_vector_type(4)));
template <int V>
__device__ __forceinline__ void load_cols_nt(const float* __restrict__ p, float (&v)[V]) {
#pragma unroll
    for (int q = 0; q < V / 4; ++q) {
        const rgnn_v4f t = __builtin_nontemporal_load(reinterpret_cast<const rgnn_v4f*>(p) + q);
        v[4 * q] = t[0]; v[4 * q + 1] = t[1]; v[4 * q + 2] = t[2]; v[4 * q + 3] = t[3];
    }
}
template <int V>
__device__ __forceinline__ void load_cols(const bf16_t* __restrict__ p, float (&v)[V]) {
    if constexpr (V == 8) {
        const uint4 t = *reinterpret_cast<const uint4*>(p);
        v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
        v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
        v[4] = __uint_as_float(t.z << 16); v[5] = __uint_as_float(t.z & 0xFFFF0000u);
        v[6] = __uint_as_float(t.w << 16); v[7] = __uint_as_float(t.w & 0xFFFF0000u);
    } else {
        static_assert(V == 4, "four or eight columns per lane");
        const uint2 t = *reinterpret_cast<const uint2*>(p);
        v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
        v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
    }
}
typedef unsigned rgnn_v4u __attribute__((ext_vector_type(4)));
template <int V>
__device__ __forceinline__ void load_cols_nt(const bf16_t* __restrict__ p, float (&v)[V]) {
    if constexpr (V == 8) {
        const rgnn_v4u t = __builtin_nontemporal_load(reinterpret_cast<const rgnn_v4u*>(p));
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            v[2 * q] = __uint_as_float(t[q] << 16);
            v[2 * q + 1] = __uint_as_float(t[q] & 0xFFFF0000u);
        }
    } else {
        load_cols(p, v);
    }
}
template <int V>
__device__ __forceinline__ void store_cols(float* __restrict__ p, const float (&v)[V]) {
#pragma unroll
    for (int q = 0; q < V / 4; ++q)
        reinterpret_cast<float4*>(p)[q] = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
}
template <int V>
__device__ __forceinline__ void store_cols(bf16_t* __restrict__ p, const float (&v)[V]) {
    if constexpr (V == 8) {
        *reinterpret_cast<uint4*>(p) = make_uint4(bf16_pack2(v[0], v[1]), bf16_pack2(v[2], v[3]), bf16_pack2(v[4], v[5]),
                                                  bf16_pack2(v[6], v[7]));
    } else {
        static_assert(V == 4, "four or eight columns per lane");
        *reinterpret_cast<uint2*>(p) = make_uint2(bf16_pack2(v[0], v[1]), bf16_pack2(v[2], v[3]));
    }
}
template <int V>
__device__ __forceinline__ void zero_cols(float (&v)[V]) {
#pragma unroll
    for (int q = 0; q < V; ++q) v[q] = 0.f;
}
template <int V>
__device__ __forceinline__ void fma_cols(float (&acc)[V], float c, const float (&v)[V]) {
#pragma unroll
    for (int q = 0; q < V; ++q) acc[q] += c * v[q];
}
template <int V>
__device__ __forceinline__ float dot_cols(const float (&a)[V], const float (&b)[V]) {
    float s = 0.f;
#pragma unroll
    for (int q = 0; q < V; ++q) s += a[q] * b[q];
    return s;
}

inline unsigned blocks_for(size_t n, unsigned per_block) { return (unsigned)((n + per_block - 1) / per_block); }

#define RGNN_CHECK_LAUNCH() RGNN_HIP(hipGetLastError())
#define RGNN_DISPATCH_D(D_, ...)                                                       \
    do {                                                                               \
        if ((D_) == 64) { constexpr int DD = 64; __VA_ARGS__; }                               \
        else if ((D_) == 32) { constexpr int DD = 32; __VA_ARGS__; }                          \
        else if ((D_) == 128) { constexpr int DD = 128; __VA_ARGS__; }                        \
        else RGNN_FAIL(RGNN_EUNSUPPORTED, "feature width %d not supported (32/64/128)", (int)(D_)); \
    } while (0)

}  // namespace rgnn
