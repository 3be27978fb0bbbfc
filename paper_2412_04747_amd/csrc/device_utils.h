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

// sum over an aligned group of W lanes (W a power of two, at most 64)
template <int W>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
    for (int o = W / 2; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
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

inline unsigned blocks_for(size_t n, unsigned per_block) { return (unsigned)((n + per_block - 1) / per_block); }

#define RGNN_CHECK_LAUNCH() RGNN_HIP(hipGetLastError())
#define RGNN_DISPATCH_D(D_, CALL)                                                      \
    do {                                                                               \
        if ((D_) == 64) { constexpr int DD = 64; CALL; }                               \
        else if ((D_) == 32) { constexpr int DD = 32; CALL; }                          \
        else if ((D_) == 128) { constexpr int DD = 128; CALL; }                        \
        else RGNN_FAIL(RGNN_EUNSUPPORTED, "feature width %d not supported (32/64/128)", (int)(D_)); \
    } while (0)

}  // namespace rgnn
