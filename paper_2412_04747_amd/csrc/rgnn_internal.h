// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <algorithm>
#include <string>
#include <vector>
#include "../../include/rgnn.h"
#include "work_lists.h"

namespace rgnn {

// ---- error plumbing ------------------------------------------------------
void set_error(const char* fmt, ...);
#define RGNN_HIP(call)                                                                  \
    do {                                                                                \
        hipError_t e_ = (call);                                                         \
        if (e_ != hipSuccess) {                                                         \
            rgnn::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
            return RGNN_EHIP;                                                           \
        }                                                                               \
    } while (0)
#define RGNN_FAIL(code, ...)          \
    do {                              \
        rgnn::set_error(__VA_ARGS__); \
        return (code);                \
    } while (0)
#define RGNN_TRY(expr)                      \
    do {                                    \
        rgnn_status_t s_ = (expr);          \
        if (s_ != RGNN_OK) return s_;       \
    } while (0)

// ---- optional kernel timing (profile.hip) ----------------------------------
class KernelTimer {
  public:
    KernelTimer(hipStream_t st, const char* name);
    ~KernelTimer();
  private:
    hipStream_t st_;
    int idx_;
};

// ---- work lists ----------------------------------------------------------
// Row tiles of a segmented row range (rows grouped by relation or node type),
// cut into `num_chunks` contiguous chunks, one per persistent workgroup.  A
// chunk owns one partial-gradient slot per distinct segment it touches; slots
// are numbered in (chunk, segment) order, which is also segment order, so the
// slots of one segment are contiguous (seg_slot_ptr).
struct TileList {
    int32_t tile_rows = 0;       // rows per tile
    int32_t num_tiles = 0;
    int32_t num_chunks = 0;
    int32_t num_slots = 0;
    int32_t num_segs = 0;
    int32_t* tile_seg = nullptr;     // [num_tiles]  device
    int32_t* tile_row0 = nullptr;    // [num_tiles]  first row of the tile
    int32_t* tile_row1 = nullptr;    // [num_tiles]  end row (exclusive; <= row0 + tile_rows)
    int32_t* chunk_tile = nullptr;   // [num_chunks+1]
    int32_t* chunk_slot = nullptr;   // [num_chunks]  first slot of the chunk
    int32_t* seg_slot_ptr = nullptr; // [num_segs+1]
};

// Segments of a CSR-like list cut into items of at most `max_len` entries.  An
// item is either a whole segment (slot < 0: the result goes to row `row`) or a
// piece of a split segment (slot >= 0: the result goes to partial row `slot`;
// split_* lists say which partial rows sum to which output row).
struct ItemList {
    int32_t num_items = 0;
    int32_t num_partials = 0;
    int32_t num_split = 0;
    int32_t* beg = nullptr;        // [num_items]
    int32_t* end = nullptr;        // [num_items]
    int32_t* row = nullptr;        // [num_items] segment id
    int32_t* slot = nullptr;       // [num_items] partial row or -1
    int32_t* split_row = nullptr;  // [num_split]
    int32_t* split_ptr = nullptr;  // [num_split+1] range of partial rows
    int32_t* part_item = nullptr;  // [num_partials] item that writes the partial row
    int32_t num_long = 0;
    int32_t* long_item = nullptr;  // [num_long] items with more than kSerialMax entries, and every piece of a cut segment
    int32_t* part_split = nullptr; // [num_partials] index into split_* of its segment
    int32_t first_single = 0;      // items [first_single, first_single + num_single) are the whole segments
    int32_t num_single = 0;        // with exactly one entry
    int32_t first_short = 0;       // items [first_short, first_short + num_short) are the whole segments with
    int32_t num_short = 0;         // 2..kShortLen entries; the single-entry ones follow directly
};

}  // namespace rgnn

namespace rgnn {
// Ids of the segments of a CSR-like list that are longer than kSerialMax entries.
struct LongList {
    int32_t n = 0;
    int32_t* ids = nullptr;
};
}  // namespace rgnn

struct rgnn_graph {
    int64_t N = 0, E = 0, P = 0, Q = 0;
    int32_t R = 0, T = 0;
    int num_cus = 0;                       // compute units of the device the graph lives on
    int64_t max_in_degree = 0, max_pair_out_degree = 0, num_single_pairs = 0;
    size_t index_bytes = 0;
    int32_t* idx[RGNN_IDX_COUNT] = {};     // device arrays, see RGNN_IDX_*
    int64_t idx_len[RGNN_IDX_COUNT] = {};
    float* in_invc = nullptr;              // [E] 1 / c_{v,r} per CSR edge
    float* out_invc = nullptr;             // [E] the same per pair-major edge: in_invc[out_epos[j]]
    rgnn::TileList pair_tiles;             // pairs segmented by relation
    rgnn::TileList node_tiles;             // nodes (in ntype_perm order) segmented by type
    rgnn::TileList all_tiles;              // all nodes as one segment (RGCN self-loop)
    rgnn::TileList pair_tiles_wide;        // same tiles as pair_tiles / node_tiles in fewer, longer chunks: for the
    rgnn::TileList node_tiles_wide;        // weight-gradient kernels, whose chunks each flush a d x d partial
    rgnn::ItemList dst_items;              // CSR edges by destination
    rgnn::ItemList pair_items;             // transposed edges by pair
    rgnn::ItemList pair_items_multi;       // the same, pairs with two or more edges only
    rgnn::ItemList srcpair_items;          // pairs by source node (never cut)
    int32_t* in_pair_tag = nullptr;        // [E] in_pair with the top bit set when the pair has a single edge
    float* pair_scale = nullptr;           // [P] 1 / c_{v,r} of the only edge of a single-edge pair, 1 for the other pairs
    int32_t* pair_ysel = nullptr;          // [P] pair id, or for a pair with one edge the top bit | that edge's destination
    int32_t* relrun_dst = nullptr;         // [Q] destination of the runs in (relation, destination) order: run_dst[relrun_idx[i]]
    int32_t* rel_src_type = nullptr;       // [R] node type of the sources of relation r (0 for a relation without edges)
    bool rel_src_tied = false;             // every relation's sources are of one node type (rel_src_type is then valid)
    rgnn::ItemList relrun_items;           // runs by relation
    rgnn::ItemList relpair_items;          // pairs by relation (rows of the compact tensors are already in this order)
    rgnn::LongList long_runs;              // runs (run_ptr) too long for one lane
    rgnn::LongList long_pairs;             // pairs (out_ptr) too long for one lane
    std::vector<void*> allocs;             // every device allocation, for destroy
};

namespace rgnn {

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// "<label>.wgrad", with static storage (kernel-timer names must outlive the call)
const char* wgrad_label(const char* label);

// Raises a kernel's dynamic LDS limit once per (kernel, device) instead of on every launch.
rgnn_status_t allow_dynamic_lds(const void* kernel, size_t bytes);

// Device address of the library's static scratch buffer on the current device (layers.hip); resolved once per device.
rgnn_status_t static_scratch(void** p);

// ---- kernel launchers (typed_linear.hip) --------------------------------
struct TypedLinearArgs {
    const TileList* tiles;
    const float* X;          // input rows
    const int32_t* gather;   // row i reads X[gather[i]] (nullptr: X[i])
    const float* W;          // [segs][KD][ND]
    float* Y;                // output rows
    int scatter_out;         // 1: row i writes Y[gather[i]], 0: Y[i]
    int accumulate;          // 1: Y += result
    const float* vec;        // optional [segs][ND]: s_out[i][h] = Y_row . vec[seg] over the h-th of s_heads column slices
    float* s_out;            // [rows][s_heads]
    int s_heads = 1;         // a power of two with ND / s_heads >= 16
    const char* label;       // name in the timing report (nullptr: default)
};
rgnn_status_t typed_linear_fwd(int d_in, int d_out, const TypedLinearArgs& a, hipStream_t st);

struct TypedLinearBwdArgs {
    const TileList* tiles;
    const float* X;          // forward input rows
    const int32_t* gather;   // forward gather (nullptr: identity)
    const float* W;          // [segs][KD][ND]
    const float* dY;         // gradient of the forward output
    int dy_gathered;         // 1: row i reads dY[gather[i]], 0: dY[i]
    float* dXrow;            // [rows][KD] per-row input gradient dY_i W^T (row i, or gather[i] if scatter_dx)
    int scatter_dx;
    const float* rowscale;   // optional [rows]: A[seg] = sum_i rowscale[i] X_row_i
    const float* vec;        // optional [segs][KD] (with rowscale): dXrow[i] += rowscale[i] * vec[seg]
    float* dW;               // [segs][KD][ND]
    float* Avec;             // [segs][KD] (with rowscale); [segs][sel_heads][KD] = sum over the rows of hcoef[i][h] X[g(i)] (with hcoef)
    float* part;             // scratch [num_slots][KD*ND + KD]
    const char* label;
    // Optional row selector (widths up to 64, ungathered dY): row i of dY is
    // ysel[i] < 0 ? scale_i * dY_alt[ysel[i] & 0x7FFFFFFF] : dY[ysel[i]].  rowscale[i] and scale_i then come
    // interleaved as ds_yscale[i] = (rowscale_i, scale_i) and `rowscale` stays null (scale_i is read only where
    // the top bit of ysel[i] is set).
    const int32_t* ysel = nullptr;
    const float* dY_alt = nullptr;
    const float2* ds_yscale = nullptr;
    // Per-head row selector (widths up to 64, sel_heads in {2, 4}, instead of rowscale / vec / ds_yscale): a selected
    // row is dY_alt[row] * a[h] + b[h] * wvec[seg] on the columns of head h, (b[0..H), a[0..H)) = hcoef[i] for row i
    const float* hcoef = nullptr;    // [rows][2][sel_heads]
    const float* wvec = nullptr;     // [segs][ND]
    int sel_heads = 0;
};
// bf16 matrix-core variant (typed_linear_bf16.hip): Y[i] = A[g(i)] W[seg]  (or W[seg]^T)
struct TypedLinearBf16Args {
    const TileList* tiles;
    const void* A;           // rows: bf16 (a_bf16) or fp32
    int a_bf16;
    const int32_t* gather;   // row i reads A[gather[i]] (nullptr: A[i])
    int scatter_out;         // 1: row i writes Y[gather[i]]
    const void* W;           // [segs][d][d]: bf16 (w_bf16) or fp32
    int w_bf16;
    int transpose_w;         // 1: multiply by W[seg]^T
    void* Y;                 // output rows: bf16 (y_bf16) or fp32
    int y_bf16;
    int accumulate;          // 1: Y += result (fp32 Y)
    const char* label;
    const void* A_alt = nullptr;   // gathered rows only: a gather entry with the top bit set reads row
                                   // (entry & 0x7FFFFFFF) of this tensor instead of A
    const float* rowscale = nullptr;   // bf16 rows only: row i of the tiles is multiplied by rowscale[i]
};
rgnn_status_t typed_linear_bf16(int d, const TypedLinearBf16Args& a, hipStream_t st);

// bf16 matrix-core weight gradient: part[slot] = sum over the chunk's rows of X[g(i)]^T dY[i];
// typed_linear_slot_reduce then adds a segment's slots into dW.
struct TypedLinearWgradBf16Args {
    const TileList* tiles;
    const void* X;           // bf16 rows
    const int32_t* gather;
    int dy_gathered;         // 1: dY rows are read through the gather list as well
    const void* dY;          // bf16 rows
    float* part;
    const char* label;
    // optional row selector for dY (ungathered dY only): row i is dY[ysel[i]], or dY_alt[ysel[i] & 0x7FFFFFFF]
    // when the top bit of ysel[i] is set
    const int32_t* ysel = nullptr;
    const void* dY_alt = nullptr;
    const float* yscale = nullptr;   // with ysel: row i is also multiplied by yscale[i]
};
rgnn_status_t typed_linear_wgrad_bf16(int d, const TypedLinearWgradBf16Args& a, hipStream_t st);
rgnn_status_t typed_linear_slot_reduce(int d_in, int d_out, const TileList& tiles, const float* part, float* dW,
                                       float* Avec, hipStream_t st);

size_t typed_linear_bwd_scratch_floats(int d_in, int d_out, const TileList& t, int vectors = 1);   // vectors: of a slot's vector part
rgnn_status_t typed_linear_bwd(int d_in, int d_out, const TypedLinearBwdArgs& a, hipStream_t st);

}  // namespace rgnn
