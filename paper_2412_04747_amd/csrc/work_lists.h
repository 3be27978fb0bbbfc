// Work lists of the kernels, planned on the host from the offset arrays of the graph index:
// row tiles of the typed-linear kernels (grouped into chunks, one workgroup each) and items of
// the traversal kernels (segments of a CSR-like list, the long ones cut into pieces).
// Plain C++ on std::vector, no device code: graph.hip uploads the plans, and the host tests
// exercise this header on its own.
#pragma once
#include <stdint.h>
#include <algorithm>
#include <vector>

namespace rgnn {

constexpr int kTileRows = 64;       // rows per typed-linear tile
constexpr int kMaxChunks = 4096;    // tile chunks (workgroups) of the typed-linear kernels: several per resident
                                    // workgroup slot, so the hardware dispatcher evens out the tail
constexpr int kWideChunksPerCU = 3; // weight-gradient lists: one chunk per workgroup a compute unit can hold (three),
                                    // so that every chunk is resident at once and none is left for a second round
constexpr int kMinChunks = 512;     // fewer chunks than this only when there are fewer tiles
constexpr int kChunkTiles = 8;      // tiles a chunk spans before the chunk count grows beyond kMinChunks
constexpr int kItemMax = 256;       // longest traversal item (entries)
constexpr int kItemTarget = 65536;  // lists are cut finer while they yield fewer items than this
constexpr int kSerialMax = 32;      // longest segment a single lane walks; longer ones get a wavefront

// Tiles of at most `tile_rows` rows that never straddle a segment, in row order, grouped into
// chunks of consecutive tiles.  A chunk accumulates one weight gradient per segment it touches
// and flushes each to a "slot"; slots are numbered in chunk order, so the slots of one segment
// are the consecutive range [seg_slot_ptr[s], seg_slot_ptr[s + 1]).
struct TilePlan {
    int32_t tile_rows = 0, num_tiles = 0, num_chunks = 0, num_slots = 0, num_segs = 0;
    std::vector<int32_t> tile_seg, tile_row0, tile_row1;   // [num_tiles] segment, first row, end row
    std::vector<int32_t> chunk_tile;                       // [num_chunks + 1]
    std::vector<int32_t> chunk_slot;                       // [num_chunks] first slot of the chunk
    std::vector<int32_t> seg_slot_ptr;                     // [num_segs + 1]
};

inline TilePlan plan_tiles(const std::vector<int32_t>& seg_ptr, int tile_rows, int max_chunks = kMaxChunks) {
    TilePlan t;
    const int S = (int)seg_ptr.size() - 1;
    for (int s = 0; s < S; ++s)
        for (int32_t a = seg_ptr[s]; a < seg_ptr[s + 1]; a += tile_rows) {
            t.tile_seg.push_back(s);
            t.tile_row0.push_back(a);
            t.tile_row1.push_back(std::min<int32_t>(a + tile_rows, seg_ptr[s + 1]));
        }
    const int nt = (int)t.tile_seg.size();
    // a chunk pays for one weight-tile load and one weight-gradient flush, so it should span several
    // tiles; but small inputs still need a few hundred chunks to occupy the compute units
    const int nc = std::min(max_chunks, std::max(std::min(nt, kMinChunks), nt / kChunkTiles));
    t.chunk_tile.assign(nc + 1, 0);
    t.chunk_slot.assign(std::max(nc, 1), 0);
    t.seg_slot_ptr.assign(S + 1, 0);
    std::vector<int32_t> seg_slots(std::max(S, 0), 0);
    int slots = 0;
    for (int c = 0; c < nc; ++c) {
        t.chunk_tile[c] = (int32_t)((int64_t)nt * c / nc);
        t.chunk_tile[c + 1] = (int32_t)((int64_t)nt * (c + 1) / nc);
        t.chunk_slot[c] = slots;
        for (int i = t.chunk_tile[c]; i < t.chunk_tile[c + 1]; ++i)
            if (i == t.chunk_tile[c] || t.tile_seg[i] != t.tile_seg[i - 1]) {
                ++slots;
                seg_slots[t.tile_seg[i]]++;
            }
    }
    for (int s = 0; s < S; ++s) t.seg_slot_ptr[s + 1] = t.seg_slot_ptr[s] + seg_slots[s];
    t.tile_rows = tile_rows;
    t.num_tiles = nt;
    t.num_chunks = nc;
    t.num_slots = slots;
    t.num_segs = S;
    return t;
}

// Segments ptr[0..S] of a CSR-like list as items of at most `max_len` entries.  An item is a
// whole segment (slot < 0: its result goes to output row `row`) or a piece of a cut segment
// (slot >= 0: its result goes to partial row `slot`; split_* say which partial rows sum to
// which output row).  Segments shorter than `min_len` are left out (their owner handles them
// elsewhere).  Items are ordered by length, longest first (stable): the lanes of a wavefront and
// the wavefronts of a workgroup then walk items of equal length and finish together, and the
// long items are scheduled before the short ones fill the tail.  Among items of equal length
// the pieces of cut segments come first; pieces of at most kShortLen entries all come before the
// whole segments of that size.  So the whole segments with 2..kShortLen entries form one
// contiguous range [first_short, first_short + num_short), directly followed by those with
// exactly one entry, [first_single, first_single + num_single); both have kernels of their own.
constexpr int kShortLen = 4;

struct ItemPlan {
    int32_t num_partials = 0, num_split = 0, first_single = 0, num_single = 0, first_short = 0, num_short = 0;
    std::vector<int32_t> beg, end, row, slot;      // [num_items]
    std::vector<int32_t> split_row, split_ptr;     // [num_split], [num_split + 1] range of partial rows
    std::vector<int32_t> part_item, part_split;    // [num_partials] item writing the partial row; index into split_*
    std::vector<int32_t> long_item;                // items with more than kSerialMax entries, and every piece
};

inline ItemPlan plan_items(const std::vector<int32_t>& ptr, int max_len, int min_len = 0) {
    ItemPlan L;
    const int S = (int)ptr.size() - 1;
    L.split_ptr.push_back(0);
    for (int s = 0; s < S; ++s) {
        const int32_t a = ptr[s], b = ptr[s + 1];
        if (b - a < min_len) continue;
        if (b - a <= max_len) {
            L.beg.push_back(a); L.end.push_back(b); L.row.push_back(s); L.slot.push_back(-1);
        } else {
            for (int32_t c = a; c < b; c += max_len) {
                L.part_item.push_back((int32_t)L.beg.size());
                L.part_split.push_back((int32_t)L.split_row.size());
                L.beg.push_back(c); L.end.push_back(std::min<int32_t>(c + max_len, b));
                L.row.push_back(s); L.slot.push_back(L.num_partials++);
            }
            L.split_row.push_back(s);
            L.split_ptr.push_back(L.num_partials);
        }
    }
    L.num_split = (int32_t)L.split_row.size();
    const int n = (int)L.beg.size();
    int longest = 0;
    for (int i = 0; i < n; ++i) longest = std::max(longest, L.end[i] - L.beg[i]);
    const int short_base = 2 * longest + 2;     // above every key of the longer items
    auto key = [&](int i) {
        const int len = L.end[i] - L.beg[i];
        if (len > kShortLen) return 2 * (longest - len) + (L.slot[i] < 0 ? 1 : 0);
        if (L.slot[i] >= 0) return short_base;                    // short pieces, before the short whole segments
        return short_base + 1 + (kShortLen - len);                // whole: kShortLen, ..., 2, 1, 0 entries
    };
    std::vector<int32_t> cnt(short_base + kShortLen + 3, 0), perm(n), inv(n);
    for (int i = 0; i < n; ++i) cnt[key(i) + 1]++;
    for (size_t l = 0; l + 1 < cnt.size(); ++l) cnt[l + 1] += cnt[l];
    for (int i = 0; i < n; ++i) { const int p = cnt[key(i)]++; perm[p] = i; inv[i] = p; }
    auto apply = [&](std::vector<int32_t>& v) {
        std::vector<int32_t> t(n);
        for (int p = 0; p < n; ++p) t[p] = v[perm[p]];
        v.swap(t);
    };
    apply(L.beg); apply(L.end); apply(L.row); apply(L.slot);
    for (auto& it : L.part_item) it = inv[it];
    L.first_single = n;
    L.first_short = n;
    for (int i = 0; i < n; ++i) {
        const int len = L.end[i] - L.beg[i];
        if (len == 1 && L.slot[i] < 0) {
            if (L.num_single == 0) L.first_single = i;
            ++L.num_single;
        }
        if (len >= 2 && len <= kShortLen && L.slot[i] < 0) {
            if (L.num_short == 0) L.first_short = i;
            ++L.num_short;
        }
        if (L.end[i] - L.beg[i] > kSerialMax || L.slot[i] >= 0) L.long_item.push_back(i);
    }
    return L;
}

// Longest item for a list of `total` entries: kItemMax on large lists; shorter on small ones, where
// a few long serial walks would otherwise be the whole run time (never below kSerialMax, so that
// every item a single lane walks stays short).
inline int item_cut(int64_t total) {
    int cut = kSerialMax;
    while (cut < kItemMax && (int64_t)cut * kItemTarget < total) cut *= 2;
    return cut;
}

// Ids of the segments of a CSR-like list that are longer than kSerialMax entries.
inline std::vector<int32_t> long_segments(const std::vector<int32_t>& ptr) {
    std::vector<int32_t> ids;
    for (size_t i = 0; i + 1 < ptr.size(); ++i)
        if (ptr[i + 1] - ptr[i] > kSerialMax) ids.push_back((int32_t)i);
    return ids;
}

}  // namespace rgnn
