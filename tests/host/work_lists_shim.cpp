// Test-only C wrapper around the host planning code of the library (work_lists.h), so that the
// CPU test suite can check the tile and item plans without a GPU.  Built by tests/test_work_lists.py.
#include "../../paper_2412_04747_amd/csrc/work_lists.h"
#include "../../paper_2412_04747_amd/csrc/schedule.h"

#include <cstring>

static rgnn::ItemPlan g_items;
static rgnn::TilePlan g_tiles;

static int copy_out(const std::vector<int32_t>& v, int32_t* out, int cap) {
    if (out && (int)v.size() <= cap && !v.empty()) std::memcpy(out, v.data(), v.size() * sizeof(int32_t));
    return (int)v.size();
}

extern "C" {

int wl_plan_items(const int32_t* ptr, int nseg, int max_len, int min_len) {
    g_items = rgnn::plan_items(std::vector<int32_t>(ptr, ptr + nseg + 1), max_len, min_len);
    return (int)g_items.beg.size();
}
// which: 0 beg, 1 end, 2 row, 3 slot, 4 split_row, 5 split_ptr, 6 part_item, 7 part_split, 8 long_item
int wl_items_field(int which, int32_t* out, int cap) {
    const std::vector<int32_t>* f[] = {&g_items.beg, &g_items.end, &g_items.row, &g_items.slot, &g_items.split_row,
                                       &g_items.split_ptr, &g_items.part_item, &g_items.part_split, &g_items.long_item};
    return copy_out(*f[which], out, cap);
}
void wl_items_scalars(int32_t* out6) {
    out6[0] = g_items.num_partials; out6[1] = g_items.num_split; out6[2] = g_items.first_single; out6[3] = g_items.num_single;
    out6[4] = g_items.first_short; out6[5] = g_items.num_short;
}

int wl_plan_tiles(const int32_t* seg_ptr, int nseg, int tile_rows, int max_chunks) {
    g_tiles = rgnn::plan_tiles(std::vector<int32_t>(seg_ptr, seg_ptr + nseg + 1), tile_rows, max_chunks);
    return g_tiles.num_tiles;
}
// which: 0 tile_seg, 1 tile_row0, 2 tile_row1, 3 chunk_tile, 4 chunk_slot, 5 seg_slot_ptr
int wl_tiles_field(int which, int32_t* out, int cap) {
    const std::vector<int32_t>* f[] = {&g_tiles.tile_seg, &g_tiles.tile_row0, &g_tiles.tile_row1, &g_tiles.chunk_tile,
                                       &g_tiles.chunk_slot, &g_tiles.seg_slot_ptr};
    return copy_out(*f[which], out, cap);
}
void wl_tiles_scalars(int32_t* out3) {
    out3[0] = g_tiles.num_chunks; out3[1] = g_tiles.num_slots; out3[2] = g_tiles.num_segs;
}
int wl_item_cut(long long total) { return rgnn::item_cut(total); }
int wl_constant(int which) {
    const int c[] = {rgnn::kTileRows, rgnn::kMaxChunks, rgnn::kWideChunksPerCU, rgnn::kMinChunks, rgnn::kChunkTiles,
                     rgnn::kItemMax, rgnn::kItemTarget, rgnn::kSerialMax, rgnn::kShortLen};
    return c[which];
}

// in: layer, dtype, d, heads, flags, R, rel_src_tied, total entries of the destination-major list (edges),
//     single / short counts of the destination list, of the pair list, of the multi-edge pair list   (14 ints)
// out: the fields of rgnn_schedule_t in declaration order (14 ints); tile chunk counts are passed through as 0
void wl_pick_schedule(const long long* in, int32_t* out) {
    rgnn::ScheduleIn s;
    s.layer = (int)in[0]; s.dtype = (int)in[1]; s.d = (int)in[2]; s.heads = (int)in[3]; s.flags = (uint32_t)in[4];
    s.R = (int)in[5]; s.rel_src_tied = in[6] != 0; s.item_len = rgnn::item_cut(in[7]);
    s.dst = {(int32_t)in[8], (int32_t)in[9]}; s.pair = {(int32_t)in[10], (int32_t)in[11]};
    s.pair_multi = {(int32_t)in[12], (int32_t)in[13]};
    const rgnn_schedule_t r = rgnn::pick_schedule(s);
    static_assert(sizeof(r) == 14 * sizeof(int32_t), "rgnn_schedule_t is fourteen int32 fields");
    std::memcpy(out, &r, sizeof(r));
}

}  // extern "C"
