// Internal definitions shared by the host planner and the HIP launch code.
#pragma once

#include <cstdint>
#include <mutex>
#include <vector>

#include "smha.h"

namespace smha {

constexpr int kTile = 64;    // keys per K/V tile and query rows per wave of the block kernel
constexpr int kSuper = 128;  // query rows per workgroup: two vertically adjacent tile rows

// Formats of one distinct mask (Sec. 4.2.1 of the paper for the block arrays).
struct MaskFormats {
    int64_t nnz = 0;
    int64_t n_valid16 = 0;
    std::vector<int32_t> row_ptr, col_idx;                 // per-row format (optional)
    std::vector<int32_t> load_row_ptr, load_col_idx;       // all non-empty tiles
    std::vector<int32_t> full_row_ptr, full_col_idx;       // completely unmasked tiles
    std::vector<int32_t> part_row_ptr, part_col_idx;       // partially masked tiles
    std::vector<uint8_t> flags;                            // per load entry, 1 = full
    std::vector<uint64_t> bitmap;                          // n_part * block words
    // 64x64 tiles visited by the block kernel (identical to the arrays above when block == 64)
    std::vector<int32_t> kt_row_ptr, kt_col, kt_bmp;       // kt_bmp: bitmap index or -1 (full)
    std::vector<uint64_t> kt_bitmap;                       // n_part64 * 64 words
};

// The block kernel walks, per 128-row query supertile, the UNION of the key tiles of its two
// 64-row tile rows, so that one staged K/V tile serves both.  code[w] tells wave w (tile row
// 2*super + w) what the tile is for it: -2 = empty (skip), -1 = full, >= 0 = index of its
// 64-word bitmap.
//
// Gathered tiles.  A tile in which only a few key columns are used at all (strided or scattered
// columns) wastes most of a step.  The planner collects the used columns of such tiles of a
// supertile, sorts them and packs them 64 at a time into gathered tiles: `gather` - 1 indexes a
// block of 64 key numbers (one per staged row; unused rows name a key past the sequence, which
// loads as zeros), col is unused, and the bitmaps say which (query, gathered key) pairs are set.
// gather = 0: an ordinary tile of 64 consecutive keys starting at 64 * col.
struct UEntry {
    int32_t col, code[2], gather;
};

// One workgroup's job: supertile `qtile`, union entries [begin, end).  slot < 0: the item
// covers the whole list and writes O directly; slot >= 0: it writes an unnormalised partial
// (O, m, l) of 128 rows to that workspace slot, and `split` is the index (within the mask) of the
// SplitRow that names all parts of its supertile; whichever part finishes last merges them.
// Its gathered tiles are the gcount consecutive blocks of key numbers starting at block gbegin
// (at most kMaxGatherPerItem).
struct Item {
    int32_t qtile, begin, end, slot;
    int32_t gbegin, gcount, split, pad;
};
constexpr int kMaxGatherPerItem = 16;
// a tile with at most this many used key columns is repacked (32 or 48 save a quarter of the steps
// of band masks but measured 5-15 % slower there: gathered tiles always take the bitmap path)
constexpr int kGatherMaxCols = 16;

// The second form of the block kernel reads, per workgroup, a contiguous stream of steps (one per
// staged K/V tile, in execution order across the workgroup's items) and a contiguous stream of items.
// StepRec = {key tile (-1: nothing to load), code for the group's first / second 64 rows (see UEntry),
// meta}; meta = index of the step's item within the workgroup's items, plus kStepFirst / kStepLast on
// an item's first / last step.  ItemRec = {batch, head, 128-row group, workspace slot or -1, split
// group or -1, 0, 0, 0}.
constexpr int32_t kStepFirst = 1 << 28, kStepLast = 1 << 29, kStepItemMask = (1 << 28) - 1;

// A supertile whose list was split: `count` partials starting at scratch slot `slot0`.
struct SplitRow {
    int32_t qtile, slot0, count, pad;
};

struct DeviceArrays {
    void *arena = nullptr;        // the one allocation every array below is a part of
    // row path
    int32_t *row_ptr = nullptr;   // [n_masks][S+1], offsets local to the mask
    int32_t *col_idx = nullptr;   // concatenated
    int64_t *col_off = nullptr;   // [n_masks] start of each mask inside col_idx
    // block path
    UEntry *uent = nullptr;
    int32_t *gidx = nullptr;                               // [n gathered tiles][64] key numbers
    uint64_t *kt_bitmap = nullptr;
    // work items at two grains (WorkLists below); [1] stays null when it would equal [0]
    Item *items[2] = {nullptr, nullptr};
    int32_t *item_off[2] = {nullptr, nullptr}, *item_cnt[2] = {nullptr, nullptr};      // [n_masks]
    SplitRow *split_rows[2] = {nullptr, nullptr};
    int32_t *split_off[2] = {nullptr, nullptr}, *split_cnt[2] = {nullptr, nullptr};    // [n_masks]
};

// The block kernel's work items for every mask of a plan: each 128-row group's list of steps, whole
// or cut into parts whose partial results are merged inside the same launch (see put_split_part in kernels.hip).
struct WorkLists {
    std::vector<Item> items;
    std::vector<int32_t> item_off, item_cnt;
    std::vector<SplitRow> split_rows;
    std::vector<int32_t> split_off, split_cnt;
    int max_items = 0, max_split_rows = 0, max_slots = 0;
};

}  // namespace smha

struct smha_plan {
    int S = 0, Sk = 0, Bm = 1, Hm = 1, block = 64;  // S queries, Sk keys
    smha_plan_opts_t opts{};
    int kernel = SMHA_KERNEL_BLOCK;
    bool has_row = false, has_block = false;
    std::vector<smha::MaskFormats> masks;
    double eq1_threshold = 0.0, model_row_us = 0.0, model_block_us = 0.0;
    double row_mean_nnz = 0.0;  // unmasked keys per query row, mean over masks

    // concatenated host copies of what the kernels read
    std::vector<int32_t> h_row_ptr, h_col_idx;
    std::vector<int64_t> h_col_off;
    std::vector<smha::UEntry> h_uent;
    std::vector<int32_t> h_gidx;  // gathered tiles: 64 key numbers each
    std::vector<uint64_t> h_kt_bitmap;
    // [0]: lists cut only where they are much longer than the typical one (throughput: many heads
    // keep the chip busy); [1]: every list cut to at most 16 steps (latency: with few heads the
    // longest list is the whole launch).  smha_forward picks by how many items the call has.
    smha::WorkLists lists[2];
    bool fine_differs = false;  // false: [1] is empty and [0] serves both
    // Tiles almost all full and lists long (dense causal and the like): at 128 columns such plans run the
    // block kernel's first form; all others its third form, whose waves skip at 16 rows x 32 keys.
    bool dense_long_lists = false;
    int64_t n_gathered = 0;

    int device = -1;  // -1: nothing uploaded
    int n_cu = 256;   // compute units of that device, rounded up to a multiple of 8
    smha::DeviceArrays dev;

    // What the block kernel needs for one call shape (batch, heads, head size): the work order (16
    // header words: start and length of each XCD's list; then (batch*head, item index) pairs) and
    // kCallSlots workspaces (partial results of split 128-row groups, then their arrival counters),
    // handed to successive calls in turn so that forwards in flight on different streams do not
    // share one.  Made by smha_plan_prepare (or by the first forward with that shape) and kept until
    // the plan is destroyed: a launch that is still queued, or a captured graph, never loses them.
    static constexpr int kCallSlots = 4;
    struct Prepared {
        int B = 0, H = 0, d = 0, lvl = 0, form = 1, per_xcd = 0, longest = 0;  // form: which block kernel the order is for
        int32_t *order = nullptr;
        int64_t step_words = 0, item_words = 0;  // second form: sizes of the step and item streams inside `order`
        size_t ws_bytes = 0, counters_at = 0;  // one workspace; byte offset of its counters
        void *ws[kCallSlots] = {nullptr, nullptr, nullptr, nullptr};
        unsigned next = 0;
    };
    mutable std::mutex prepared_mutex;
    mutable std::vector<Prepared *> prepared;
};

namespace smha {

// plan.cpp
smha_status_t finish_plan(smha_plan *p);      // selector, work lists, concatenation
// which workgroup of the block kernel takes which item, for B x H heads on `slots` workgroups per XCD
void build_work_order(const smha_plan *plan, int lvl, int B, int H, int slots, std::vector<int32_t> &table, int &per_xcd);
// bytes of one workspace for that call shape: partials first, then 4 counters per (batch*head, split group)
size_t workspace_bytes(const smha_plan *plan, int lvl, int B, int H, int d, size_t *counters_at);
// device.hip
smha_status_t upload_plan(smha_plan *p, int device_id);
void release_device(smha_plan *p);
// device byte masks [n_masks][S][S] -> host bit rows [n_masks][S][ceil(S/64)] (packed on the GPU)
smha_status_t pack_device_mask(const uint8_t *dev_mask, int n_masks, int Sq, int Sk, uint64_t *host_words);
// What the GPU reports about one 64x64 tile of a dense device mask: which of its 64 key columns
// any query uses, how many entries are set, how many of its sixteen 16x16 sub-tiles are not empty,
// and, for a partially filled tile, where its 64 bitmap words were put (slot within the mask).
struct TileInfo {
    uint64_t used;
    uint32_t cnt_v16;  // entries set (bits 0-15), non-empty 16x16 sub-tiles (bits 16-23)
    uint32_t slot;
};
// Classifies every tile of n_masks dense masks [Sq][Sk] on the GPU.  info: [mask][tile row][tile col];
// part_bits[mask]: 64 words per partially filled tile, in slot order.
smha_status_t classify_device_mask(const uint8_t *dev_mask, int n_masks, int Sq, int Sk,
                                   std::vector<TileInfo> &info, std::vector<std::vector<uint64_t>> &part_bits);
int current_device_or_negative();

}  // namespace smha
