// Internal declarations shared by the host plan (pk_plan.cpp) and the device
// code (pk_device.hip).  Not part of the C ABI.
#pragma once

#include <cstdint>
#include <cstddef>
#include <string>
#include <vector>

#include "pk.h"

namespace pk {

constexpr int kColdMax   = 8;      // keys with at most this many occurrences: one lane group per key
constexpr int kWarmMax   = 256;    // up to this many: one wavefront per key; above: split, partial sums
constexpr int kTileWords = 2048;   // bitmap words scanned by one block (256 threads x 8 words)
constexpr int kRankWords = 8;      // one rank sample per 8 words (256 keys)
constexpr int kPosTileMax = 512;   // occurrences handled per block iteration in the backward pass (upper end)
constexpr int kPosTileMin = 64;
constexpr int kMarkWords = 16384;  // bitmap words (512K keys, 64 KB of LDS) owned by one block of the mark kernel
constexpr int kSortCap   = 16384;  // distinct keys whose occurrences one block of the sort kernel groups in LDS
constexpr size_t kAlign = 256;

// Per field, device side (indexed by field index).
struct FieldMeta {
    uint32_t base_row;   // first row of the field's table inside its pack
    uint32_t rows;       // rows of the field's table
    int32_t  col;        // first output column of the field
    int32_t  pack;
    int32_t  slot;       // rank of the field among its pack's fields
    int32_t  pool;       // PK_SUM / PK_MEAN
};

// Per pack, device side, static.
struct PackMeta {
    int32_t dim;
    int32_t dtype;
    int32_t n_fields;
    int32_t first_slot;      // index of the pack's slot 0 in the slot-ordered arrays
    int32_t has_mean;
    int32_t first_tile;      // first bitmap tile (of kTileWords words) of the pack
    int32_t n_tiles;
    int32_t first_stable;    // index of the pack's first table in the (pack, key) ordered table list
};

// A slice of a pack's key space (kMarkWords bitmap words) and the fields whose
// tables overlap it; static, device side.
struct MarkItem {
    int32_t pack;
    uint32_t key_lo;         // first key of the slice (multiple of 32)
    int32_t n_words;         // bitmap words of the slice
    int32_t field_begin;     // range in the item field list
    int32_t field_end;
    int32_t pad[3];
};

// A table that at least one field reads, and those fields; static, device side,
// listed in (pack, first key) order.
struct TableMeta {
    int32_t pack;
    uint32_t key_lo;         // first key of the table inside its pack
    uint32_t rows;
    int32_t field_begin;     // range in the table field list
    int32_t field_end;
    int32_t pad[3];
};

// Per pack, device side, rewritten by every forward call.
struct PackState {
    int32_t nnz;        // occurrences in the pack
    int32_t start;      // position of the pack's first occurrence in the packed order
    int32_t n_unique;
    int32_t error;      // only pack 0's word is used
    int32_t pad[4];
};

struct Pack {
    int32_t dim = 0, dtype = 0;
    int64_t rows = 0;
    bool has_mean = false;
    std::vector<int32_t> tables;
    std::vector<int32_t> fields;
    int32_t first_slot = 0;
    int32_t first_tile = 0, n_tiles = 0;
    int32_t first_stable = 0;
};

// Byte offsets of the workspace's arrays for one (plan, B, nnz).
struct Layout {
    size_t state, fb, delta, packed_offsets, keys, inverse, bagref, baglen, seg_ent, tile_hdr,
           unique, seg, ghot, bitmap, tile_desc, sort_desc, rank, total;
    size_t clear_bytes;          // scan descriptors, contiguous from `tile_desc`
    int64_t n_tiles_total;
    int32_t dmax;
    int32_t pos_tile;            // occurrences per backward tile for this nnz
};

}  // namespace pk

struct pk_plan {
    std::vector<pk_table_desc> tables;
    std::vector<pk_field_desc> fields;
    pk_plan_opts opts{};
    std::vector<pk::Pack> packs;
    std::vector<int32_t> table_pack;
    std::vector<int64_t> table_base;
    std::vector<int32_t> field_pack, field_slot;
    std::vector<int64_t> field_col;
    std::vector<int32_t> slot_field;      // fields in (pack, slot) order
    std::vector<pk::MarkItem> mark_items;
    std::vector<int32_t> mark_fields;     // per item: the fields whose table overlaps the slice
    std::vector<pk::TableMeta> sort_tables;   // tables with fields, in (pack, first key) order
    std::vector<int32_t> table_fields;        // per entry of sort_tables: the fields that read it
    int64_t out_dim = 0;
    bool any_mean = false;
    int32_t n_tiles_total = 0;
    int32_t dmax = 0;
    void* device_state = nullptr;         // owned by pk_device.hip (metadata upload, events)
};

namespace pk {
void set_error(const std::string& msg);
pk_status fail(pk_status s, const std::string& msg);
Layout make_layout(const pk_plan* plan, int32_t B, int64_t nnz);
int32_t pos_tile_for(int64_t nnz);
void destroy_device_state(pk_plan* plan);   // defined in pk_device.hip
}  // namespace pk
