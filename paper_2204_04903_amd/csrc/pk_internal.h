// Internal declarations shared by the host plan (pk_plan.cpp) and the device
// code (pk_device.hip).  Not part of the C ABI.
#pragma once

#include <cstdint>
#include <cstddef>
#include <algorithm>
#include <string>
#include <vector>

#include "pk.h"

namespace pk {

constexpr int kColdMax   = 8;      // keys with at most this many occurrences: one lane group per key
constexpr int kWarmMax   = 256;    // up to this many: one wavefront per key; above: split, partial sums
constexpr int kRankWords = 3;      // in memory a rank sample follows every 3 bitmap words (96 keys): a lookup is one 16-byte read
constexpr int kPosTileMax = 512;   // occurrences handled per block iteration in the backward pass (upper end)
constexpr int kPosTileMin = 64;
constexpr size_t kAlign = 256;

// The dedup cuts every table's key range into slices of 2^k keys; one block owns a slice and keeps
// the slice's bitmap, its popcount prefix and the occurrence counters of its distinct keys in LDS.
// Two shapes of slice block: 1024 threads for slices of up to 128 K keys (small batches, where a
// block scans its table's IDs itself, and large batches with tables too long for the other shape),
// and 256 threads for slices of up to 32 K keys (large batches: many small blocks hide the latency
// of the few dependent memory accesses a slice makes).
constexpr int kSliceLogMin = 10;           // 1 K keys
constexpr int kSliceLogMax = 17;           // 128 K keys: 4096 bitmap words
constexpr int kSliceLogFine = 15;          // 32 K keys: 1024 bitmap words
constexpr int kSliceWordsMax = 1 << (kSliceLogMax - 5);
constexpr int kSliceOccLarge = 2048;       // occurrences per slice aimed at when the occurrences are partitioned
constexpr int64_t kSmallNnz = 1 << 19;     // below this many occurrences the forward pass is one launch
constexpr int kSmallSlicesMax = 4096;      // ... if it has no more slices than this (descriptors the library owns)
constexpr int kTableSlicesMax = 8192;      // slices per table (their counters are staged in LDS): rows <= 2^30
constexpr int64_t kFineRowsMax = (int64_t)4096 << kSliceLogFine;   // longest table the 32 K-key shape is used with

#if defined(__HIPCC__)
#define PK_HD __host__ __device__
#else
#define PK_HD
#endif

// Slices of one table for a partitioned call: 2^log_keys keys each, n of them.  The aim is `target`
// occurrences per slice, given how many occurrences the table's fields have in THIS batch (the
// offsets say so: a layer's fields differ widely in length, Sec. II-B).  The kernels derive the cut
// from the offsets; the host only needs the most slices a batch can give (slice_count_max).
struct SliceGeom { int32_t log_keys; int32_t n; };
constexpr int kSliceWantMax = 1024;        // slices asked for a table on account of its occurrences
PK_HD inline SliceGeom slice_geom(uint32_t rows, int64_t occ, int32_t target, int32_t log_max)
{
    int64_t want = (occ + target - 1) / target;
    if (want < 1) want = 1;
    if (want > kSliceWantMax) want = kSliceWantMax;
    const int64_t per = ((int64_t)rows + want - 1) / want;
    int lg = kSliceLogMin;
    while (lg < log_max && ((int64_t)1 << lg) < per) ++lg;
    SliceGeom g;
    g.log_keys = lg;
    g.n = (int32_t)(((int64_t)rows + ((int64_t)1 << lg) - 1) >> lg);
    return g;
}
// The most slices slice_geom gives a table of a batch with nnz occurrences: either the slices are as
// large as they may be (2^log_max keys), or there are at most as many as were asked for.
inline int32_t slice_count_max(uint32_t rows, int64_t nnz, int32_t target, int32_t log_max)
{
    const int64_t coarse = ((int64_t)rows + ((int64_t)1 << log_max) - 1) >> log_max;
    const int64_t fine = ((int64_t)rows + ((int64_t)1 << kSliceLogMin) - 1) >> kSliceLogMin;
    const int64_t want = std::min<int64_t>(kSliceWantMax, nnz / target + 1);
    return (int32_t)std::min(fine, std::max(coarse, want));
}

// Small batches: the cut depends on the plan alone (up to 8 slices per table, fewer when there are
// many tables), so the list of slices is made once, on the host.
inline SliceGeom slice_geom_small(int64_t rows, int32_t n_tables)
{
    int64_t want = 1024 / (n_tables > 0 ? n_tables : 1);
    if (want > 8) want = 8;
    if (want < 1) want = 1;
    const int64_t per = (rows + want - 1) / want;
    int lg = kSliceLogMin;
    while (lg < kSliceLogMax && ((int64_t)1 << lg) < per) ++lg;
    SliceGeom g;
    g.log_keys = lg;
    g.n = (int32_t)((rows + ((int64_t)1 << lg) - 1) >> lg);
    return g;
}

// One slice of the small-batch cut; static, device side, in (pack, table, slice) order.
struct SmallSlice {
    int32_t table;           // index in the table list
    int32_t idx;             // slice of the table
    int32_t log_keys;
    int32_t n_table_slices;
    int32_t pack_first;      // the pack's first slice
    int32_t is_last;         // the pack's last slice
    int32_t pack;
    int32_t field_begin, field_end;   // the table's fields in the table field list
    uint32_t key_lo, rows;   // the table's first key inside its pack, its rows
    int32_t pad;
};

// Per field, device side (indexed by field index).
struct FieldMeta {
    uint32_t base_row;   // first row of the field's table inside its pack
    uint32_t rows;       // rows of the field's table
    int32_t  col;        // first output column of the field
    int32_t  pack;
    int32_t  slot;       // rank of the field among its pack's fields
    int32_t  pool;       // PK_SUM / PK_MEAN
    int32_t  stable;     // the field's table in the (pack, first key) ordered table list
    int32_t  pad;
    uint64_t magic;      // floor((2^64 - 1) / rows): folds an ID without a division
};

// Per pack, device side, static.
struct PackMeta {
    int32_t dim;
    int32_t dtype;
    int32_t n_fields;
    int32_t first_slot;      // index of the pack's slot 0 in the slot-ordered arrays
    int32_t has_mean;
    int32_t first_stable;    // index of the pack's first table in the (pack, key) ordered table list
    int32_t n_stables;       // tables of the pack that some field reads
    int32_t pad;
};

// A table that at least one field reads, and those fields; static, device side,
// listed in (pack, first key) order.
struct TableMeta {
    int32_t pack;
    uint32_t key_lo;         // first key of the table inside its pack
    uint32_t rows;
    int32_t field_begin;     // range in the table field list
    int32_t field_end;
    uint32_t word_base;      // first word of the table's bitmap and rank samples (a multiple of 4)
    int32_t pad[2];
};

// What the inverse kernel needs of a (pack, slot): static, device side, in slot order.
struct SlotMeta {
    uint32_t key_lo;         // first key of the slot's table inside its pack
    uint32_t word_base;      // where the table's bitmap starts
    uint32_t rows;           // rows of the table
    int32_t  pack;
};

// The cut of one table for the batch at hand (written by the keys kernel, read by the kernels after it).
struct TableCut {
    int32_t log_keys;        // 2^log_keys keys per slice
    int32_t n;               // slices of the table
    int32_t first;           // the table's first slice (slices are numbered over all packs)
    int32_t occ;             // occurrences of the table's fields in this batch
};

// One slice as the partitioned path hands it to the slice kernel (written by the scan kernel).
struct SliceInfo {
    int32_t table;           // index in the table list
    int32_t idx;             // slice of the table
    int32_t start;           // position of the slice's first record in the records (all packs)
    int32_t count;           // records
};

// Per pack, device side, rewritten by every forward call.
struct PackState {
    int32_t nnz;        // occurrences in the pack
    int32_t start;      // position of the pack's first occurrence in the packed order
    int32_t n_unique;
    int32_t error;      // bit 0: offsets rejected; bit 1: a scan waited too long
    int32_t first_slice;    // partitioned path: the pack's first slice
    int32_t pad[3];
};

struct Pack {
    int32_t dim = 0, dtype = 0;
    int64_t rows = 0;
    bool has_mean = false;
    std::vector<int32_t> tables;
    std::vector<int32_t> fields;
    int32_t first_slot = 0;
    int32_t first_stable = 0, n_stables = 0;
};

// Byte offsets of the workspace's arrays for one (plan, B, nnz).
struct Layout {
    size_t state, packed_offsets, keys, inverse, seg_ent, tile_hdr, unique, seg, ghot,
           clear_begin, slice_total, slice_nu, big_list, slice_cursor, slice_usum, slice_info, tgeom, fscan, tile_hist, rec, bitmap, total;
    size_t clear_bytes;          // what the partitioned path clears before its first kernel: per-pack state,
                                 // slice totals and distinct-key counts, contiguous from `clear_begin`
    int32_t n_slices;            // slices of all tables for this call
    int32_t max_table_slices;    // most slices any table has
    int32_t log_max;             // partitioned path: largest slice (log2 of its keys) of this call
    int32_t dmax;
    int32_t pos_tile;            // occurrences per backward tile for this nnz
    int32_t bags_per_tile;       // bags per tile of the keys and scatter kernels
    int32_t tile_hist_stride;    // entries per tile of the stored per-slice counts (0: not stored, the scatter kernel counts again)
    bool small;                  // the forward pass's dedup is one launch (every slice block scans its table's IDs)
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
    std::vector<pk::TableMeta> sort_tables;   // tables with fields, in (pack, first key) order
    std::vector<int32_t> table_fields;        // per entry of sort_tables: the fields that read it
    std::vector<pk::SmallSlice> small_slices; // the cut used by the one-launch forward pass
    int64_t out_dim = 0;
    bool any_mean = false;
    int64_t bitmap_words = 0;             // all tables' bitmaps with their rank samples
    int32_t max_table_fields = 0;         // most fields reading one table
    int32_t dmax = 0;
    void* device_state = nullptr;         // owned by pk_device.hip (metadata upload, events)
    uint64_t serial = 0;                  // distinguishes plans, also when one is created where another was freed
};

namespace pk {
void set_error(const std::string& msg);
pk_status fail(pk_status s, const std::string& msg);
Layout make_layout(const pk_plan* plan, int32_t B, int64_t nnz);
int32_t pos_tile_for(int64_t nnz);
void destroy_device_state(pk_plan* plan);   // defined in pk_device.hip
}  // namespace pk
