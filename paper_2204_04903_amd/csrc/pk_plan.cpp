// Host-side plan: which fields share a packed operation, and where everything
// lives.  No HIP calls in this file, so the plan can be built and inspected on
// a machine without a GPU.
//
// Packing rule (Sec. III-B, D-Packing): fields are packed together when their
// embedding tables share the feature dimension, so the number of packed
// operations follows the number of distinct dimensions, not of fields (Fig. 7:
// three same-dimension tables are served by one set of packed operators).
#include "pk_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <atomic>
#include <new>

namespace pk {

static thread_local std::string g_error;

void set_error(const std::string& msg) { g_error = msg; }

pk_status fail(pk_status s, const std::string& msg)
{
    g_error = msg;
    return s;
}

static size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Occurrences per block iteration of the backward pass: small problems get small
// tiles so that the launch still has thousands of blocks.
int32_t pos_tile_for(int64_t nnz)
{
    int64_t t = nnz < (1 << 19) ? 128 : nnz < (2 << 20) ? 256 : 512;
    if (t < kPosTileMin) t = kPosTileMin;
    if (t > kPosTileMax) t = kPosTileMax;
    return (int32_t)t;
}

// the most slices all tables together (and any one table) can have in a partitioned call: the tables'
// shares of the occurrences are not known before the batch is
static void count_slices(const pk_plan* plan, int64_t nnz, int32_t log_max, int64_t* total, int32_t* most)
{
    int64_t each = 0, coarse = 0;
    *most = 0;
    for (const TableMeta& tm : plan->sort_tables) {
        const int32_t n = slice_count_max(tm.rows, nnz, kSliceOccLarge, log_max);
        each += n;
        coarse += ((int64_t)tm.rows + ((int64_t)1 << log_max) - 1) >> log_max;
        *most = std::max(*most, n);
    }
    // the slices asked for on account of occurrences number at most nnz / target + one per table
    *total = std::min<int64_t>(each, coarse + nnz / kSliceOccLarge + (int64_t)plan->sort_tables.size());
}

Layout make_layout(const pk_plan* plan, int32_t B, int64_t nnz)
{
    const size_t F = plan->fields.size(), P = plan->packs.size();
    const size_t n = (size_t)std::max<int64_t>(nnz, 1);
    Layout L{};
    int64_t slices = (int64_t)plan->small_slices.size();
    int32_t most = 0;
    L.small = nnz < kSmallNnz && slices <= kSmallSlicesMax && !(plan->opts.debug & 2);
    L.log_max = kSliceLogMax;
    if (!L.small) {
        L.log_max = kSliceLogFine;
        for (const TableMeta& tm : plan->sort_tables)
            if ((int64_t)tm.rows > kFineRowsMax) L.log_max = kSliceLogMax;
        count_slices(plan, nnz, L.log_max, &slices, &most);
    }
    L.n_slices = (int32_t)slices;
    L.max_table_slices = most;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    L.clear_begin    = off;
    L.state          = take(P * sizeof(PackState));
    L.slice_total    = take(L.small ? 0 : (size_t)slices * 4);
    L.slice_nu       = take(L.small ? 0 : (size_t)slices * 4);
    L.big_list       = take(L.small ? 0 : (size_t)(256 + 64) * 4);          // listed slices, then their count
    L.clear_bytes    = off - L.clear_begin;
    L.slice_cursor   = take(L.small ? 0 : (size_t)slices * 4);
    L.slice_usum     = take(L.small ? 0 : (size_t)slices * 4);
    L.slice_info     = take(L.small ? 0 : (size_t)slices * sizeof(SliceInfo));
    L.tgeom          = take(L.small ? 0 : plan->sort_tables.size() * sizeof(TableCut));
    L.fscan          = take(L.small ? 0 : (3 * F + 3) * 4);          // the field scan of the batch, with its verdict
    // bags per tile of the keys and scatter kernels: about 16 K occurrences, 32 to 1024 bags (a mix of short
    // and very long bags counts as long)
    const int64_t n_bags = (int64_t)F * B;
    const int64_t avg_len = std::max<int64_t>(nnz / std::max<int64_t>(n_bags, 1), 1);
    L.bags_per_tile  = avg_len >= 48 ? 32 : avg_len >= 32 ? 128 : avg_len >= 12 ? 512 : 1024;
    // the keys kernel's counts per (tile, slice of the tile's table), so that the scatter kernel need not count
    // again; only while that table stays small
    const int64_t n_tiles = (int64_t)F * ((B + L.bags_per_tile - 1) / L.bags_per_tile);
    L.tile_hist_stride = (!L.small && n_tiles * (int64_t)most <= ((int64_t)8 << 20)) ? most : 0;
    L.tile_hist      = take((size_t)n_tiles * (size_t)L.tile_hist_stride * 4);
    L.packed_offsets = take((F * (size_t)B + P) * 4);
    L.keys           = take(n * 4);
    L.inverse        = take(n * 4);
    L.seg_ent        = take(n * (plan->any_mean ? 8 : 4));
    L.pos_tile       = pos_tile_for(nnz);
    const size_t tile_cap = n / L.pos_tile + P + 2;      // backward tiles of all packs
    L.tile_hdr       = take(tile_cap * 16);
    L.unique         = take(n * 4);
    L.seg            = take((n + P + 1) * 4);
    L.dmax           = plan->dmax;
    L.ghot           = take(tile_cap * (size_t)plan->dmax * 8);
    L.rec            = take(L.small ? 0 : n * 8);
    L.bitmap         = take(L.small ? 0 : (size_t)plan->bitmap_words * 4);
    L.total = off;
    return L;
}

}  // namespace pk

using namespace pk;

extern "C" {

const char* pk_last_error(void) { return g_error.c_str(); }

pk_status pk_plan_create(const pk_table_desc* tables, int32_t n_tables, const pk_field_desc* fields,
                         int32_t n_fields, const pk_plan_opts* opts, pk_plan** out)
{
    if (!out) return fail(PK_EINVAL, "pk_plan_create: out is NULL");
    *out = nullptr;
    if (!tables || !fields) return fail(PK_EINVAL, "pk_plan_create: tables or fields is NULL");
    if (n_tables <= 0 || n_fields <= 0) return fail(PK_EINVAL, "pk_plan_create: n_tables and n_fields must be positive");
    for (int32_t t = 0; t < n_tables; ++t) {
        if (tables[t].rows <= 0 || tables[t].dim <= 0)
            return fail(PK_EINVAL, "pk_plan_create: table " + std::to_string(t) + " has non-positive rows or dim");
        if (tables[t].dtype != PK_F32 && tables[t].dtype != PK_BF16)
            return fail(PK_EINVAL, "pk_plan_create: table " + std::to_string(t) + " has an unknown dtype");
        if (tables[t].dim > 256)
            return fail(PK_EOVERFLOW, "pk_plan_create: table " + std::to_string(t) + " has dim > 256");
    }
    for (int32_t f = 0; f < n_fields; ++f) {
        if (fields[f].table < 0 || fields[f].table >= n_tables)
            return fail(PK_EINVAL, "pk_plan_create: field " + std::to_string(f) + " names a table out of range");
        if (fields[f].pool != PK_SUM && fields[f].pool != PK_MEAN)
            return fail(PK_EINVAL, "pk_plan_create: field " + std::to_string(f) + " has an unknown pooling mode");
    }
    if (n_fields > 4096 || n_tables > 4096)
        return fail(PK_EOVERFLOW, "pk_plan_create: at most 4096 fields and 4096 tables (their metadata is staged in LDS)");
    for (int32_t t = 0; t < n_tables; ++t)
        if (tables[t].rows > ((int64_t)kTableSlicesMax << kSliceLogMax))
            return fail(PK_EOVERFLOW, "pk_plan_create: table " + std::to_string(t) + " has more than 2^30 rows");
    if (opts && (opts->max_batch < 0 || opts->max_nnz < 0 || opts->max_shards < 0))
        return fail(PK_EINVAL, "pk_plan_create: negative option");
    if (opts && (opts->interleave_groups < 0 || opts->interleave_groups > 8))
        return fail(PK_EINVAL, "pk_plan_create: interleave_groups must be 0 (automatic) to 8");
    if (opts && (opts->debug < 0 || opts->debug > 3))
        return fail(PK_EINVAL, "pk_plan_create: unknown debug bits");
    if (opts && opts->field_volume)
        for (int32_t f = 0; f < n_fields; ++f)
            if (!(opts->field_volume[f] >= 0.0))
                return fail(PK_EINVAL, "pk_plan_create: field_volume[" + std::to_string(f) + "] is negative or not a number");

    pk_plan* pl = new (std::nothrow) pk_plan();
    if (!pl) return fail(PK_ENOMEM, "pk_plan_create: out of host memory");
    static std::atomic<uint64_t> next_serial{1};
    pl->serial = next_serial.fetch_add(1);
    pl->tables.assign(tables, tables + n_tables);
    pl->fields.assign(fields, fields + n_fields);
    if (opts) pl->opts = *opts;
    pl->opts.field_volume = nullptr;   // not retained

    // distinct (dim, dtype) pairs, ascending
    std::vector<std::pair<int32_t, int32_t>> keys;
    for (auto& t : pl->tables) keys.emplace_back(t.dim, t.dtype);
    std::sort(keys.begin(), keys.end());
    keys.erase(std::unique(keys.begin(), keys.end()), keys.end());
    std::vector<std::vector<int32_t>> group(keys.size());            // tables per pair, ascending table index
    for (int32_t t = 0; t < n_tables; ++t) {
        auto it = std::lower_bound(keys.begin(), keys.end(), std::make_pair(tables[t].dim, tables[t].dtype));
        group[it - keys.begin()].push_back(t);
    }
    // Eq. 1 (Sec. III-B): volume of a packed operation = floats it gathers = sum over its
    // tables of dim x occurrences.  A pack whose volume is above the average is split into
    // round(volume / smallest volume) shards (the paper's example: dim 8 -> one operation,
    // dim 32 -> four), at most max_shards and at most one per table; its tables are dealt to
    // the shards in turn.
    std::vector<int32_t> n_shards(keys.size(), 1);
    if (opts && opts->max_shards > 1) {
        std::vector<double> occ(n_tables, 0.0), vol(keys.size(), 0.0);
        for (int32_t f = 0; f < n_fields; ++f) occ[fields[f].table] += opts->field_volume ? opts->field_volume[f] : 1.0;
        double vmin = 0.0, vsum = 0.0;
        int n_vol = 0;
        for (size_t g = 0; g < keys.size(); ++g) {
            for (int32_t t : group[g]) vol[g] += (double)tables[t].dim * occ[t];
            if (vol[g] > 0.0 && (vmin == 0.0 || vol[g] < vmin)) vmin = vol[g];
            if (vol[g] > 0.0) { vsum += vol[g]; ++n_vol; }
        }
        const double vmean = n_vol > 0 ? vsum / n_vol : 0.0;
        for (size_t g = 0; g < keys.size(); ++g) {
            int64_t s = (vmin > 0.0 && vol[g] > vmean) ? (int64_t)std::floor(vol[g] / vmin + 0.5) : 1;
            s = std::min<int64_t>(s, opts->max_shards);
            s = std::min<int64_t>(s, (int64_t)group[g].size());
            n_shards[g] = (int32_t)std::max<int64_t>(s, 1);
        }
    }
    pl->table_pack.resize(n_tables);
    pl->table_base.resize(n_tables);
    for (size_t g = 0; g < keys.size(); ++g) {
        const size_t p0 = pl->packs.size();
        pl->packs.resize(p0 + n_shards[g]);
        for (int32_t s = 0; s < n_shards[g]; ++s) { pl->packs[p0 + s].dim = keys[g].first; pl->packs[p0 + s].dtype = keys[g].second; }
        for (size_t i = 0; i < group[g].size(); ++i) {
            const int32_t t = group[g][i];
            const int32_t p = (int32_t)(p0 + i % n_shards[g]);
            pl->table_pack[t] = p;
            pl->table_base[t] = pl->packs[p].rows;
            pl->packs[p].rows += tables[t].rows;
            pl->packs[p].tables.push_back(t);
        }
    }
    for (auto& pk_ : pl->packs)
        if (pk_.rows >= ((int64_t)1 << 32)) {
            delete pl;
            return fail(PK_EOVERFLOW, "pk_plan_create: a pack has 2^32 or more rows");
        }
    pl->field_pack.resize(n_fields);
    pl->field_slot.resize(n_fields);
    pl->field_col.resize(n_fields);
    int64_t col = 0;
    for (int32_t f = 0; f < n_fields; ++f) {
        int32_t p = pl->table_pack[fields[f].table];
        pl->field_pack[f] = p;
        pl->field_slot[f] = (int32_t)pl->packs[p].fields.size();
        pl->packs[p].fields.push_back(f);
        pl->field_col[f] = col;
        col += tables[fields[f].table].dim;
        if (fields[f].pool == PK_MEAN) { pl->packs[p].has_mean = true; pl->any_mean = true; }
    }
    pl->out_dim = col;
    if (col >= ((int64_t)1 << 31)) {
        delete pl;
        return fail(PK_EOVERFLOW, "pk_plan_create: out_dim does not fit 31 bits");
    }
    int32_t slot0 = 0;
    for (auto& pk_ : pl->packs) {
        pk_.first_slot = slot0;
        slot0 += (int32_t)pk_.fields.size();
        for (int32_t f : pk_.fields) pl->slot_field.push_back(f);
    }
    // tables that some field reads, in (pack, first key) order, with their fields; each gets a
    // bitmap region of its own, padded to whole largest slices so that its place does not depend
    // on how finely a call cuts the table
    for (size_t p = 0; p < pl->packs.size(); ++p) {
        pl->packs[p].first_stable = (int32_t)pl->sort_tables.size();
        for (int32_t t : pl->packs[p].tables) {                // ascending table index = ascending first key
            TableMeta tm{};
            tm.pack = (int32_t)p;
            tm.key_lo = (uint32_t)pl->table_base[t];
            tm.rows = (uint32_t)tables[t].rows;
            tm.field_begin = (int32_t)pl->table_fields.size();
            for (int32_t f = 0; f < n_fields; ++f)
                if (fields[f].table == t) pl->table_fields.push_back(f);
            tm.field_end = (int32_t)pl->table_fields.size();
            if (tm.field_end == tm.field_begin) continue;
            tm.word_base = (uint32_t)pl->bitmap_words;
            // three bitmap words and a rank sample to every 16 bytes; the table's words padded to whole largest slices
            const int64_t table_words = ((tables[t].rows + ((int64_t)1 << kSliceLogMax) - 1) >> kSliceLogMax) * kSliceWordsMax;
            pl->bitmap_words += ((table_words + 2) / 3 + 1) * 4;
            pl->max_table_fields = std::max(pl->max_table_fields, tm.field_end - tm.field_begin);
            pl->sort_tables.push_back(tm);
        }
        pl->packs[p].n_stables = (int32_t)pl->sort_tables.size() - pl->packs[p].first_stable;
    }
    if (pl->bitmap_words >= ((int64_t)1 << 32)) {
        delete pl;
        return fail(PK_EOVERFLOW, "pk_plan_create: the tables' bitmaps do not fit 2^32 words");
    }
    // the cut of the one-launch forward pass
    for (size_t p = 0; p < pl->packs.size(); ++p) {
        const Pack& k = pl->packs[p];
        const int32_t pack_first = (int32_t)pl->small_slices.size();
        for (int32_t i = 0; i < k.n_stables; ++i) {
            const TableMeta& tm = pl->sort_tables[k.first_stable + i];
            const SliceGeom g = slice_geom_small(tm.rows, (int32_t)pl->sort_tables.size());
            for (int32_t j = 0; j < g.n; ++j) {
                SmallSlice ss{};
                ss.table = k.first_stable + i; ss.idx = j; ss.log_keys = g.log_keys; ss.n_table_slices = g.n;
                ss.pack_first = pack_first; ss.is_last = (i + 1 == k.n_stables && j + 1 == g.n) ? 1 : 0;
                ss.pack = (int32_t)p; ss.field_begin = tm.field_begin; ss.field_end = tm.field_end;
                ss.key_lo = tm.key_lo; ss.rows = tm.rows;
                pl->small_slices.push_back(ss);
            }
        }
    }
    for (auto& pk_ : pl->packs) pl->dmax = std::max(pl->dmax, pk_.dim);
    *out = pl;
    return PK_OK;
}

void pk_plan_destroy(pk_plan* plan)
{
    if (!plan) return;
    if (plan->device_state) destroy_device_state(plan);
    delete plan;
}

int32_t pk_plan_num_packs(const pk_plan* plan) { return plan ? (int32_t)plan->packs.size() : -1; }

pk_status pk_plan_pack_info(const pk_plan* plan, int32_t p, int32_t* dim, int32_t* dtype, int64_t* total_rows,
                            int32_t* n_fields, int32_t* n_tables, int32_t* key_bytes)
{
    if (!plan) return fail(PK_EINVAL, "pk_plan_pack_info: plan is NULL");
    if (p < 0 || p >= (int32_t)plan->packs.size()) return fail(PK_EINVAL, "pk_plan_pack_info: pack out of range");
    const Pack& k = plan->packs[p];
    if (dim) *dim = k.dim;
    if (dtype) *dtype = k.dtype;
    if (total_rows) *total_rows = k.rows;
    if (n_fields) *n_fields = (int32_t)k.fields.size();
    if (n_tables) *n_tables = (int32_t)k.tables.size();
    if (key_bytes) *key_bytes = 4;
    return PK_OK;
}

pk_status pk_plan_pack_fields(const pk_plan* plan, int32_t p, int32_t* fields_out)
{
    if (!plan || !fields_out) return fail(PK_EINVAL, "pk_plan_pack_fields: NULL argument");
    if (p < 0 || p >= (int32_t)plan->packs.size()) return fail(PK_EINVAL, "pk_plan_pack_fields: pack out of range");
    std::copy(plan->packs[p].fields.begin(), plan->packs[p].fields.end(), fields_out);
    return PK_OK;
}

pk_status pk_plan_table_slot(const pk_plan* plan, int32_t table, int32_t* pack, int64_t* base_row)
{
    if (!plan) return fail(PK_EINVAL, "pk_plan_table_slot: plan is NULL");
    if (table < 0 || table >= (int32_t)plan->tables.size()) return fail(PK_EINVAL, "pk_plan_table_slot: table out of range");
    if (pack) *pack = plan->table_pack[table];
    if (base_row) *base_row = plan->table_base[table];
    return PK_OK;
}

pk_status pk_plan_field_col(const pk_plan* plan, int32_t field, int64_t* col_offset)
{
    if (!plan) return fail(PK_EINVAL, "pk_plan_field_col: plan is NULL");
    if (field < 0 || field >= (int32_t)plan->fields.size()) return fail(PK_EINVAL, "pk_plan_field_col: field out of range");
    if (col_offset) *col_offset = plan->field_col[field];
    return PK_OK;
}

int64_t pk_plan_out_dim(const pk_plan* plan) { return plan ? plan->out_dim : -1; }

size_t pk_workspace_bytes(const pk_plan* plan, int32_t B, int64_t nnz)
{
    if (!plan) { set_error("pk_workspace_bytes: plan is NULL"); return 0; }
    if (B <= 0 || nnz < 0) { set_error("pk_workspace_bytes: B must be positive and nnz non-negative"); return 0; }
    if (nnz >= ((int64_t)1 << 31)) { set_error("pk_workspace_bytes: nnz must be below 2^31"); return 0; }
    return make_layout(plan, B, nnz).total;
}

// Sec. III-C, Eq. 2: BS_micro = min over operators of RBound / RInstance, for the workspace
// (RInstance from the layout at the observed occurrences per sample) and the activations.
int32_t pk_micro_batch_size(const pk_plan* plan, int32_t B, int64_t nnz, size_t ws_bound_bytes, size_t act_bound_bytes)
{
    if (!plan) { set_error("pk_micro_batch_size: plan is NULL"); return -1; }
    if (B <= 0 || nnz < 0 || nnz >= ((int64_t)1 << 31)) {
        set_error("pk_micro_batch_size: B must be positive and nnz in [0, 2^31)");
        return -1;
    }
    auto nnz_of = [&](int64_t b) { return (nnz * b + B - 1) / B; };
    auto ws_of = [&](int64_t b) { return make_layout(plan, (int32_t)b, nnz_of(b)).total; };
    int64_t bs = B;
    if (ws_bound_bytes) {
        const size_t fixed = make_layout(plan, 1, 0).total;          // bitmap, rank samples, descriptors of an empty batch
        if (ws_bound_bytes <= fixed) return 0;
        const double r_instance = std::max(1.0, ((double)ws_of(B) - (double)fixed) / (double)B);
        int64_t b = (int64_t)std::min<double>((double)B, (double)(ws_bound_bytes - fixed) / r_instance);
        // the layout rounds its arrays up, so the ratio can be off by a few samples: settle on
        // the largest size whose workspace really fits
        while (b < B && ws_of(b + 1) <= ws_bound_bytes) ++b;
        while (b > 0 && ws_of(b) > ws_bound_bytes) --b;
        bs = std::min(bs, b);
    }
    if (act_bound_bytes) bs = std::min<int64_t>(bs, (int64_t)(act_bound_bytes / (size_t)(8 * std::max<int64_t>(plan->out_dim, 1))));
    if (bs <= 0) return 0;
    const int64_t M = (B + bs - 1) / bs;
    return (int32_t)((B + M - 1) / M);
}

}  // extern "C"
