// Host side: per-plan device state, profiling brackets, launch helpers and the per-pack template dispatch.
// Part of pk_device.hip: included there, in this order, inside its anonymous namespace.

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct DeviceState {
    int device = -1;
    int n_cus = 256;                      // compute units of the device
    void* blob = nullptr;
    FieldMeta* fmeta = nullptr;
    PackMeta* pmeta = nullptr;
    int32_t* slot_field = nullptr;
    uint64_t* small_desc = nullptr;       // look-back descriptors of the one-launch forward pass (zero between calls)
    int32_t* small_done = nullptr;        // ... and its count of blocks that are through their look-back
    SmallSlice* small_slices = nullptr;   // the cut of the one-launch forward pass
    TableField* tfields = nullptr;        // the table field list with what the slice blocks need of a field
    TableMeta* sort_tables = nullptr;
    int32_t* table_fields = nullptr;
    SlotMeta* slot_meta = nullptr;        // per (pack, slot): what the inverse kernel needs of the slot's table
    std::mutex mu;
    // Side streams: packs (and the pooling of a pack vs the dedup chain) are independent
    // pieces of memory-bound work; running them side by side hides launch gaps and
    // latency tails (the interleaving of packed operations of Sec. III-C, on one GPU).
    static constexpr int kSide = 8;
    hipStream_t side[kSide] = {};
    hipEvent_t ev_fork = nullptr;
    hipEvent_t ev_join[kSide] = {};
    bool overlap = true;
    std::vector<int64_t> hh_n_hot;        // HybridHash: rows in each pack's Hot-storage
    // profiling
    bool prof_on = false;
    std::vector<hipEvent_t> events;
    size_t events_used = 0;
    struct Rec { const char* name; size_t e0; };
    std::vector<Rec> recs;
};

std::string hip_msg(const char* what, hipError_t e)
{
    return std::string(what) + ": " + hipGetErrorString(e);
}

// The plan's device-side metadata as host arrays, and where each array goes inside one block of
// device memory (256-byte aligned pieces): look-back descriptors and their counter first.
struct MetaImage {
    std::vector<FieldMeta> fm;
    std::vector<PackMeta> pmv;
    std::vector<TableField> tfi;
    std::vector<SlotMeta> slm;
    size_t o_desc, o_done, o_fm, o_pm, o_slot, o_ss, o_tfi, o_tab, o_tf, o_slm, total;
};

void build_meta_image(const pk_plan* plan, MetaImage* mi)
{
    const size_t F = plan->fields.size(), P = plan->packs.size();
    mi->fm.resize(F);
    for (size_t f = 0; f < F; ++f) {
        const int32_t t = plan->fields[f].table;
        mi->fm[f].base_row = (uint32_t)plan->table_base[t];
        mi->fm[f].rows = (uint32_t)plan->tables[t].rows;
        mi->fm[f].col = (int32_t)plan->field_col[f];
        mi->fm[f].pack = plan->field_pack[f];
        mi->fm[f].slot = plan->field_slot[f];
        mi->fm[f].pool = plan->fields[f].pool;
        mi->fm[f].stable = -1;
        mi->fm[f].pad = 0;
        mi->fm[f].magic = ~(uint64_t)0 / (uint64_t)plan->tables[t].rows;
    }
    for (size_t i = 0; i < plan->sort_tables.size(); ++i)
        for (int32_t j = plan->sort_tables[i].field_begin; j < plan->sort_tables[i].field_end; ++j)
            mi->fm[plan->table_fields[j]].stable = (int32_t)i;
    mi->pmv.resize(P);
    for (size_t p = 0; p < P; ++p) {
        const Pack& k = plan->packs[p];
        mi->pmv[p].dim = k.dim; mi->pmv[p].dtype = k.dtype; mi->pmv[p].n_fields = (int32_t)k.fields.size();
        mi->pmv[p].first_slot = k.first_slot; mi->pmv[p].has_mean = k.has_mean ? 1 : 0;
        mi->pmv[p].first_stable = k.first_stable; mi->pmv[p].n_stables = k.n_stables; mi->pmv[p].pad = 0;
    }
    mi->tfi.resize(plan->table_fields.size());
    for (size_t i = 0; i < mi->tfi.size(); ++i) {
        const int32_t f = plan->table_fields[i];
        mi->tfi[i] = TableField{f, plan->field_slot[f], (int32_t)plan->field_col[f], plan->fields[f].pool};
    }
    mi->slm.resize(F);
    for (size_t j = 0; j < F; ++j) {
        const FieldMeta& m = mi->fm[plan->slot_field[j]];
        const TableMeta& tm = plan->sort_tables[m.stable];
        mi->slm[j] = SlotMeta{tm.key_lo, tm.word_base, tm.rows, m.pack};
    }
    auto pad = [](size_t b) { return (b + 255) / 256 * 256; };
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += pad(bytes); return o; };
    mi->o_desc = take(((size_t)kSmallSlicesMax + kSmallSlicesMax / 64 + 4096 + 2) * 8);   // per slice, then per group of 64
    mi->o_done = take(256);
    mi->o_fm   = take(F * sizeof(FieldMeta));
    mi->o_pm   = take(P * sizeof(PackMeta));
    mi->o_slot = take(F * 4);
    mi->o_ss   = take(plan->small_slices.size() * sizeof(SmallSlice));
    mi->o_tfi  = take(mi->tfi.size() * sizeof(TableField));
    mi->o_tab  = take(plan->sort_tables.size() * sizeof(TableMeta));
    mi->o_tf   = take(plan->table_fields.size() * 4);
    mi->o_slm  = take(F * sizeof(SlotMeta));
    mi->total = off;
}

void point_into(DeviceState* ds, char* base, const MetaImage& mi)
{
    ds->small_desc = reinterpret_cast<uint64_t*>(base + mi.o_desc);
    ds->small_done = reinterpret_cast<int32_t*>(base + mi.o_done);
    ds->fmeta = reinterpret_cast<FieldMeta*>(base + mi.o_fm);
    ds->pmeta = reinterpret_cast<PackMeta*>(base + mi.o_pm);
    ds->slot_field = reinterpret_cast<int32_t*>(base + mi.o_slot);
    ds->small_slices = reinterpret_cast<SmallSlice*>(base + mi.o_ss);
    ds->tfields = reinterpret_cast<TableField*>(base + mi.o_tfi);
    ds->sort_tables = reinterpret_cast<TableMeta*>(base + mi.o_tab);
    ds->table_fields = reinterpret_cast<int32_t*>(base + mi.o_tf);
    ds->slot_meta = reinterpret_cast<SlotMeta*>(base + mi.o_slm);
}

// the pieces of the image that hold data (the descriptors and their counter only have to be zero)
template <typename Fn>
void for_meta_pieces(const pk_plan* plan, const MetaImage& mi, Fn&& fn)
{
    fn(mi.o_fm, mi.fm.data(), mi.fm.size() * sizeof(FieldMeta));
    fn(mi.o_pm, mi.pmv.data(), mi.pmv.size() * sizeof(PackMeta));
    fn(mi.o_slot, plan->slot_field.data(), plan->slot_field.size() * 4);
    fn(mi.o_ss, plan->small_slices.data(), plan->small_slices.size() * sizeof(SmallSlice));
    fn(mi.o_tfi, mi.tfi.data(), mi.tfi.size() * sizeof(TableField));
    fn(mi.o_tab, plan->sort_tables.data(), plan->sort_tables.size() * sizeof(TableMeta));
    fn(mi.o_tf, plan->table_fields.data(), plan->table_fields.size() * 4);
    fn(mi.o_slm, mi.slm.data(), mi.slm.size() * sizeof(SlotMeta));
}

pk_status ensure_device_state(const pk_plan* cplan, DeviceState** out)
{
    pk_plan* plan = const_cast<pk_plan*>(cplan);
    static std::mutex create_mu;
    std::lock_guard<std::mutex> lock(create_mu);
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(PK_EHIP, hip_msg("hipGetDevice", e));
    DeviceState* ds = static_cast<DeviceState*>(plan->device_state);
    if (ds && ds->device == dev) { *out = ds; return PK_OK; }
    if (ds) return fail(PK_EINVAL, "a plan can be used on one device only");
    ds = new DeviceState();
    ds->device = dev;
    if (hipDeviceGetAttribute(&ds->n_cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || ds->n_cus <= 0) ds->n_cus = 256;
    MetaImage mi;
    build_meta_image(plan, &mi);
    e = hipMalloc(&ds->blob, mi.total);
    if (e != hipSuccess) { delete ds; return fail(PK_EHIP, hip_msg("hipMalloc(plan metadata)", e)); }
    char* base = static_cast<char*>(ds->blob);
    point_into(ds, base, mi);
    e = hipMemset(base, 0, mi.o_fm);                   // descriptors and their counter start at zero
    for_meta_pieces(plan, mi, [&](size_t off, const void* src, size_t bytes) {
        if (e == hipSuccess && bytes) e = hipMemcpy(base + off, src, bytes, hipMemcpyHostToDevice);
    });
    if (e != hipSuccess) { (void)hipFree(ds->blob); delete ds; return fail(PK_EHIP, hip_msg("hipMemcpy(plan metadata)", e)); }
    for (int i = 0; i < DeviceState::kSide && e == hipSuccess; ++i) {
        e = hipStreamCreateWithFlags(&ds->side[i], hipStreamNonBlocking);     // default priority
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ds->ev_join[i], hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ds->ev_fork, hipEventDisableTiming);
    if (e != hipSuccess) { (void)hipFree(ds->blob); delete ds; return fail(PK_EHIP, hip_msg("side stream setup", e)); }
    if (plan->opts.debug & 1) ds->overlap = false;
    plan->device_state = ds;
    *out = ds;
    return PK_OK;
}

// fork: side streams wait for what the caller's stream has enqueued so far
pk_status fork_streams(DeviceState* ds, hipStream_t main, int n, int first = 0)
{
    hipError_t e = hipEventRecord(ds->ev_fork, main);
    for (int i = first; i < first + n && e == hipSuccess; ++i) e = hipStreamWaitEvent(ds->side[i], ds->ev_fork, 0);
    return e == hipSuccess ? PK_OK : fail(PK_EHIP, hip_msg("stream fork", e));
}

// join: the caller's stream waits for everything enqueued on the side streams
pk_status join_streams(DeviceState* ds, hipStream_t main, int n, int first = 0)
{
    hipError_t e = hipSuccess;
    for (int i = first; i < first + n && e == hipSuccess; ++i) {
        e = hipEventRecord(ds->ev_join[i], ds->side[i]);
        if (e == hipSuccess) e = hipStreamWaitEvent(main, ds->ev_join[i], 0);
    }
    return e == hipSuccess ? PK_OK : fail(PK_EHIP, hip_msg("stream join", e));
}

void prof_begin(DeviceState* ds, const char* name, hipStream_t s)
{
    if (!ds->prof_on) return;
    if (ds->events_used + 2 > ds->events.size()) {
        const size_t old = ds->events.size();
        ds->events.resize(old + 512);
        for (size_t i = old; i < ds->events.size(); ++i) (void)hipEventCreate(&ds->events[i]);
    }
    ds->recs.push_back({name, ds->events_used});
    (void)hipEventRecord(ds->events[ds->events_used], s);
}

void prof_end(DeviceState* ds, hipStream_t s)
{
    if (!ds->prof_on) return;
    (void)hipEventRecord(ds->events[ds->events_used + 1], s);
    ds->events_used += 2;
}

#define PK_LAUNCH(name, kernel, grid, block, shmem, ...)                                        \
    do {                                                                                        \
        prof_begin(ds, name, stream);                                                           \
        kernel<<<grid, block, shmem, stream>>>(__VA_ARGS__);                                    \
        prof_end(ds, stream);                                                                   \
        hipError_t e_ = hipGetLastError();                                                      \
        if (e_ != hipSuccess) return fail(PK_EHIP, hip_msg("launch of " name, e_));             \
    } while (0)

unsigned blocks_for(int64_t items, int64_t per_block, int64_t cap)
{
    int64_t b = (items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (unsigned)b;
}

int pow2_ceil(int v) { int p = 1; while (p < v) p <<= 1; return p; }

// pack p's packed_offsets start (entries): the packs before it hold k*B+1 each
int64_t po_off(const pk_plan* plan, int p, int32_t B)
{
    return (int64_t)plan->packs[p].first_slot * B + p;
}

struct Ws {
    char* base;
    Layout L;
    template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(base + off); }
};

pk_status check_common(const pk_plan* plan, int32_t B, int64_t nnz, const void* ws, size_t ws_bytes, const char* who)
{
    if (!plan) return fail(PK_EINVAL, std::string(who) + ": plan is NULL");
    if (B <= 0) return fail(PK_ESHAPE, std::string(who) + ": B must be positive");
    if (nnz < 0) return fail(PK_ESHAPE, std::string(who) + ": nnz must be non-negative");
    if (nnz >= ((int64_t)1 << 31)) return fail(PK_EOVERFLOW, std::string(who) + ": nnz must be below 2^31");
    if (plan->opts.max_batch > 0 && B > plan->opts.max_batch) return fail(PK_ESHAPE, std::string(who) + ": B exceeds the plan's max_batch");
    if (plan->opts.max_nnz > 0 && nnz > plan->opts.max_nnz) return fail(PK_ESHAPE, std::string(who) + ": nnz exceeds the plan's max_nnz");
    if ((int64_t)B * plan->out_dim >= ((int64_t)1 << 32)) return fail(PK_EOVERFLOW, std::string(who) + ": B * out_dim must be below 2^32");
    if ((int64_t)B * (int64_t)plan->fields.size() >= ((int64_t)1 << 31)) return fail(PK_EOVERFLOW, std::string(who) + ": n_fields * B must be below 2^31");
    if (!ws) return fail(PK_EINVAL, std::string(who) + ": workspace is NULL");
    if (reinterpret_cast<uintptr_t>(ws) % kAlign) return fail(PK_EWORKSPACE, std::string(who) + ": workspace must be 256-byte aligned");
    if (ws_bytes < make_layout(plan, B, nnz).total) return fail(PK_EWORKSPACE, std::string(who) + ": workspace is smaller than pk_workspace_bytes");
    return PK_OK;
}

// ---- per-pack template dispatch ------------------------------------------------
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// every field of the pack starts at an output column that is a multiple of 4
bool cols_aligned(const pk_plan* plan, int p)
{
    for (int32_t f : plan->packs[p].fields)
        if (plan->field_col[f] % 4) return false;
    return true;
}

struct PoolArgs {
    const void* W; const uint32_t* keys; const int32_t* po; const PackState* st; uint32_t rows; const FieldMeta* fmeta;
    const int32_t* slot_field; int B; int D; int64_t n_bags; float* out; int64_t out_stride; unsigned grid_cap;
    bool aligned; HotView hv;
};
struct AdaArgs {
    void* W; float* A; const PackState* st; int p; const uint32_t* unique; const int32_t* seg;
    double* ghot; int dmax; const int4* tile_hdr; int tp; int n_host; const uint32_t* seg_ent; int ent_mult;
    int has_mean; const float* grad; int64_t gstride; int64_t out_dim; uint32_t addr_max; int D;
    float lr; float eps; int64_t nnz_bound; bool aligned; HotView hv;
};

template <typename WT, int VEC, int LPR, int NCH>
pk_status launch_pool(DeviceState* ds, hipStream_t stream, const PoolArgs& a)
{
    constexpr int GPB = NT / LPR;
    const unsigned grid = blocks_for(a.n_bags, GPB, a.grid_cap);
    if (a.hv.slot_of)
        PK_LAUNCH("pk_pool", (pk_pool_kernel<WT, VEC, LPR, NCH, true>), dim3(grid), dim3(NT), 0,
                  static_cast<const WT*>(a.W), a.keys, a.po, a.st, a.rows, a.fmeta, a.slot_field, a.B, a.D, a.n_bags,
                  a.out, a.out_stride, a.hv);
    else
        PK_LAUNCH("pk_pool", (pk_pool_kernel<WT, VEC, LPR, NCH, false>), dim3(grid), dim3(NT), 0,
                  static_cast<const WT*>(a.W), a.keys, a.po, a.st, a.rows, a.fmeta, a.slot_field, a.B, a.D, a.n_bags,
                  a.out, a.out_stride, a.hv);
    return PK_OK;
}

template <typename WT, int VEC, int LPR, int NCH>
pk_status launch_adagrad(DeviceState* ds, hipStream_t stream, const AdaArgs& a)
{
    const unsigned grid = (blocks_for(a.nnz_bound, a.tp, 256 * 16) + 7u) & ~7u;
    if (a.has_mean)
        PK_LAUNCH("pk_adagrad", (pk_adagrad_kernel<WT, VEC, LPR, NCH, true>), dim3(grid), dim3(NT), 0,
                  static_cast<WT*>(a.W), a.A, a.st, a.p, a.unique, a.seg, a.ghot, a.dmax, a.tile_hdr,
                  a.tp, a.n_host, a.seg_ent, a.ent_mult, a.grad, a.gstride, a.out_dim, a.addr_max, a.D, a.lr, a.eps, a.hv);
    else
        PK_LAUNCH("pk_adagrad", (pk_adagrad_kernel<WT, VEC, LPR, NCH, false>), dim3(grid), dim3(NT), 0,
                  static_cast<WT*>(a.W), a.A, a.st, a.p, a.unique, a.seg, a.ghot, a.dmax, a.tile_hdr,
                  a.tp, a.n_host, a.seg_ent, a.ent_mult, a.grad, a.gstride, a.out_dim, a.addr_max, a.D, a.lr, a.eps, a.hv);
    return PK_OK;
}

// Picks lanes-per-row so that one row is one coalesced access: 16 bytes per
// lane when the dimension allows it, else one element per lane.
#define PK_DISPATCH_BODY(FN)                                                                    \
    if (D % VECW == 0 && a.aligned) {                                                           \
        switch (pow2_ceil(D / VECW)) {                                                          \
            case 1:  return FN<WT, VECW, 1, 1>(ds, stream, a);                                  \
            case 2:  return FN<WT, VECW, 2, 1>(ds, stream, a);                                  \
            case 4:  return FN<WT, VECW, 4, 1>(ds, stream, a);                                  \
            case 8:  return FN<WT, VECW, 8, 1>(ds, stream, a);                                  \
            case 16: return FN<WT, VECW, 16, 1>(ds, stream, a);                                 \
            case 32: return FN<WT, VECW, 32, 1>(ds, stream, a);                                 \
            case 64: return FN<WT, VECW, 64, 1>(ds, stream, a);                                 \
        }                                                                                       \
    }                                                                                           \
    if (D <= 4)   return FN<WT, 1, 4, 1>(ds, stream, a);                                        \
    if (D <= 16)  return FN<WT, 1, 16, 1>(ds, stream, a);                                       \
    if (D <= 64)  return FN<WT, 1, 64, 1>(ds, stream, a);                                       \
    if (D <= 128) return FN<WT, 1, 64, 2>(ds, stream, a);                                       \
    if (D <= 256) return FN<WT, 1, 64, 4>(ds, stream, a);                                       \
    return fail(PK_EOVERFLOW, "dim above 256");

template <typename WT, int VECW>
pk_status dispatch_pool(DeviceState* ds, hipStream_t stream, int D, const PoolArgs& a) { PK_DISPATCH_BODY(launch_pool) }
template <typename WT, int VECW>
pk_status dispatch_adagrad(DeviceState* ds, hipStream_t stream, int D, const AdaArgs& a) { PK_DISPATCH_BODY(launch_adagrad) }

// shape of the pooling code for a pack, as numbered in pk_fused_kernel, and its lanes per row
int pool_variant(int dtype, int D, bool aligned, int* lpr_out)
{
    static const int lanes[12] = {1, 2, 4, 8, 16, 32, 64, 4, 16, 64, 64, 64};
    const int vecw = dtype == PK_F32 ? 4 : 8;
    int shape;
    if (D % vecw == 0 && aligned && pow2_ceil(D / vecw) <= 64) {
        shape = 0;
        while ((1 << shape) < pow2_ceil(D / vecw)) ++shape;
    } else {
        shape = D <= 4 ? 7 : D <= 16 ? 8 : D <= 64 ? 9 : D <= 128 ? 10 : 11;
    }
    *lpr_out = lanes[shape];
    return (dtype == PK_F32 ? 0 : 12) + shape;
}

template <typename WT>
pk_status hh_swap(DeviceState* ds, hipStream_t stream, const pk_hh_pack& h, int64_t n_hot_old, int64_t n_new, int D,
                  const int32_t* evict_slot, const uint32_t* ins_row, const uint32_t* counts)
{
    // how many rows move is only known on the device; the grids cover the most that can
    const unsigned grid = blocks_for(std::max<int64_t>(n_new, n_hot_old), NT / 64, 4096);
    PK_LAUNCH("pk_hh_evict", pk_hh_evict_kernel<WT>, dim3(grid), dim3(NT), 0, static_cast<WT*>(h.W_cold), h.A_cold,
              static_cast<const WT*>(h.W_hot), h.A_hot, h.hot_row, h.slot_of, evict_slot, counts, D);
    PK_LAUNCH("pk_hh_insert", pk_hh_insert_kernel<WT>, dim3(grid), dim3(NT), 0, static_cast<const WT*>(h.W_cold),
              h.A_cold, static_cast<WT*>(h.W_hot), h.A_hot, h.hot_row, h.slot_of, evict_slot, ins_row, counts, n_hot_old,
              h.hot_rows, D);
    return PK_OK;
}
