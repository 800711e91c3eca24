// Device code and launch logic of the packed multi-field embedding layer for
// gfx950 (wave64).  The path is gather / reduce / scatter and is bound by HBM
// bandwidth, so there is no MFMA here: the work is in keeping every access
// coalesced across the embedding dimension, in touching each distinct row once
// (the point of Unique, Sec. II-D), and in launching once per pack instead of
// once per field (D-Packing, Sec. III-B).
//
// Stages of one step (all packs of the plan share the integer stages):
//   small batches, forward pass in ONE launch (fused): slice blocks (H1 + H2: every block owns a
//             slice of a table's key range and finds its occurrences in the IDs), blocks that write
//             the packed bag offsets, and pooling blocks (H3-H5, keys formed from the IDs)
//   large batches:
//   clear     per-pack state, slice totals and look-back descriptors of this call
//   keys      H1: key = base_row + (uint64)id mod rows in packed order, packed bag offsets,
//             occurrences per slice
//   pool      H3-H5: per pack, gather rows by key, pool per bag, write concatenated
//   scan      H2: places of the slices' records
//   scatter   H2: one (key in slice, bag) record per occurrence, grouped by slice
//   slices    H2: per slice, in LDS: mark (bitmap, number of distinct keys), a scan, then place: distinct
//             keys (ascending), occurrences grouped by key, segment offsets, headers of the backward tiles
//   inverse   H2: inverse[q] = rank(key[q]) from the bitmap and rank samples of the slices
//   adagrad   H6+H7: per pack, per distinct key: reduce gradients, update row in place
//   hot       H7: keys whose occurrences span several backward tiles, from their partial sums
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "pk_internal.h"

using namespace pk;

// The scratch of pk_forward_static: workspace, plan metadata and look-back descriptors of callers that
// cannot allocate.  Every GPU the library runs on holds its own copy until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// One translation unit; the kernels and their launch helpers are kept in section files:
//   dev_common.h   block scans, folding hash, look-back prefix sums, tile order
//   dev_dedup.h    keys, slice scan, scatter, slices, inverse (H1, H2)
//   dev_rows.h     row access, plain or hybrid row addressing
//   dev_pool.h     pooling (H3-H5) and the one launch of the forward pass for small batches
//   dev_adagrad.h  gradient reduction + Adagrad (H6, H7)
//   dev_hybrid.h   HybridHash bookkeeping kernels
//   host_launch.h  device state of a plan, profiling brackets, launchers, template dispatch
// and this file holds the entry points of the C ABI.
namespace {

#include "dev_common.h"
#include "dev_dedup.h"
#include "dev_rows.h"
#include "dev_pool.h"
#include "dev_adagrad.h"
#include "dev_hybrid.h"
#include "host_launch.h"

}  // namespace

namespace pk {
void destroy_device_state(pk_plan* plan)
{
    DeviceState* ds = static_cast<DeviceState*>(plan->device_state);
    if (!ds) return;
    for (hipEvent_t ev : ds->events) (void)hipEventDestroy(ev);
    for (int i = 0; i < DeviceState::kSide; ++i) {
        if (ds->side[i]) { (void)hipStreamSynchronize(ds->side[i]); (void)hipStreamDestroy(ds->side[i]); }
        if (ds->ev_join[i]) (void)hipEventDestroy(ds->ev_join[i]);
    }
    if (ds->ev_fork) (void)hipEventDestroy(ds->ev_fork);
    if (ds->blob) (void)hipFree(ds->blob);
    delete ds;
    plan->device_state = nullptr;
}
}  // namespace pk

#ifdef PK_PHASE_TIMES
static long long* g_ptimes_dev = nullptr;
extern "C" int pk_debug_ptimes(long long* out, int n_blocks)
{
    (void)hipDeviceSynchronize();
    return (int)hipMemcpy(out, g_ptimes_dev, (size_t)n_blocks * 16 * 8, hipMemcpyDeviceToHost);
}
#endif

extern "C" {

// The forward pass, or one of its two stages (Sec. III-C, D-Interleaving runs them on different
// streams for different micro-batches): kDedup = H1 + H2, kPool = H3-H5 from a workspace that a
// dedup stage filled.  hot: per pack, where the rows of a Hot-storage live (HybridHash), or NULL.
enum { kDedup = 1, kPool = 2 };

static pk_status forward_impl(const pk_plan* plan, DeviceState* ds_given, int stages, const char* who, void* const* W, const HotView* hot,
                              const int64_t* ids, const int32_t* offsets, int32_t B, int64_t nnz, float* out,
                              int64_t out_row_stride, void* workspace, size_t ws_bytes, void* hip_stream)
{
    const bool do_dedup = stages & kDedup, do_pool = stages & kPool;
    pk_status rc = check_common(plan, B, nnz, workspace, ws_bytes, who);
    if (rc != PK_OK) return rc;
    if (do_dedup && (!offsets || (!ids && nnz > 0))) return fail(PK_EINVAL, std::string(who) + ": NULL argument");
    if (do_pool && (!W || !out)) return fail(PK_EINVAL, std::string(who) + ": NULL argument");
    const int P = (int)plan->packs.size(), F = (int)plan->fields.size();
    for (int p = 0; p < P && do_pool; ++p)
        if (!W[p]) return fail(PK_EINVAL, std::string(who) + ": W[" + std::to_string(p) + "] is NULL");
    if (do_pool && out_row_stride < plan->out_dim)
        return fail(PK_ESHAPE, std::string(who) + ": out_row_stride is smaller than out_dim");
    DeviceState* ds = ds_given;
    if (!ds) {
        rc = ensure_device_state(plan, &ds);
        if (rc != PK_OK) return rc;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    Ws ws{static_cast<char*>(workspace), make_layout(plan, B, nnz)};
    const Layout& L = ws.L;

    PackState* st = ws.at<PackState>(L.state);
    int32_t* packed_offsets = ws.at<int32_t>(L.packed_offsets);
    uint32_t* keys = ws.at<uint32_t>(L.keys);
    int32_t* inverse = ws.at<int32_t>(L.inverse);
    uint32_t* seg_ent = ws.at<uint32_t>(L.seg_ent);
    int4* tile_hdr = ws.at<int4>(L.tile_hdr);
    uint32_t* unique = ws.at<uint32_t>(L.unique);
    int32_t* seg = ws.at<int32_t>(L.seg);
    double* ghot = ws.at<double>(L.ghot);
    const int T = (int)plan->sort_tables.size();
    const int64_t n_bags = (int64_t)F * B;

    auto pool_aligned = [&](int p) {
        return cols_aligned(plan, p) && aligned16(out) && out_row_stride % 4 == 0 && aligned16(W[p]);
    };
    SliceArgs sa{};
    sa.tmeta = ds->sort_tables; sa.tfields = ds->tfields; sa.T = T;
    sa.fmeta = ds->fmeta; sa.pm = ds->pmeta; sa.slot_field = ds->slot_field; sa.st = st; sa.P = P;
    sa.F = F; sa.B = B; sa.nnz = nnz;
    sa.ids = ids; sa.offsets = offsets; sa.small_slices = ds->small_slices;
    sa.packed_offsets = packed_offsets;
    sa.keys = keys; sa.inverse = inverse;
    sa.unique = unique; sa.seg_all = seg; sa.ent_all = seg_ent; sa.ent_mult = plan->any_mean ? 2 : 1;
    sa.tile_hdr = tile_hdr; sa.tp = L.pos_tile; sa.ghot = ghot; sa.dmax = L.dmax;
    sa.n_slices = L.n_slices;
    sa.out_dim = plan->out_dim;
#ifdef PK_PHASE_TIMES
    static long long* g_pt = nullptr;
    if (!g_pt) { (void)hipMalloc(&g_pt, (size_t)16 * 65536 * 8); }
    (void)hipMemsetAsync(g_pt, 0, (size_t)16 * 65536 * 8, stream);
    sa.ptimes = g_pt;
    g_ptimes_dev = g_pt;
#endif

    // ---- small batches: dedup (and pooling) in one launch ----
    if (L.small && do_dedup) {
        const bool fuse_pool = do_pool && !hot && P <= kFusedPacks;
        sa.target = 0; sa.log_max = kSliceLogMax;
        sa.desc = ds->small_desc; sa.gdesc = ds->small_desc + kSmallSlicesMax; sa.done = ds->small_done;
        PoolJob pj{};
        int nb = 0, np = 0;
        for (int p = 0; p < P && fuse_pool; ++p) {
            const Pack& k = plan->packs[p];
            if (k.fields.empty()) continue;
            int lpr = 1;
            PoolPack& q = pj.pack[np++];
            q.W = W[p]; q.slot_field = ds->slot_field + k.first_slot;
            q.n_bags = (int64_t)k.fields.size() * B; q.D = k.dim; q.rows = (uint32_t)k.rows;
            q.variant = pool_variant(k.dtype, k.dim, pool_aligned(p), &lpr);
            q.block_begin = nb;
            nb += (int)blocks_for(q.n_bags, kSliceThreads / lpr, 2048);
        }
        pj.n_packs = np; pj.B = B; pj.n_blocks = nb; pj.out = out; pj.out_stride = out_row_stride;
        const int meta_blocks = (int)blocks_for(n_bags, kSliceThreads * 4, 64);
        const size_t dyn = (size_t)std::max(1, plan->max_table_fields) * kSliceTfWords * 4;
        const unsigned fused_blocks = (unsigned)(L.n_slices + meta_blocks + nb);
        if ((int)fused_blocks <= ds->n_cus)
            PK_LAUNCH("pk_fused", pk_fused_kernel<4>, dim3(fused_blocks), dim3(kSliceThreads), dyn, sa, pj, L.n_slices, meta_blocks);
        else
            PK_LAUNCH("pk_fused", pk_fused_kernel<8>, dim3(fused_blocks), dim3(kSliceThreads), dyn, sa, pj, L.n_slices, meta_blocks);
        if (!do_pool || fuse_pool) return PK_OK;
    }

    // ---- large batches: partition the occurrences by slice, then one block per slice ----
    // bags per tile of the keys and scatter kernels: about 16 K occurrences, 32 to 1024 bags
    const int bt = L.bags_per_tile;
    const int64_t n_tiles = (int64_t)F * ((B + bt - 1) / bt);
    const size_t scan_words = field_scan_words(F) + 2 * (size_t)T + 1;
    if (do_dedup && !L.small &&
        std::max({scan_words, 2 * (size_t)L.max_table_slices, field_scan_words(F) + 4 * (size_t)F}) * 4 > 64 * 1024)
        return fail(PK_EOVERFLOW, std::string(who) + ": fields, tables and slices per table together exceed what the "
                                  "dedup kernels stage in LDS");
    if (do_dedup && !L.small) {
        sa.target = kSliceOccLarge; sa.log_max = L.log_max;
        sa.desc = nullptr; sa.gdesc = nullptr; sa.done = nullptr;
        sa.slice_info = ws.at<SliceInfo>(L.slice_info); sa.rec = ws.at<uint2>(L.rec);
        sa.cut = ws.at<TableCut>(L.tgeom);
        sa.bitmap = ws.at<uint32_t>(L.bitmap);
        int32_t* slice_total = ws.at<int32_t>(L.slice_total);
        // block 0 of the first launch clears the pack states itself (it then fills them); the others zero the rest
        const size_t state_bytes = L.slice_total - L.clear_begin;
        const int64_t n_clear4 = (int64_t)((L.clear_bytes - state_bytes) / 16);
        const size_t setup_lds = scan_words * 4;
        PK_LAUNCH("pk_setup", pk_setup_kernel, dim3(blocks_for(n_clear4, kSetupThreads, 256)), dim3(kSetupThreads), setup_lds,
                  ws.at<uint4>(L.slice_total), n_clear4, offsets, B, F, P, T, nnz, sa.target, sa.log_max, ds->fmeta, ds->pmeta,
                  ds->sort_tables, ds->slot_field, st, packed_offsets, seg, ws.at<TableCut>(L.tgeom), L.n_slices,
                  ws.at<int32_t>(L.fscan));
        const dim3 key_grid(blocks_for(n_tiles, 1, 256 * 8));
        const size_t keys_lds = (size_t)L.max_table_slices * 4;
#define PK_KEYS_LAUNCH(BT)                                                                                      \
    PK_LAUNCH("pk_keys", pk_keys_kernel<BT>, key_grid, dim3(NT), keys_lds, ids, offsets, B, F, ds->fmeta, ds->pmeta, st,  \
              keys, packed_offsets, slice_total, ws.at<TableCut>(L.tgeom), ws.at<int32_t>(L.fscan),                    \
              L.tile_hist_stride ? ws.at<int32_t>(L.tile_hist) : nullptr, L.tile_hist_stride)
        switch (bt) {
            case 32: PK_KEYS_LAUNCH(32); break;
            case 128: PK_KEYS_LAUNCH(128); break;
            case 512: PK_KEYS_LAUNCH(512); break;
            default: PK_KEYS_LAUNCH(1024); break;
        }
#undef PK_KEYS_LAUNCH
    }

    // Pooling needs the keys only.  Large batches: it runs on side streams beside the rest of
    // the dedup chain.  Interleaving groups (Sec. III-C, K-Interleaving): pack p belongs to group
    // p mod G; a group's packed operations follow one another on the group's stream, the groups
    // run side by side.  G = 0 lets the size decide (2 groups for large batches: a process has 4 hardware queues and the dedup chain uses two; none for small).
    const int G = plan->opts.interleave_groups;
    const bool overlap = ds->overlap && !ds->prof_on && !L.small &&
                         (G >= 2 || (G == 0 && (P > 1 || nnz >= (1 << 20)) && nnz >= (1 << 18)));
    const int n_side = overlap && do_pool ? std::min<int>(P, G >= 2 ? G : 2) : 0;
    if (n_side) { rc = fork_streams(ds, stream, n_side); if (rc != PK_OK) return rc; }
    for (int p = 0; p < P && do_pool; ++p) {
        const Pack& k = plan->packs[p];
        if (k.fields.empty()) continue;
        PoolArgs a{W[p], keys, packed_offsets + po_off(plan, p, B), st + p, (uint32_t)k.rows, ds->fmeta,
                   ds->slot_field + k.first_slot, B, k.dim, (int64_t)k.fields.size() * B, out, out_row_stride, 256 * 32,
                   pool_aligned(p), hot ? hot[p] : HotView{nullptr, nullptr, nullptr}};
        hipStream_t ps = n_side ? ds->side[p % n_side] : stream;
        rc = k.dtype == PK_F32 ? dispatch_pool<float, 4>(ds, ps, k.dim, a)
                               : dispatch_pool<uint16_t, 8>(ds, ps, k.dim, a);
        if (rc != PK_OK) return rc;
    }
    if (do_dedup && !L.small) {
        int32_t* slice_total = ws.at<int32_t>(L.slice_total);
        int32_t* slice_cursor = ws.at<int32_t>(L.slice_cursor);
        int32_t* big_list = ws.at<int32_t>(L.big_list);
        PK_LAUNCH("pk_slice_scan", pk_slice_scan_kernel, dim3(blocks_for(L.n_slices, kScanThreads, 1 << 20)),
                  dim3(kScanThreads), (size_t)(T + 1) * 4,
                  ws.at<TableCut>(L.tgeom), T, slice_total, slice_cursor, ws.at<SliceInfo>(L.slice_info),
                  L.n_slices, L.log_max == kSliceLogFine ? kBigSliceCount : 0x7FFFFFFF, big_list + kBigSlicesMax, big_list);
        const size_t sc_lds = 2 * (size_t)L.max_table_slices * 4;
        const dim3 tile_grid(blocks_for(n_tiles, 1, 256 * 8));
#define PK_SCATTER_LAUNCH(BT)                                                                                   \
    PK_LAUNCH("pk_scatter", pk_scatter_kernel<BT>, tile_grid, dim3(NT), sc_lds, offsets, B, F, nnz, sa.log_max, ds->fmeta,  \
              ws.at<TableCut>(L.tgeom), st, keys, slice_cursor, ws.at<uint2>(L.rec), L.max_table_slices, plan->out_dim,     \
              ws.at<int32_t>(L.fscan), L.tile_hist_stride ? ws.at<int32_t>(L.tile_hist) : nullptr, L.tile_hist_stride)
        switch (bt) {
            case 32: PK_SCATTER_LAUNCH(32); break;
            case 128: PK_SCATTER_LAUNCH(128); break;
            case 512: PK_SCATTER_LAUNCH(512); break;
            default: PK_SCATTER_LAUNCH(1024); break;
        }
#undef PK_SCATTER_LAUNCH
        const size_t tf_lds = (size_t)std::max(1, plan->max_table_fields) * kSliceTfWords * 4;
        if (L.n_slices > 0) {
            SliceArgs sm = sa, sp = sa;
            sm.slice_nu = ws.at<int32_t>(L.slice_nu);       // the mark launch writes the counts ...
            sp.slice_nu = ws.at<int32_t>(L.slice_usum);     // ... the place launch reads their running sums
            sm.big_list = sp.big_list = big_list;
            sm.n_big = sp.n_big = big_list + kBigSlicesMax;
            const dim3 sgrid((unsigned)L.n_slices);
            const bool fine = L.log_max == kSliceLogFine;
            // the listed slices run beside the others, on a stream of their own (not while kernels are timed one by one)
            const bool beside = fine && ds->overlap && !ds->prof_on && do_pool;   // (a dedup on its own is itself running beside other work: a process has four hardware queues)
            hipStream_t main_stream = stream;
            if (beside) { rc = fork_streams(ds, main_stream, 1, DeviceState::kSide - 1); if (rc != PK_OK) return rc; }
            if (fine) {
                stream = beside ? ds->side[DeviceState::kSide - 1] : main_stream;
                PK_LAUNCH("pk_slices_mark_big", pk_slices_big_kernel<kSliceMark>, dim3(kBigSlicesMax), dim3(kSliceThreads), tf_lds, sm);
                stream = main_stream;
                PK_LAUNCH("pk_slices_mark", pk_slices_kernel<kSliceMark>, sgrid, dim3(kFineThreads), tf_lds, sm);
            } else {
                PK_LAUNCH("pk_slices_mark", pk_slices_wide_kernel<kSliceMark>, sgrid, dim3(kSliceThreads), tf_lds, sm);
            }
            if (beside) { rc = join_streams(ds, main_stream, 1, DeviceState::kSide - 1); if (rc != PK_OK) return rc; }
            PK_LAUNCH("pk_unique_scan", pk_unique_scan_kernel, dim3(blocks_for(L.n_slices, kScanThreads, 1 << 20)),
                      dim3(kScanThreads), 0, sm.slice_nu, L.n_slices, sp.slice_nu);
            if (beside) { rc = fork_streams(ds, main_stream, 1, DeviceState::kSide - 1); if (rc != PK_OK) return rc; }
            if (fine) {
                stream = beside ? ds->side[DeviceState::kSide - 1] : main_stream;
                PK_LAUNCH("pk_slices_place_big", pk_slices_big_kernel<kSlicePlace>, dim3(kBigSlicesMax), dim3(kSliceThreads), tf_lds, sp);
                stream = main_stream;
                PK_LAUNCH("pk_slices_place", pk_slices_kernel<kSlicePlace>, sgrid, dim3(kFineThreads), tf_lds, sp);
            } else {
                PK_LAUNCH("pk_slices_place", pk_slices_wide_kernel<kSlicePlace>, sgrid, dim3(kSliceThreads), tf_lds, sp);
            }
            if (beside) { rc = join_streams(ds, main_stream, 1, DeviceState::kSide - 1); if (rc != PK_OK) return rc; }
        }
        const size_t inv_lds = (field_scan_words(F) + 4 * (size_t)F) * 4;
        // (every block stages the field scan and the slots' metadata: with many fields fewer blocks take more tiles each)
        const unsigned xq = (blocks_for(nnz, 1024, F > 256 ? 256 * 4 : 256 * 16) + 7u) & ~7u;
        PK_LAUNCH("pk_inverse", pk_inverse_kernel<1024>, dim3(xq), dim3(NT), inv_lds, F, ws.at<int32_t>(L.fscan), ds->slot_meta, st,
                  keys, reinterpret_cast<const uint4*>(sa.bitmap), inverse);
    }
    if (n_side) { rc = join_streams(ds, stream, n_side); if (rc != PK_OK) return rc; }
    return PK_OK;
}

pk_status pk_forward(const pk_plan* plan, void* const* W, const int64_t* ids, const int32_t* offsets, int32_t B,
                     int64_t nnz, float* out, int64_t out_row_stride, void* workspace, size_t ws_bytes,
                     void* hip_stream)
{
    return forward_impl(plan, nullptr, kDedup | kPool, "pk_forward", W, nullptr, ids, offsets, B, nnz, out, out_row_stride,
                        workspace, ws_bytes, hip_stream);
}

pk_status pk_forward_dedup(const pk_plan* plan, const int64_t* ids, const int32_t* offsets, int32_t B, int64_t nnz,
                   void* workspace, size_t ws_bytes, void* hip_stream)
{
    return forward_impl(plan, nullptr, kDedup, "pk_forward_dedup", nullptr, nullptr, ids, offsets, B, nnz, nullptr, 0, workspace,
                        ws_bytes, hip_stream);
}

pk_status pk_forward_pool(const pk_plan* plan, void* const* W, int32_t B, int64_t nnz, float* out, int64_t out_row_stride,
                  void* workspace, size_t ws_bytes, void* hip_stream)
{
    return forward_impl(plan, nullptr, kPool, "pk_forward_pool", W, nullptr, nullptr, nullptr, B, nnz, out, out_row_stride, workspace,
                        ws_bytes, hip_stream);
}

// ---- the forward pass for callers that cannot allocate --------------------------------------
// Plan metadata reaches the scratch through kernel arguments (no copy engine, no staging buffer).
struct PutChunk { unsigned char b[2048]; };
__global__ void __launch_bounds__(256)
pk_put_kernel(unsigned char* dst, PutChunk c, int n)
{
    for (int i = threadIdx.x; i < n; i += 256) dst[i] = c.b[i];
}

namespace {
constexpr int kStaticDevices = 64;
struct StaticDev {
    unsigned char* ptr = nullptr;        // this device's copy of `scratch`
    uint64_t plan_serial = 0;            // whose metadata the scratch holds
    DeviceState ds;                      // pointers into the scratch; no streams, no events
};
StaticDev g_static[kStaticDevices];
std::mutex g_static_mu;
}  // namespace

pk_status pk_forward_static(const pk_plan* plan, void* const* W, const int64_t* ids, const int32_t* offsets, int32_t B,
                            int64_t nnz, float* out, int64_t out_row_stride, void* hip_stream)
{
    if (!plan) return fail(PK_EINVAL, "pk_forward_static: plan is NULL");
    if (B <= 0 || nnz < 0 || nnz >= ((int64_t)1 << 31)) return fail(PK_ESHAPE, "pk_forward_static: bad B or nnz");
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(PK_EHIP, hip_msg("hipGetDevice", e));
    if (dev < 0 || dev >= kStaticDevices) return fail(PK_EINVAL, "pk_forward_static: device index out of range");
    std::lock_guard<std::mutex> lock(g_static_mu);
    StaticDev& sd = g_static[dev];
    if (!sd.ptr) {                               // once per device, with that device current
        unsigned char* ptr = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return fail(PK_EHIP, hip_msg("hipGetSymbolAddress(scratch)", e));
        sd.ptr = ptr;
        sd.ds.device = dev;
        if (hipDeviceGetAttribute(&sd.ds.n_cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || sd.ds.n_cus <= 0) sd.ds.n_cus = 256;
        sd.ds.overlap = false;                   // no internal streams: every kernel on the caller's stream
    }
    MetaImage mi;
    build_meta_image(plan, &mi);
    const Layout L = make_layout(plan, B, nnz);
    if (mi.total + L.total > kStaticScratchBytes)
        return fail(PK_EWORKSPACE, "pk_forward_static: this plan, B and nnz need " + std::to_string(mi.total + L.total) +
                                   " bytes of scratch; the static scratch holds " + std::to_string(kStaticScratchBytes));
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (sd.plan_serial != plan->serial) {        // another plan's metadata (or none) is there: put this plan's
        pk_status rc = PK_OK;
        for_meta_pieces(plan, mi, [&](size_t off, const void* src, size_t bytes) {
            for (size_t done = 0; done < bytes && rc == PK_OK; done += sizeof(PutChunk)) {
                PutChunk c;
                const size_t n = std::min(sizeof(PutChunk), bytes - done);
                std::copy(static_cast<const unsigned char*>(src) + done, static_cast<const unsigned char*>(src) + done + n, c.b);
                pk_put_kernel<<<1, 256, 0, stream>>>(sd.ptr + off + done, c, (int)n);
                if (hipGetLastError() != hipSuccess) rc = fail(PK_EHIP, "pk_forward_static: launch of pk_put failed");
            }
        });
        if (rc != PK_OK) return rc;
        sd.plan_serial = plan->serial;
    }
    point_into(&sd.ds, reinterpret_cast<char*>(sd.ptr), mi);
    return forward_impl(plan, &sd.ds, kDedup | kPool, "pk_forward_static", W, nullptr, ids, offsets, B, nnz, out, out_row_stride,
                        sd.ptr + mi.total, kStaticScratchBytes - mi.total, hip_stream);
}

static pk_status backward_impl(const pk_plan* plan, void* const* W, float* const* A, const HotView* hot,
                               const float* grad_out, int64_t grad_row_stride, int32_t B, int64_t nnz, float lr,
                               float eps, void* workspace, size_t ws_bytes, void* hip_stream)
{
    pk_status rc = check_common(plan, B, nnz, workspace, ws_bytes, "pk_backward_update");
    if (rc != PK_OK) return rc;
    if (!W || !A || !grad_out) return fail(PK_EINVAL, "pk_backward_update: NULL argument");
    const int P = (int)plan->packs.size();
    for (int p = 0; p < P; ++p)
        if (!W[p] || !A[p]) return fail(PK_EINVAL, "pk_backward_update: W or A of pack " + std::to_string(p) + " is NULL");
    if (grad_row_stride < plan->out_dim) return fail(PK_ESHAPE, "pk_backward_update: grad_row_stride is smaller than out_dim");
    if ((int64_t)B * grad_row_stride >= ((int64_t)1 << 32)) return fail(PK_EOVERFLOW, "pk_backward_update: B * grad_row_stride must be below 2^32");
    DeviceState* ds = nullptr;
    rc = ensure_device_state(plan, &ds);
    if (rc != PK_OK) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    Ws ws{static_cast<char*>(workspace), make_layout(plan, B, nnz)};
    const Layout& L = ws.L;
    PackState* st = ws.at<PackState>(L.state);
    // packs touch disjoint tables: one side stream each
    const int G = plan->opts.interleave_groups;
    const bool overlap = ds->overlap && !ds->prof_on && P > 1 && G != 1;
    const int n_side = overlap ? std::min<int>(P, G >= 2 ? G : 2) : 0;
    if (n_side) { rc = fork_streams(ds, stream, n_side); if (rc != PK_OK) return rc; }
    for (int p = 0; p < P; ++p) {
        const Pack& k = plan->packs[p];
        hipStream_t ps = n_side ? ds->side[p % n_side] : stream;
        if (k.fields.empty()) continue;
        AdaArgs a{W[p], A[p], st + p, p, ws.at<uint32_t>(L.unique), ws.at<int32_t>(L.seg), ws.at<double>(L.ghot),
                  L.dmax, ws.at<int4>(L.tile_hdr), L.pos_tile, P == 1 ? (int)nnz : -1,
                  ws.at<uint32_t>(L.seg_ent), plan->any_mean ? 2 : 1, k.has_mean ? 1 : 0, grad_out, grad_row_stride,
                  plan->out_dim, (uint32_t)((int64_t)(B - 1) * grad_row_stride + plan->out_dim - k.dim), k.dim, lr,
                  eps, nnz,
                  cols_aligned(plan, p) && aligned16(grad_out) && grad_row_stride % 4 == 0 && aligned16(W[p]) &&
                      aligned16(A[p]),
                  hot ? hot[p] : HotView{nullptr, nullptr, nullptr}};
        rc = k.dtype == PK_F32 ? dispatch_adagrad<float, 4>(ds, ps, k.dim, a)
                               : dispatch_adagrad<uint16_t, 8>(ds, ps, k.dim, a);
        if (rc != PK_OK) return rc;
    }
    if (n_side) { rc = join_streams(ds, stream, n_side); if (rc != PK_OK) return rc; }
    // long keys that cross tile boundaries, all packs at once
    const unsigned hgrid = blocks_for(nnz / L.pos_tile + 1, NT / 64, 1024);
    for (int p0 = 0; p0 < P; p0 += 16) {
        HotPacks hp{};
        const int np = std::min(16, P - p0);
        for (int i = 0; i < np; ++i) {
            hp.W[i] = W[p0 + i]; hp.A[i] = A[p0 + i];
            hp.hv[i] = hot ? hot[p0 + i] : HotView{nullptr, nullptr, nullptr};
        }
        PK_LAUNCH("pk_adagrad_hot", pk_adagrad_hot_kernel, dim3(hgrid, np), dim3(NT), 0, hp, p0, ds->pmeta, st,
                  ws.at<uint32_t>(L.unique), ws.at<int32_t>(L.seg), ws.at<double>(L.ghot), L.dmax,
                  ws.at<int4>(L.tile_hdr), L.pos_tile, lr, eps);
    }
    return PK_OK;
}

pk_status pk_backward_update(const pk_plan* plan, void* const* W, float* const* A, const float* grad_out,
                             int64_t grad_row_stride, int32_t B, int64_t nnz, float lr, float eps, void* workspace,
                             size_t ws_bytes, void* hip_stream)
{
    return backward_impl(plan, W, A, nullptr, grad_out, grad_row_stride, B, nnz, lr, eps, workspace, ws_bytes,
                         hip_stream);
}

// ---- HybridHash ------------------------------------------------------------------
static pk_status hh_check(const pk_plan* plan, const pk_hh_pack* packs, const char* who)
{
    if (!plan || !packs) return fail(PK_EINVAL, std::string(who) + ": NULL argument");
    for (size_t p = 0; p < plan->packs.size(); ++p) {
        const pk_hh_pack& h = packs[p];
        if (!h.W_cold || !h.A_cold || !h.slot_of || !h.fcounter || h.hot_rows < 0 ||
            (h.hot_rows > 0 && (!h.W_hot || !h.A_hot || !h.hot_row)))
            return fail(PK_EINVAL, std::string(who) + ": pack " + std::to_string(p) + " has a NULL buffer or a negative hot_rows");
        if (h.hot_rows >= ((int64_t)1 << 31)) return fail(PK_EOVERFLOW, std::string(who) + ": hot_rows must be below 2^31");
    }
    return PK_OK;
}

static void hh_views(const pk_plan* plan, const pk_hh_pack* packs, std::vector<void*>* W, std::vector<float*>* A,
                     std::vector<HotView>* hv)
{
    for (size_t p = 0; p < plan->packs.size(); ++p) {
        W->push_back(packs[p].W_cold);
        A->push_back(packs[p].A_cold);
        hv->push_back(HotView{packs[p].slot_of, packs[p].W_hot, packs[p].A_hot});
    }
}


static size_t hh_tiles(int64_t rows) { return (size_t)((rows + kHhTile - 1) / kHhTile); }

// scratch: histogram | per-pack counters | move counters | per-tile counts | slots to free | rows to load
struct HhScratch {
    size_t hist, counters, moves, tile_eq, evict, ins, total;
};

static HhScratch hh_scratch_layout(const pk_plan* plan, const pk_hh_pack* packs)
{
    size_t tiles = 0, hot = 0;
    for (size_t p = 0; p < plan->packs.size(); ++p) {
        tiles = std::max(tiles, hh_tiles(plan->packs[p].rows));
        hot = std::max(hot, (size_t)std::max<int64_t>(packs[p].hot_rows, 0));
    }
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    HhScratch L{};
    size_t off = 0;
    L.hist = off;     off += up((size_t)kHhBins * 4);
    L.counters = off; off += up(plan->packs.size() * 16);
    L.moves = off;    off += 256;
    L.tile_eq = off;  off += up(tiles * 4);
    L.evict = off;    off += up(hot * 4);
    L.ins = off;      off += up(hot * 4);
    L.total = off;
    return L;
}

size_t pk_hh_scratch_bytes(const pk_plan* plan, const pk_hh_pack* packs)
{
    if (!plan || !packs) { set_error("pk_hh_scratch_bytes: NULL argument"); return 0; }
    return hh_scratch_layout(plan, packs).total;
}

pk_status pk_hh_init(pk_plan* plan, const pk_hh_pack* packs, void* hip_stream)
{
    pk_status rc = hh_check(plan, packs, "pk_hh_init");
    if (rc != PK_OK) return rc;
    DeviceState* ds = nullptr;
    rc = ensure_device_state(plan, &ds);
    if (rc != PK_OK) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    ds->hh_n_hot.assign(plan->packs.size(), 0);
    for (size_t p = 0; p < plan->packs.size(); ++p) {
        const size_t rows = (size_t)plan->packs[p].rows;
        hipError_t e = hipMemsetAsync(packs[p].slot_of, 0xFF, rows * 4, stream);
        if (e == hipSuccess) e = hipMemsetAsync(packs[p].fcounter, 0, rows * 4, stream);
        if (e != hipSuccess) return fail(PK_EHIP, hip_msg("pk_hh_init", e));
    }
    return PK_OK;
}

pk_status pk_hh_forward(const pk_plan* plan, const pk_hh_pack* packs, const int64_t* ids, const int32_t* offsets,
                        int32_t B, int64_t nnz, float* out, int64_t out_row_stride, void* workspace,
                        size_t ws_bytes, void* hip_stream)
{
    pk_status rc = hh_check(plan, packs, "pk_hh_forward");
    if (rc != PK_OK) return rc;
    std::vector<void*> W; std::vector<float*> A; std::vector<HotView> hv;
    hh_views(plan, packs, &W, &A, &hv);
    return forward_impl(plan, nullptr, kDedup | kPool, "pk_hh_forward", W.data(), hv.data(), ids, offsets, B, nnz, out,
                        out_row_stride, workspace, ws_bytes,
                        hip_stream);
}

pk_status pk_hh_backward_update(const pk_plan* plan, const pk_hh_pack* packs, const float* grad_out,
                                int64_t grad_row_stride, int32_t B, int64_t nnz, float lr, float eps,
                                void* workspace, size_t ws_bytes, void* hip_stream)
{
    pk_status rc = hh_check(plan, packs, "pk_hh_backward_update");
    if (rc != PK_OK) return rc;
    std::vector<void*> W; std::vector<float*> A; std::vector<HotView> hv;
    hh_views(plan, packs, &W, &A, &hv);
    return backward_impl(plan, W.data(), A.data(), hv.data(), grad_out, grad_row_stride, B, nnz, lr, eps, workspace,
                         ws_bytes, hip_stream);
}

pk_status pk_hh_end_iteration(pk_plan* plan, const pk_hh_pack* packs, int64_t itr, int32_t warmup_iters,
                              int32_t flush_iters, int32_t B, int64_t nnz, const void* workspace, size_t ws_bytes,
                              void* scratch, size_t scratch_bytes, void* hip_stream, int64_t* queried, int64_t* hits,
                              int32_t* flushed)
{
    pk_status rc = hh_check(plan, packs, "pk_hh_end_iteration");
    if (rc != PK_OK) return rc;
    rc = check_common(plan, B, nnz, workspace, ws_bytes, "pk_hh_end_iteration");
    if (rc != PK_OK) return rc;
    if (itr < 0 || warmup_iters < 0 || flush_iters <= 0) return fail(PK_EINVAL, "pk_hh_end_iteration: bad iteration arguments");
    if (!scratch || reinterpret_cast<uintptr_t>(scratch) % kAlign || scratch_bytes < pk_hh_scratch_bytes(plan, packs))
        return fail(PK_EWORKSPACE, "pk_hh_end_iteration: scratch is NULL, misaligned or smaller than pk_hh_scratch_bytes");
    DeviceState* ds = nullptr;
    rc = ensure_device_state(plan, &ds);
    if (rc != PK_OK) return rc;
    const int P = (int)plan->packs.size();
    if ((int)ds->hh_n_hot.size() != P) return fail(PK_EINVAL, "pk_hh_end_iteration: pk_hh_init has not run on this plan");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Layout L = make_layout(plan, B, nnz);
    const char* wsb = static_cast<const char*>(workspace);
    const PackState* st = reinterpret_cast<const PackState*>(wsb + L.state);
    const uint32_t* unique = reinterpret_cast<const uint32_t*>(wsb + L.unique);
    char* sc = static_cast<char*>(scratch);
    const HhScratch S = hh_scratch_layout(plan, packs);
    uint32_t* hist = reinterpret_cast<uint32_t*>(sc + S.hist);
    unsigned long long* counters = reinterpret_cast<unsigned long long*>(sc + S.counters);
    uint32_t* moves = reinterpret_cast<uint32_t*>(sc + S.moves);
    int32_t* tile_eq = reinterpret_cast<int32_t*>(sc + S.tile_eq);
    int32_t* evict_slot = reinterpret_cast<int32_t*>(sc + S.evict);
    uint32_t* ins_row = reinterpret_cast<uint32_t*>(sc + S.ins);

    // FCounter (both branches of Alg. 1 count the queried IDs) and the hit statistics
    hipError_t e = hipMemsetAsync(counters, 0, (size_t)P * 16, stream);
    if (e != hipSuccess) return fail(PK_EHIP, hip_msg("pk_hh_end_iteration", e));
    for (int p = 0; p < P; ++p) {
        if (plan->packs[p].fields.empty()) continue;
        PK_LAUNCH("pk_hh_count", pk_hh_count_kernel, dim3(blocks_for(nnz, NT * 4, 1024)), dim3(NT), 0, st, p, unique,
                  packs[p].slot_of, packs[p].fcounter, counters);
    }
    const bool flush = itr >= warmup_iters && itr % flush_iters == 0;
    if (flushed) *flushed = flush ? 1 : 0;
    if (queried || hits) {
        std::vector<unsigned long long> c((size_t)P * 2);
        e = hipStreamSynchronize(stream);
        if (e == hipSuccess) e = hipMemcpy(c.data(), counters, c.size() * 8, hipMemcpyDeviceToHost);
        if (e != hipSuccess) return fail(PK_EHIP, hip_msg("pk_hh_end_iteration", e));
        for (int p = 0; p < P; ++p) {
            if (queried) queried[p] = (int64_t)c[2 * p];
            if (hits) hits[p] = (int64_t)c[2 * p + 1];
        }
    }
    if (!flush) return PK_OK;

    // reload: pick the top-k rows of FCounter; rows that leave are written back, rows that enter
    // are loaded, rows that stay are not touched
    std::vector<uint32_t> h_hist(kHhBins);
    for (int p = 0; p < P; ++p) {
        const Pack& k = plan->packs[p];
        const pk_hh_pack& h = packs[p];
        if (k.fields.empty() || h.hot_rows == 0) continue;
        e = hipMemsetAsync(hist, 0, (size_t)kHhBins * 4, stream);
        if (e == hipSuccess) e = hipMemsetAsync(moves, 0, 8, stream);
        if (e != hipSuccess) return fail(PK_EHIP, hip_msg("pk_hh_end_iteration", e));
        PK_LAUNCH("pk_hh_hist", pk_hh_hist_kernel, dim3(blocks_for(k.rows, NT * 64, 1024)), dim3(NT), 0, h.fcounter,
                  k.rows, hist);
        e = hipStreamSynchronize(stream);
        if (e == hipSuccess) e = hipMemcpy(h_hist.data(), hist, (size_t)kHhBins * 4, hipMemcpyDeviceToHost);
        if (e != hipSuccess) return fail(PK_EHIP, hip_msg("pk_hh_end_iteration", e));
        // threshold: the smallest count that still enters; rows above it all enter
        int64_t above = 0;
        uint32_t thr = 0;
        int64_t need_eq = 0;
        for (int b = kHhBins - 1; b >= 1; --b) {
            if (above + h_hist[b] >= h.hot_rows) { thr = (uint32_t)b; need_eq = h.hot_rows - above; break; }
            above += h_hist[b];
        }
        if (thr == 0) { thr = 1; need_eq = h_hist[1]; above -= h_hist[1]; }     // room for every queried row
        const int64_t n_new = above + std::min<int64_t>(need_eq, h_hist[thr]);
        if (n_new == 0) continue;
        const unsigned nt = (unsigned)hh_tiles(k.rows);
        PK_LAUNCH("pk_hh_tilecount", pk_hh_tilecount_kernel, dim3(nt), dim3(NT), 0, h.fcounter, k.rows, thr, tile_eq);
        PK_LAUNCH("pk_hh_scan", pk_hh_scan_kernel, dim3(1), dim3(1024), 0, tile_eq, (int)nt);
        PK_LAUNCH("pk_hh_diff", pk_hh_diff_kernel, dim3(nt), dim3(NT), 0, h.fcounter, k.rows, thr, (int)need_eq, tile_eq,
                  h.slot_of, evict_slot, ins_row, moves, h.hot_rows);
        rc = k.dtype == PK_F32 ? hh_swap<float>(ds, stream, h, ds->hh_n_hot[p], n_new, k.dim, evict_slot, ins_row, moves)
                               : hh_swap<uint16_t>(ds, stream, h, ds->hh_n_hot[p], n_new, k.dim, evict_slot, ins_row, moves);
        if (rc != PK_OK) return rc;
        ds->hh_n_hot[p] = n_new;
    }
    return PK_OK;
}

pk_status pk_hh_hot_count(const pk_plan* plan, int32_t p, int64_t* n_hot)
{
    if (!plan || !n_hot) return fail(PK_EINVAL, "pk_hh_hot_count: NULL argument");
    if (p < 0 || p >= (int32_t)plan->packs.size()) return fail(PK_EINVAL, "pk_hh_hot_count: pack out of range");
    const DeviceState* ds = static_cast<const DeviceState*>(plan->device_state);
    *n_hot = (ds && (size_t)p < ds->hh_n_hot.size()) ? ds->hh_n_hot[p] : 0;
    return PK_OK;
}

// ---- Partition: one GPU's share ------------------------------------------------------------
size_t pk_partition_scratch_bytes(const pk_plan* plan, int64_t nnz, int32_t n_owners)
{
    if (!plan || nnz < 0 || n_owners < 1 || n_owners > kPartOwnersMax) {
        set_error("pk_partition_scratch_bytes: plan is NULL, nnz negative or n_owners outside 1..64");
        return 0;
    }
    return (size_t)(nnz / kPartChunk + 2) * (size_t)n_owners * 4;
}

pk_status pk_partition_unique(const pk_plan* plan, const void* workspace, size_t ws_bytes, int32_t B, int64_t nnz,
                              int32_t p, int32_t n_owners, uint32_t* part_keys, int32_t* part_index,
                              int32_t* part_offsets, void* scratch, size_t scratch_bytes, void* hip_stream)
{
    pk_status rc = check_common(plan, B, nnz, workspace, ws_bytes, "pk_partition_unique");
    if (rc != PK_OK) return rc;
    if (p < 0 || p >= (int32_t)plan->packs.size()) return fail(PK_EINVAL, "pk_partition_unique: pack out of range");
    if (n_owners < 1 || n_owners > kPartOwnersMax) return fail(PK_EINVAL, "pk_partition_unique: n_owners must be 1 to 64");
    if (!part_keys || !part_index || !part_offsets) return fail(PK_EINVAL, "pk_partition_unique: NULL argument");
    if (!scratch || scratch_bytes < pk_partition_scratch_bytes(plan, nnz, n_owners))
        return fail(PK_EWORKSPACE, "pk_partition_unique: scratch is NULL or smaller than pk_partition_scratch_bytes");
    DeviceState* ds = nullptr;
    rc = ensure_device_state(plan, &ds);
    if (rc != PK_OK) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Layout L = make_layout(plan, B, nnz);
    const char* wsb = static_cast<const char*>(workspace);
    const PackState* st = reinterpret_cast<const PackState*>(wsb + L.state);
    const uint32_t* unique = reinterpret_cast<const uint32_t*>(wsb + L.unique);
    int32_t* counts = static_cast<int32_t*>(scratch);
    const unsigned grid = blocks_for(nnz / kPartChunk + 1, 1, 4096);
    PK_LAUNCH("pk_partition_count", pk_partition_count_kernel, dim3(grid), dim3(NT), 0, st, p, unique, n_owners, counts);
    PK_LAUNCH("pk_partition_scan", pk_partition_scan_kernel, dim3(1), dim3(kScanThreads), 0, st, p, n_owners, counts,
              part_offsets);
    PK_LAUNCH("pk_partition_place", pk_partition_place_kernel, dim3(grid), dim3(64), 0, st, p, unique, n_owners, counts,
              part_keys, part_index);
    return PK_OK;
}

pk_status pk_ctx_pack(const pk_plan* plan, const void* workspace, int32_t B, int64_t nnz, int32_t p,
                      const uint32_t** keys, const uint32_t** unique, const int32_t** inverse,
                      const int32_t** packed_offsets, const int32_t** seg_offsets, int64_t* nnz_p, int64_t* n_unique)
{
    if (!plan || !workspace) return fail(PK_EINVAL, "pk_ctx_pack: NULL argument");
    if (p < 0 || p >= (int32_t)plan->packs.size()) return fail(PK_EINVAL, "pk_ctx_pack: pack out of range");
    if (B <= 0 || nnz < 0) return fail(PK_ESHAPE, "pk_ctx_pack: bad B or nnz");
    const Layout L = make_layout(plan, B, nnz);
    const char* base = static_cast<const char*>(workspace);
    PackState s;
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(&s, base + L.state + (size_t)p * sizeof(PackState), sizeof(PackState), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(PK_EHIP, hip_msg("pk_ctx_pack", e));
    if (keys) *keys = reinterpret_cast<const uint32_t*>(base + L.keys) + s.start;
    if (unique) *unique = reinterpret_cast<const uint32_t*>(base + L.unique) + s.start;
    if (inverse) *inverse = reinterpret_cast<const int32_t*>(base + L.inverse) + s.start;
    if (packed_offsets) *packed_offsets = reinterpret_cast<const int32_t*>(base + L.packed_offsets) + po_off(plan, p, B);
    if (seg_offsets) *seg_offsets = reinterpret_cast<const int32_t*>(base + L.seg) + s.start + p;
    if (nnz_p) *nnz_p = s.nnz;
    if (n_unique) *n_unique = s.n_unique;
    return PK_OK;
}

pk_status pk_ctx_error(const pk_plan* plan, const void* workspace, int32_t* error_word)
{
    if (!plan || !workspace || !error_word) return fail(PK_EINVAL, "pk_ctx_error: NULL argument");
    std::vector<PackState> s(plan->packs.size());
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(s.data(), workspace, s.size() * sizeof(PackState), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(PK_EHIP, hip_msg("pk_ctx_error", e));
    *error_word = 0;
    for (size_t p = 0; p < s.size(); ++p) *error_word |= s[p].error;      // every pack keeps a word of its own
    return PK_OK;
}

pk_status pk_profile_enable(pk_plan* plan, int32_t enable)
{
    if (!plan) return fail(PK_EINVAL, "pk_profile_enable: plan is NULL");
    DeviceState* ds = nullptr;
    pk_status rc = ensure_device_state(plan, &ds);
    if (rc != PK_OK) return rc;
    ds->prof_on = enable != 0;
    if (!enable) { ds->recs.clear(); ds->events_used = 0; }
    return PK_OK;
}

int32_t pk_profile_read(pk_plan* plan, const char** names, double* total_ms, int64_t* launches, int32_t max_entries)
{
    if (!plan || !plan->device_state || !names || !total_ms || !launches) return 0;
    DeviceState* ds = static_cast<DeviceState*>(plan->device_state);
    (void)hipDeviceSynchronize();
    std::vector<const char*> order;
    std::map<const char*, std::pair<double, int64_t>> acc;
    for (const auto& r : ds->recs) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ds->events[r.e0], ds->events[r.e0 + 1]) != hipSuccess) continue;
        auto it = acc.find(r.name);
        if (it == acc.end()) { order.push_back(r.name); it = acc.emplace(r.name, std::make_pair(0.0, (int64_t)0)).first; }
        it->second.first += ms;
        it->second.second += 1;
    }
    ds->recs.clear();
    ds->events_used = 0;
    int32_t n = 0;
    for (const char* nm : order) {
        if (n >= max_entries) break;
        names[n] = nm; total_ms[n] = acc[nm].first; launches[n] = acc[nm].second;
        ++n;
    }
    return n;
}

}  // extern "C"
