// H1 and H2: packed keys, distinct keys (ascending), the inverse index and the per-key occurrence
// lists, by slices of the key space.
// Part of pk_device.hip: included there, in this order, inside its anonymous namespace.
//
// Unique (Sec. II-D) is a set over the pack's rows, so it is built where a set of rows is cheap:
// a table's key range is cut into slices of 2^k keys, and ONE block owns a slice.  In LDS it keeps
// the slice's bitmap (which rows occur), the popcount prefix of the bitmap's words (the index of a
// key among the slice's distinct keys is a prefix plus a popcount) and one counter per distinct
// key.  From those it writes, for its slice, the ascending distinct keys, the segment offsets, the
// headers of the backward tiles and the occurrences grouped by key -- everything the backward
// pass reads.  What a slice needs from the others is two numbers, the distinct keys and the
// occurrences of the slices before it in the pack; they travel through look-back descriptors.
//
// Which occurrences belong to a slice:
//   small batches   every slice block scans the IDs of its table's fields and keeps those whose
//                   row falls into its slice (the IDs of a table are few and sit in L2), so the
//                   whole dedup, with the pooling beside it, is ONE launch;
//   large batches   the occurrences are partitioned by slice first: the keys kernel counts them
//                   per slice (block-local counts in LDS, one global add per touched slice), a
//                   one-block scan turns the counts into places, a scatter kernel writes a
//                   (key in slice, bag) record per occurrence to its slice's place, and the slice
//                   kernel reads its records; the inverse index is then looked up per occurrence
//                   from the bitmap and rank samples the slice kernel leaves in memory.

// ---------------------------------------------------------------------------
// Field boundaries, and where each field's occurrences go in the packed order (fields in
// (pack, slot) order, one after the other).  s_fb [F+1], s_delta [F] (packed position minus
// position in ids), s_slotpos [F+1] (packed position of each (pack, slot)).  Returns non-zero
// when the boundaries are unusable (offsets[0] != 0, offsets[F*B] != nnz, or decreasing).
// ---------------------------------------------------------------------------
constexpr size_t field_scan_words(int F) { return (size_t)(3 * F + 2); }

template <int NTH>
__device__ __forceinline__ int field_scan(const int32_t* __restrict__ offsets, int B, int F, int64_t nnz,
                                          const int32_t* __restrict__ slot_field, int32_t* s_fb, int32_t* s_delta,
                                          int32_t* s_slotpos)
{
    const int tid = threadIdx.x;
    for (int f = tid; f <= F; f += NTH) s_fb[f] = offsets[(int64_t)f * B];
    __syncthreads();
    int mine = 0;
    for (int f = tid; f < F; f += NTH) mine |= s_fb[f + 1] < s_fb[f];
    if (tid == 0) mine |= (s_fb[0] != 0 || (int64_t)s_fb[F] != nnz);
    const int bad = __syncthreads_or(mine);
    int carry = 0;
    for (int base = 0; base < F; base += NTH) {
        const int i = base + tid;
        int len = 0, f = 0;
        if (i < F) {
            f = slot_field[i];
            len = bad ? 0 : s_fb[f + 1] - s_fb[f];
        }
        int tot;
        const int ex = block_excl_scan<NTH>(len, &tot);
        if (i < F) {
            s_slotpos[i] = carry + ex;
            s_delta[f] = carry + ex - s_fb[f];
        }
        carry += tot;
    }
    if (tid == 0) s_slotpos[F] = carry;
    __syncthreads();
    return bad;
}

// the same from the copy the keys kernel left in memory: fscan = s_fb | s_delta | s_slotpos | verdict
template <int NTH>
__device__ __forceinline__ int field_scan_load(const int32_t* __restrict__ fscan, int F, int32_t* s_fb)
{
    for (int i = threadIdx.x; i < 3 * F + 2; i += NTH) s_fb[i] = fscan[i];
    const int bad = fscan[3 * F + 2];
    __syncthreads();
    return bad;
}

// The cut of every table for this batch, from the field sizes the offsets give (s_fb: where every
// field's occurrences begin).  s_first [T+1]: the first slice of every table, in table-list order
// (slices are numbered over all packs); s_lg [T]: log2 of the keys per slice.
template <int NTH>
__device__ __forceinline__ void table_cut(const TableMeta* __restrict__ tmeta, const FieldMeta* __restrict__ fmeta,
                                          int T, int F, const int32_t* s_fb, int target, int log_max,
                                          int32_t* s_first, int32_t* s_lg, TableCut* out)
{
    for (int t = threadIdx.x; t < T; t += NTH) s_lg[t] = 0;       // first the tables' occurrences
    __syncthreads();
    for (int f = threadIdx.x; f < F; f += NTH) atomicAdd(&s_lg[fmeta[f].stable], max(s_fb[f + 1] - s_fb[f], 0));
    __syncthreads();
    int carry = 0;
    for (int base = 0; base < T; base += NTH) {
        const int t = base + (int)threadIdx.x;
        SliceGeom g{0, 0};
        int occ = 0;
        if (t < T) {
            occ = s_lg[t];
            g = slice_geom(tmeta[t].rows, occ, target, log_max);
        }
        int tot;
        const int ex = block_excl_scan<NTH>(g.n, &tot);
        if (t < T) {
            s_first[t] = carry + ex;
            s_lg[t] = g.log_keys;
            if (out) out[t] = TableCut{g.log_keys, g.n, carry + ex, occ};
        }
        carry += tot;
    }
    if (threadIdx.x == 0) s_first[T] = carry;
    __syncthreads();
}

// the same from the array the keys kernel wrote
template <int NTH>
__device__ __forceinline__ void table_cut_load(const TableCut* __restrict__ cut, int T, int32_t* s_first, int32_t* s_lg)
{
    for (int t = threadIdx.x; t < T; t += NTH) {
        const TableCut c = cut[t];
        s_first[t] = c.first;
        if (s_lg) s_lg[t] = c.log_keys;
        if (t == T - 1) s_first[T] = c.first + c.n;
    }
    if (T == 0 && threadIdx.x == 0) s_first[0] = 0;
    __syncthreads();
}

// the bag of field-local offsets `offs` [B+1] that holds position q (offsets that are not monotone give
// some bag of the field: the answer stays in range)
__device__ __forceinline__ int find_bag(const int32_t* __restrict__ offs, int B, int q, int guess)
{
    if ((unsigned)guess < (unsigned)B && offs[guess] <= q && q < offs[guess + 1]) return guess;
    int lo = 0, hi = B + 1;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (offs[mid] <= q) lo = mid + 1; else hi = mid;
    }
    return min(max(lo - 1, 0), B - 1);
}

// Large batches, first launch: the per-slice counters are zeroed by all blocks; block 0 clears the
// pack states and makes what every later kernel reads instead of deriving it again: the field scan
// (with its verdict), the cut of every table for this batch, and the packs' sizes.
constexpr int kSetupThreads = 1024;         // block 0's scans run over up to 4096 fields and tables
__global__ void __launch_bounds__(kSetupThreads)
pk_setup_kernel(uint4* zero, int64_t n4, const int32_t* __restrict__ offsets, int B, int F, int P, int T, int64_t nnz,
                int target, int log_max, const FieldMeta* __restrict__ fmeta, const PackMeta* __restrict__ pm,
                const TableMeta* __restrict__ tmeta, const int32_t* __restrict__ slot_field, PackState* st,
                int32_t* __restrict__ packed_offsets, int32_t* __restrict__ seg_all, TableCut* __restrict__ cut,
                int n_slices_max, int32_t* __restrict__ fscan)
{
    extern __shared__ int32_t s_dyn[];                     // block 0: field scan | first slices, slice sizes
    const uint4 z = make_uint4(0, 0, 0, 0);
    for (int64_t i = (int64_t)blockIdx.x * kSetupThreads + threadIdx.x; i < n4; i += (int64_t)gridDim.x * kSetupThreads) zero[i] = z;
    if (blockIdx.x != 0) return;
    int32_t* s_fb = s_dyn;
    int32_t* s_delta = s_fb + (F + 1);
    int32_t* s_slotpos = s_delta + F;
    int32_t* s_first = s_slotpos + (F + 1);
    int32_t* s_lg = s_first + (T + 1);
    const int tid = threadIdx.x;
    int bad = field_scan<kSetupThreads>(offsets, B, F, nnz, slot_field, s_fb, s_delta, s_slotpos);
    table_cut<kSetupThreads>(tmeta, fmeta, T, F, s_fb, target, log_max, s_first, s_lg, cut);
    bad |= s_first[T] > n_slices_max;                      // cannot be for offsets that pass the scan: the slices' arrays are that long
    for (int i = tid; i < 3 * F + 2; i += kSetupThreads) fscan[i] = s_fb[i];
    if (tid == 0) fscan[3 * F + 2] = bad;
    for (int p = tid; p < P; p += kSetupThreads) {
        const PackMeta k = pm[p];
        const int start = s_slotpos[k.first_slot];
        const int n = s_slotpos[k.first_slot + k.n_fields] - start;
        PackState ps{};
        ps.nnz = n; ps.start = start; ps.first_slice = s_first[k.first_stable]; ps.error = bad ? 1 : 0;
        st[p] = ps;
        if (k.n_stables == 0) seg_all[start + p] = 0;      // no table that a field reads: no slice writes the end of its segments
        packed_offsets[(int64_t)k.first_slot * B + p + (int64_t)k.n_fields * B] = n;
    }
}

// ---------------------------------------------------------------------------
// Large batches, H1: packed keys (Sec. III-B: one packed ID tensor per pack), packed bag offsets,
// and how many occurrences fall into every slice.  A tile is BT consecutive bags of ONE field, so
// its IDs are contiguous and hit one table; the tile's counts per slice are tallied in LDS and
// added to the slices' totals with one global add per touched slice.  The offsets of a tile are
// checked here: inside their field's range and not decreasing, else bit 0 of the pack's error
// word is raised and the tile is skipped (the kernels after this one skip that pack).
// ---------------------------------------------------------------------------
struct TileOf {
    int f, b0, nb;
    __device__ __forceinline__ TileOf(int64_t tile, int tiles_per_field, int B, int BT)
    {
        f = (int)(tile / tiles_per_field);
        b0 = (int)(tile - (int64_t)f * tiles_per_field) * BT;
        nb = min(BT, B - b0);
    }
};

template <int BT>
__global__ void __launch_bounds__(NT)
pk_keys_kernel(const int64_t* __restrict__ ids, const int32_t* __restrict__ offsets, int B, int F,
               const FieldMeta* __restrict__ fmeta, const PackMeta* __restrict__ pm, PackState* st,
               uint32_t* __restrict__ keys, int32_t* __restrict__ packed_offsets, int32_t* slice_total,
               const TableCut* __restrict__ cut, const int32_t* __restrict__ fscan, int32_t* __restrict__ tile_hist,
               int tile_hist_stride)
{
    extern __shared__ int32_t s_hist[];                    // the tile's counts per slice of its table
    __shared__ int32_t s_po[BT + 1];
    __shared__ int s_flag;
    const int tid = threadIdx.x;
    if (fscan[3 * F + 2]) return;                          // the field boundaries are unusable: the packs' error words say so
    const int32_t* fb = fscan;                             // where every field's occurrences begin
    const int32_t* delta = fscan + (F + 1);                // packed position minus position in ids, per field
    const int32_t* slotpos = delta + F;                    // packed position of each (pack, slot)
    const int tpf = (B + BT - 1) / BT;
    const int64_t n_tiles = (int64_t)F * tpf;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const TileOf tl(tile, tpf, B, BT);
        const int f = tl.f;
        const FieldMeta m = fmeta[f];
        const PackMeta k = pm[m.pack];
        const TableCut tc = cut[m.stable];
        const int f_lo = fb[f], f_hi = fb[f + 1];
        const int dl = delta[f];
        const int pbase = slotpos[k.first_slot];
        SliceGeom g;
        g.log_keys = tc.log_keys;
        g.n = tc.n;
        const int64_t g0 = (int64_t)f * B + tl.b0;
        __syncthreads();                                   // the previous tile's LDS is consumed
        for (int t = tid; t <= tl.nb; t += NT) s_po[t] = offsets[g0 + t];
        for (int s = tid; s < g.n; s += NT) s_hist[s] = 0;
        if (tid == 0) s_flag = 0;
        __syncthreads();
        for (int t = tid; t < tl.nb; t += NT)
            if (s_po[t] > s_po[t + 1] || s_po[t] < f_lo || s_po[t + 1] > f_hi) s_flag = 1;
        __syncthreads();
        if (s_flag) {
            if (tid == 0) atomicOr(&st[m.pack].error, 1);
            continue;
        }
        for (int t = tid; t < tl.nb; t += NT)
            packed_offsets[(int64_t)k.first_slot * B + m.pack + (int64_t)m.slot * B + tl.b0 + t] = s_po[t] + dl - pbase;
        const int q_lo = s_po[0], q_hi = s_po[tl.nb];
        for (int base = q_lo; base < q_hi; base += 4 * NT) {       // the same trips for every lane: lanes combine their counts
            int64_t idv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {                  // the loads of four rounds in flight together
                const int i = base + tid + j * NT;
                idv[j] = i < q_hi ? ids[i] : 0;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = base + tid + j * NT;
                const bool on = i < q_hi;
                const uint32_t kk = on ? fold_id(idv[j], m.rows, m.magic) : 0u;
                if (on) keys[i + dl] = m.base_row + kk;
                if (g.n <= kFewCounters) (void)lds_inc_few<false>(s_hist, kk >> g.log_keys, on, g.n);
                else if (on) atomicAdd(&s_hist[kk >> g.log_keys], 1);
            }
        }
        __syncthreads();
        const int slice0 = tc.first;
        for (int s = tid; s < g.n; s += NT) {
            const int c = s_hist[s];
            if (c) atomicAdd(&slice_total[slice0 + s], c);
            if (tile_hist) tile_hist[tile * tile_hist_stride + s] = c;     // the scatter kernel takes its counts from here
        }
    }
}

constexpr int kBigSlicesMax = 256;         // listed slices with many records
constexpr int kBigSliceFlag = 1 << 30;     // in SliceInfo::table: the slice is listed
constexpr int kBigSliceCount = 6144;       // records from which a slice is listed

// Large batches: the slices' totals become places.  A block takes 1024 slices; what lies before them
// it adds up itself (there are some thousand slices: a block reads a few values per thread).  Every slice
// gets its table, its index in the table, the place of its first record and the number of records; the
// cursors of the scatter kernel start at those places.
constexpr int kScanThreads = 1024;
__global__ void __launch_bounds__(kScanThreads)
pk_slice_scan_kernel(const TableCut* __restrict__ cut, int T,
                     const int32_t* __restrict__ slice_total, int32_t* __restrict__ slice_cursor,
                     SliceInfo* __restrict__ slice_info, int n_slices, int big_count, int32_t* n_big,
                     int32_t* __restrict__ big_list)
{
    extern __shared__ int32_t s_first[];                   // [T+1]
    table_cut_load<kScanThreads>(cut, T, s_first, nullptr);
    const int base = blockIdx.x * kScanThreads;
    int before = 0;
    for (int i = threadIdx.x; i < base; i += kScanThreads) before += slice_total[i];
    int carry;
    (void)block_excl_scan<kScanThreads>(before, &carry);
    const int s = base + (int)threadIdx.x;
    const int c = s < n_slices ? slice_total[s] : 0;
    int tot;
    const int ex = block_excl_scan<kScanThreads>(c, &tot);
    if (s < n_slices) {
        const int t = upper_bound_i32(s_first, T + 1, s) - 1;
        SliceInfo si;
        si.table = t; si.idx = s - s_first[t]; si.start = carry + ex; si.count = c;
        if (s >= s_first[T]) { si.table = -1; si.idx = 0; si.count = 0; }      // room for slices this batch does not have
        // A slice that holds a hot key has many times the records of the others: such slices are listed,
        // and blocks of four times the threads take them, in launches that run beside the others'.
        if (c > big_count && si.table >= 0) {
            const int at = atomicAdd(n_big, 1);
            if (at < kBigSlicesMax) {
                big_list[at] = s;
                si.table |= kBigSliceFlag;
            }
        }
        slice_info[s] = si;
        slice_cursor[s] = carry + ex;
    }
}

// Large batches: one record per occurrence, (key inside its slice, place of its bag's gradient chunk), written to
// the slice's place.  A tile counts its occurrences per slice in LDS, reserves room in every
// touched slice with one global add, and then places its records from block-local cursors.
template <int BT>
__global__ void __launch_bounds__(NT)
pk_scatter_kernel(const int32_t* __restrict__ offsets, int B, int F, int64_t nnz, int log_max,
                  const FieldMeta* __restrict__ fmeta, const TableCut* __restrict__ cut,
                  const PackState* __restrict__ st, const uint32_t* __restrict__ keys, int32_t* slice_cursor,
                  uint2* __restrict__ rec, int hist_words, int64_t out_dim, const int32_t* __restrict__ fscan,
                  const int32_t* __restrict__ tile_hist, int tile_hist_stride)
{
    extern __shared__ int32_t s_dyn[];                     // counts | places, per slice of the tile's table
    __shared__ int32_t s_po[BT + 1];
    int32_t* s_hist = s_dyn;
    int32_t* s_place = s_hist + hist_words;
    const int tid = threadIdx.x;
    if (fscan[3 * F + 2]) return;
    const int32_t* delta = fscan + (F + 1);
    const int tpf = (B + BT - 1) / BT;
    const int64_t n_tiles = (int64_t)F * tpf;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const TileOf tl(tile, tpf, B, BT);
        const int f = tl.f;
        const FieldMeta m = fmeta[f];
        if (st[m.pack].error) continue;                    // the keys kernel rejected offsets of this pack
        const TableCut tc = cut[m.stable];
        const int dl = delta[f];
        SliceGeom g;
        g.log_keys = tc.log_keys;
        g.n = tc.n;
        const int64_t g0 = (int64_t)f * B + tl.b0;
        __syncthreads();
        for (int t = tid; t <= tl.nb; t += NT) s_po[t] = offsets[g0 + t];
        for (int s = tid; s < g.n; s += NT) s_hist[s] = tile_hist ? tile_hist[tile * tile_hist_stride + s] : 0;
        __syncthreads();
        const int q_lo = s_po[0], q_hi = s_po[tl.nb];
        if (tile_hist) {
            // one word of every 128 bytes of the tile's keys, so that the placing pass finds them in the cache
            uint32_t pf = 0;
            for (int i = q_lo + tid * 32; i < q_hi; i += NT * 32) pf ^= keys[i + dl];
            asm volatile("" ::"v"(pf));
        }
        if (!tile_hist)                                    // (the keys kernel's counts of this tile were not kept)
        for (int base = q_lo; base < q_hi; base += 4 * NT) {      // four loads in flight
            uint32_t kv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + tid + u * NT;
                kv[u] = i < q_hi ? keys[i + dl] - m.base_row : 0xFFFFFFFFu;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t s = kv[u] >> g.log_keys;
                if (g.n <= kFewCounters) (void)lds_inc_few<false>(s_hist, s, s < (uint32_t)g.n, g.n);
                else if (s < (uint32_t)g.n) atomicAdd(&s_hist[s], 1);
            }
        }
        __syncthreads();
        const int slice0 = tc.first;
        for (int s = tid; s < g.n; s += NT) {
            const int c = s_hist[s];
            s_place[s] = c ? atomicAdd(&slice_cursor[slice0 + s], c) : 0;
            s_hist[s] = 0;
        }
        __syncthreads();
        // Every wavefront takes a contiguous quarter of the tile's positions, 64 at a time, so that a lane's
        // positions rise by 64 from one to the next: where bags are not short, the bag of a position is found
        // by stepping on from the bag of the lane's previous one (one search at the start).
        const int lane = tid & 63;
        const int per_wave = ((q_hi - q_lo + NT - 1) / NT) * 64;
        const int w_lo = q_lo + (tid >> 6) * per_wave, w_hi = min(w_lo + per_wave, q_hi);
        const bool stepped = (int64_t)tl.nb * 64 <= (int64_t)6 * (q_hi - q_lo);     // (short bags: a search per position is shorter)
        int t = stepped && w_lo + lane < w_hi ? upper_bound_i32(s_po, tl.nb + 1, w_lo + lane) - 1 : 0;
        constexpr int UP = 8;                              // key loads in flight (they come from memory: nothing has read them since they were written)
        for (int base = w_lo; base < w_hi; base += UP * 64) {
            uint32_t kv[UP];
#pragma unroll
            for (int u = 0; u < UP; ++u) {
                const int i = base + u * 64 + lane;
                kv[u] = i < w_hi ? keys[i + dl] - m.base_row : 0xFFFFFFFFu;
            }
#pragma unroll
            for (int u = 0; u < UP; ++u) {
                const int i = base + u * 64 + lane;
                const uint32_t kk = kv[u];
                const uint32_t s = kk >> g.log_keys;
                const bool valid = i < w_hi && s < (uint32_t)g.n;
                if (i < w_hi) {
                    if (stepped) { while (t + 1 < tl.nb && s_po[t + 1] <= i) ++t; }
                    else if (valid) t = upper_bound_i32(s_po, tl.nb + 1, i) - 1;
                }
                int at_local = 0;
                if (g.n <= kFewCounters) at_local = lds_inc_few<true>(s_hist, s, valid, g.n);   // (all lanes of the wavefront are here)
                else if (valid) at_local = atomicAdd(&s_hist[s], 1);
                if (!valid) continue;
                const int64_t at = (int64_t)s_place[s] + at_local;
                // the record: key inside the slice, the gradient's scale (bag length for mean pooling, 1 for sum;
                // 0 = too long for its bits, to be looked up) above it, and the place of the bag's gradient chunk
                uint32_t len = 1u;
                if (m.pool == PK_MEAN) {
                    const uint32_t L = (uint32_t)max(s_po[t + 1] - s_po[t], 1);
                    len = (L >> (32 - log_max)) ? 0u : L;
                }
                if ((uint64_t)at < (uint64_t)nnz)
                    rec[at] = make_uint2((kk - (s << g.log_keys)) | (len << log_max),
                                         (uint32_t)((int64_t)(tl.b0 + t) * out_dim + m.col));
            }
        }
    }
}

// ---------------------------------------------------------------------------
// The slice kernel's body.
// ---------------------------------------------------------------------------
// a field of a table as the slice blocks need it; static, device side, indexed like the table field list
struct TableField { int32_t field, slot, col, pool; };

struct SliceArgs {
    const TableMeta* tmeta; const TableField* tfields; int T;
    const PackMeta* pm; const int32_t* slot_field; PackState* st; int P;
    int F, B; int64_t nnz; int target, log_max;
    const int64_t* ids; const int32_t* offsets; const SmallSlice* small_slices;   // small batches: the block finds its occurrences itself
    const SliceInfo* slice_info; const uint2* rec;              // large batches: the slice's records
    const TableCut* cut;                                        // ... and the tables' cuts for this batch
    const FieldMeta* fmeta;
    int32_t* packed_offsets;
    uint32_t* keys; int32_t* inverse;                           // written here for small batches only
    uint32_t* bitmap; int32_t* slice_nu;                        // large batches only: bitmaps with rank samples, distinct keys per slice
    const int32_t* big_list; const int32_t* n_big;              // ... and the listed slices with many records
    uint32_t* unique; int32_t* seg_all; uint32_t* ent_all; int ent_mult;
    int4* tile_hdr; int tp; double* ghot; int dmax;
    uint64_t* desc; uint64_t* gdesc; int32_t* done; int n_slices;   // small batches: descriptors the library owns, cleaned by the last block
    int64_t out_dim;
#ifdef PK_PHASE_TIMES
    long long* ptimes;
#endif
};
#ifdef PK_PHASE_TIMES
#define PK_PT(a, blk, k) do { if (threadIdx.x == 0 && (a).ptimes) (a).ptimes[(size_t)(blk) * 16 + (k)] = wall_clock64(); } while (0)
#else
#define PK_PT(a, blk, k) do { } while (0)
#endif

// LDS words of a slice block: bitmap words | their popcount prefix | counters of a round of distinct keys.
// Small batches: the same words first hold the field scan, and the upper three quarters of the
// counters hold the slice's occurrences when they are few (12 bytes each, kept from the first pass over the IDs,
// so that the IDs are read once).
constexpr int slice_lds_words(int log_max, int ranks) { return 2 * (1 << (log_max - 5)) + ranks; }
constexpr int kSliceTfWords = 5;           // dynamic LDS words per field of a table

// one occurrence of a slice
struct SliceRec {
    uint32_t kl;       // key minus the slice's first key
    int32_t x;         // small batches: the field's index in the table's field list; large: the place of the gradient chunk
    int32_t q;         // small batches: position in ids
    int32_t b, L;      // small batches: bag of the field and its length, if known (b >= 0); large: L = the record's scale
};

// MODE: what the block does with its slice
//   kSliceFused  small batches: everything, occurrences found in the IDs, sums of the slices before it by look-back
//   kSliceMark   large batches, first half: which keys occur -> the slice's bitmap and its number of distinct keys
//   kSlicePlace  large batches, second half (after a scan of those numbers): everything else
// (With thousands of slices in flight a look-back makes every block wait for the slowest slice before it;
// two launches with a scan between them let every block run without waiting.)
enum { kSliceFused = 0, kSliceMark = 1, kSlicePlace = 2 };

template <int MODE, int NTH, int LOGMAX, int RANKS, bool BIG = false>
__device__ __forceinline__ void slice_body(const SliceArgs& a, int slice, int32_t* s_main, int32_t* s_tf)
{
    constexpr bool FROM_IDS = MODE == kSliceFused;
    constexpr bool GROUPED = FROM_IDS || BIG || NTH > 256;          // lanes that share a key combine their counter updates
    constexpr int WMAX = 1 << (LOGMAX - 5);
    constexpr int CACHE = FROM_IDS ? (RANKS * 3 / 4) / 3 : 0;      // occurrences kept in LDS (12 bytes each)
    static_assert(!FROM_IDS || (RANKS - 3 * CACHE >= CACHE), "cached occurrences need as many counters");
    constexpr int kBagBits = 20;                                   // of a cached occurrence's third word: its bag; above them its length
    constexpr uint32_t kLenMany = (1u << (32 - kBagBits)) - 1u;    // ... a length of this or more is looked up again
    static_assert(!FROM_IDS || slice_lds_words(LOGMAX, RANKS) >= 3 * 4096 + 2, "the field scan must fit the block's LDS");
    const int tid = threadIdx.x;
    uint32_t* s_bits = reinterpret_cast<uint32_t*>(s_main);
    uint32_t* s_pre = s_bits + WMAX;
    int32_t* s_cnt = s_main + 2 * WMAX;
    uint32_t* s_ckey = reinterpret_cast<uint32_t*>(s_cnt + (RANKS - 3 * CACHE));   // key inside the slice | field of the table
    uint32_t* s_cpos = s_ckey + CACHE;                                             // position in ids
    uint32_t* s_cbag = s_cpos + CACHE;                                             // bag | its length
    __shared__ uint32_t s_bc[4];
    __shared__ int s_ncache;
    const int F = a.F, B = a.B;
    const int64_t out_dim = a.out_dim;

    PK_PT(a, slice, 0);
    // ---- which slice, of which table; where the pack's arrays start ----
    int t, idx, lg, n_tslices, pack_first, is_last, p, nf, field_begin, pstart, nnz_p, rec_start = 0, rec_count = 0;
    uint32_t key_lo, rows, own_flags = 0;
    if (FROM_IDS) {
        const SmallSlice ss = a.small_slices[slice];
        t = ss.table; idx = ss.idx; lg = ss.log_keys; n_tslices = ss.n_table_slices; pack_first = ss.pack_first;
        is_last = ss.is_last; p = ss.pack; field_begin = ss.field_begin; nf = ss.field_end - ss.field_begin;
        key_lo = ss.key_lo; rows = ss.rows;
    } else {
        const SliceInfo si = a.slice_info[slice];
        if (si.table < 0) return;                                      // room for a slice this batch does not have
        if (BIG != ((si.table & kBigSliceFlag) != 0)) return;          // listed slices belong to the launch that takes the list
        t = si.table & ~kBigSliceFlag; idx = si.idx; rec_start = si.start; rec_count = si.count;
        const TableMeta tm = a.tmeta[t];
        p = tm.pack; field_begin = tm.field_begin; nf = tm.field_end - tm.field_begin; key_lo = tm.key_lo; rows = tm.rows;
        const TableCut tc = a.cut[t];
        lg = tc.log_keys; n_tslices = tc.n;
        pack_first = 0; is_last = 0;
    }
    const PackMeta k = a.pm[p];
    if (FROM_IDS) {
        int32_t* s_fb = s_main;
        int32_t* s_delta = s_fb + (F + 1);
        int32_t* s_slotpos = s_delta + F;
        const int bad = field_scan<NTH>(a.offsets, B, F, a.nnz, a.slot_field, s_fb, s_delta, s_slotpos);
        pstart = s_slotpos[k.first_slot];
        nnz_p = s_slotpos[k.first_slot + k.n_fields] - pstart;
        for (int j = tid; j < nf; j += NTH) {
            const TableField tf = a.tfields[field_begin + j];
            s_tf[kSliceTfWords * j] = s_fb[tf.field];
            s_tf[kSliceTfWords * j + 1] = s_fb[tf.field + 1];
            s_tf[kSliceTfWords * j + 2] = s_delta[tf.field];
            s_tf[kSliceTfWords * j + 3] = tf.col;
            s_tf[kSliceTfWords * j + 4] = tf.pool | (tf.field << 1);
        }
        __syncthreads();
        if (bad) {                                         // every block sees the same boundaries: nobody publishes, nobody waits
            if (is_last && tid == 0) { a.st[p].n_unique = 0; a.st[p].error = 1; }
            return;
        }
        // the offsets of this slice's share of the table's bags: inside the field and not decreasing
        int viol = 0;
        const int b_lo = (int)((int64_t)B * idx / n_tslices), b_hi = (int)((int64_t)B * (idx + 1) / n_tslices);
        for (int j = 0; j < nf; ++j) {
            const int32_t* offs = a.offsets + (int64_t)(s_tf[kSliceTfWords * j + 4] >> 1) * B;
            for (int b = b_lo + tid; b < b_hi; b += NTH) {
                const int o0 = offs[b], o1 = offs[b + 1];
                viol |= o0 > o1 || o0 < s_tf[kSliceTfWords * j] || o1 > s_tf[kSliceTfWords * j + 1];
            }
        }
        if (__syncthreads_or(viol)) own_flags |= 1u;
    } else {
        pstart = a.st[p].start;
        nnz_p = a.st[p].nnz;
        pack_first = a.st[p].first_slice;
        is_last = t == k.first_stable + k.n_stables - 1 && idx + 1 == n_tslices;   // last slice of the pack's last table
        if (a.st[p].error) return;                         // offsets of this pack were rejected: no block of it publishes or waits
        for (int j = tid; j < nf; j += NTH) {
            const TableField tf = a.tfields[field_begin + j];
            s_tf[kSliceTfWords * j] = tf.slot;
            s_tf[kSliceTfWords * j + 3] = tf.col;
            s_tf[kSliceTfWords * j + 4] = tf.pool;
        }
    }
    PK_PT(a, slice, 1);
    const uint64_t magic = FROM_IDS ? fold_magic(rows) : 0;  // (one division per block; the IDs are folded without)
    const uint32_t lo = (uint32_t)idx << lg;               // first key of the slice inside its table
    const uint32_t nkeys = min((uint32_t)1 << lg, rows - lo);
    const int words = 1 << (lg - 5);
    bool cached = false;
    int n_rec = 0;

    // all occurrences of the slice, in any order: fn(SliceRec, on).  Every lane makes the same trips and
    // calls fn every time, with on = false where it has no occurrence, so that fn may combine lanes.
    auto for_records = [&](auto&& fn) {
        if (FROM_IDS && cached) {
            for (int base = 0; base < n_rec; base += NTH) {
                const int i = base + tid;
                const bool on = i < n_rec;
                const uint32_t ek = on ? s_ckey[i] : 0u, eq = on ? s_cpos[i] : 0u, eb = on ? s_cbag[i] : 0u;
                const uint32_t L = eb >> kBagBits;
                fn(SliceRec{ek & ((1u << LOGMAX) - 1u), (int32_t)(ek >> LOGMAX), (int32_t)eq,
                            L == kLenMany ? -1 : (int32_t)(eb & ((1u << kBagBits) - 1u)), (int32_t)L}, on);
            }
        } else if (FROM_IDS) {
            for (int j = 0; j < nf; ++j) {
                const int q0 = s_tf[kSliceTfWords * j], q1 = s_tf[kSliceTfWords * j + 1];
                for (int base = q0; base < q1; base += 4 * NTH) {
                    int64_t idv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int i = base + tid + u * NTH;
                        idv[u] = i < q1 ? a.ids[i] : 0;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int i = base + tid + u * NTH;
                        const uint32_t kk = i < q1 ? fold_id(idv[u], rows, magic) : 0xFFFFFFFFu;
                        const bool on = i < q1 && (kk >> lg) == (uint32_t)idx;
                        fn(SliceRec{on ? kk - lo : 0u, j, i, -1, 0}, on);
                    }
                }
            }
        } else {
            const uint2* __restrict__ rec = a.rec + rec_start;
            constexpr int UN = BIG ? 8 : 4;                // records per thread in flight: a listed slice is long
            for (int base = 0; base < rec_count; base += UN * NTH) {
                uint2 r[UN];
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int i = base + tid + u * NTH;
                    r[u] = i < rec_count ? rec[i] : make_uint2(0xFFFFFFFFu, 0);
                }
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const uint32_t kl = r[u].x & ((1u << LOGMAX) - 1u);
                    const bool on = r[u].x != 0xFFFFFFFFu && kl < nkeys;
                    fn(SliceRec{on ? kl : 0u, (int32_t)r[u].y, 0, -1, (int32_t)(r[u].x >> LOGMAX)}, on);
                }
            }
        }
    };
    // the bag of an occurrence found in the IDs, and its length
    auto bag_of = [&](int j, int q, int* L) {
        const int32_t* offs = a.offsets + (int64_t)(s_tf[kSliceTfWords * j + 4] >> 1) * B;
        const int b = find_bag(offs, B, q, q - s_tf[kSliceTfWords * j]);
        *L = offs[b + 1] - offs[b];
        return b;
    };

    // ---- which keys occur ----
    // The slice's bitmap in memory: word w of the table's bitmap stands at w + w / 3 of the table's
    // region, so that every 16 bytes hold three words and, in the fourth, the rank of their first key.
    uint32_t* bmw = FROM_IDS ? nullptr : a.bitmap + a.tmeta[t].word_base;
    const uint32_t tw0 = (uint32_t)idx * (uint32_t)words;
    if (MODE == kSlicePlace) {
        for (int w = tid; w < words; w += NTH) s_bits[w] = bmw[tw0 + w + (tw0 + w) / 3u];
    } else {
        for (int w = tid; w < words; w += NTH) s_bits[w] = 0;
    }
    if (tid == 0) s_ncache = 0;
    __syncthreads();
    int mine = 0;
    if (MODE != kSlicePlace)
    for_records([&](const SliceRec& r, bool on) {
        if (on) {
            const uint32_t bit = 1u << (r.kl & 31);
            if (!(s_bits[r.kl >> 5] & bit)) atomicOr(&s_bits[r.kl >> 5], bit);
            ++mine;
        }
        if (FROM_IDS) {                                    // keep the occurrence while it is at hand
            const uint64_t m = __ballot(on);
            if (m) {
                const int lane = tid & 63, leader = __ffsll((unsigned long long)m) - 1;
                int base = 0;
                if (lane == leader) base = atomicAdd(&s_ncache, __popcll(m));
                base = __shfl(base, leader, 64);
                const int at = base + __popcll(m & ((1ull << lane) - 1ull));
                if (on && at < CACHE) { s_ckey[at] = r.kl | ((uint32_t)r.x << LOGMAX); s_cpos[at] = (uint32_t)r.q; }
            }
        }
    });
    (void)block_excl_scan<NTH>(mine, &n_rec);              // its barriers also complete the bitmap
    if (!FROM_IDS) n_rec = rec_count;
    cached = FROM_IDS && n_rec <= CACHE && B <= (1 << kBagBits);
    if (cached) {                                          // the bags of the kept occurrences, all lookups in flight together
        for (int i = tid; i < n_rec; i += NTH) {
            int L;
            const int b = bag_of((int)(s_ckey[i] >> LOGMAX), (int)s_cpos[i], &L);
            s_cbag[i] = (uint32_t)b | (min((uint32_t)max(L, 0), kLenMany) << kBagBits);
        }
    }
    PK_PT(a, slice, 2);
    // popcount prefix of the words: thread i owns words [i * wpt, (i + 1) * wpt)
    const int wpt = max(1, words / NTH);
    int c = 0;
    if (tid * wpt < words)
        for (int j = 0; j < wpt; ++j) c += __popc(s_bits[tid * wpt + j]);
    int n_u;
    const int ex = block_excl_scan<NTH>(c, &n_u);
    if (tid * wpt < words) {
        int run = ex;
        for (int j = 0; j < wpt; ++j) {
            s_pre[tid * wpt + j] = (uint32_t)run;
            run += __popc(s_bits[tid * wpt + j]);
        }
    }
    if (MODE == kSliceMark) {                              // the bitmap and the count go to memory; the rest follows the scan
        for (int w = tid; w < words; w += NTH) bmw[tw0 + w + (tw0 + w) / 3u] = s_bits[w];
        if (tid == 0) a.slice_nu[slice] = n_u;
        return;
    }
    // the counts of this slice are out early: the slices after it add them up while it goes on
    if (FROM_IDS && tid == 0)
        publish_desc(a.desc + slice, make_desc(slice == pack_first ? kDescPfx : kDescAgg, (uint32_t)n_u, (uint32_t)n_rec, own_flags));
    PK_PT(a, slice, 3);

    int base_u = 0, rec_before = 0;
    uint32_t* __restrict__ uq = a.unique + pstart;
    int32_t* __restrict__ seg = a.seg_all + pstart + p;
    // Distinct keys and occurrences of the pack's slices before this one; then what needs them: the slice's
    // distinct keys (ascending) in their place, bitmap and rank samples for the inverse kernel, the pack's
    // totals.  Returns false when the sums cannot be right (then nothing is written).
    auto after_lookback = [&]() -> bool {
        if (!FROM_IDS) {
            if (tid == 0) { s_bc[0] = (uint32_t)(a.slice_nu[slice] - a.slice_nu[pack_first]); s_bc[2] = 0; }   // scanned: distinct keys before
        } else if (tid < 64) {
            uint32_t pa = 0, pb = 0, pf = 0;
            if (slice != pack_first) {
                const int g0 = (pack_first >> 6) + p;      // the pack's first group descriptor (packs never share one)
                lookback_grouped(a.desc, a.gdesc, pack_first, g0, slice, (uint32_t)n_u, (uint32_t)n_rec, own_flags, &pa, &pb, &pf);
                if (tid == 0) {
                    const uint64_t incl = make_desc(kDescPfx, pa + (uint32_t)n_u, pb + (uint32_t)n_rec, pf | own_flags);
                    publish_desc(a.desc + slice, incl);
                    if (((slice - pack_first) & 63) == 63) publish_desc(a.gdesc + g0 + ((slice - pack_first) >> 6), incl);
                }
            }
            if (tid == 0) {
                s_bc[0] = pa; s_bc[1] = pb; s_bc[2] = pf | own_flags;
                if (FROM_IDS) {
                    // The descriptors belong to the library and must be zero when the next call starts: the
                    // block that finishes its look-back last (every block has then published, and read what
                    // it needed) clears them.  Reading the own descriptor back first makes sure that the
                    // store has arrived before this block counts as finished (same address: same order).
                    const uint64_t back = __hip_atomic_load(a.desc + slice, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    s_bc[3] = ((back >> 62) == kDescPfx && atomicAdd(a.done, 1) == a.n_slices - 1) ? 1u : 0u;
                }
            }
        }
        __syncthreads();
        PK_PT(a, slice, 4);
        base_u = (int)s_bc[0];
        rec_before = FROM_IDS ? (int)s_bc[1] : rec_start - pstart;
        const uint32_t flags = s_bc[2];
        if (FROM_IDS && s_bc[3]) {
            for (int i = tid; i < a.n_slices; i += NTH) publish_desc(a.desc + i, 0);
            for (int i = tid; i < (a.n_slices >> 6) + a.P + 2; i += NTH) publish_desc(a.gdesc + i, 0);
            if (tid == 0) *a.done = 0;
        }
        // whatever the descriptors held, no write below leaves the pack's arrays
        if (base_u < 0 || rec_before < 0 || (int64_t)base_u + n_u > (int64_t)nnz_p ||
            (int64_t)rec_before + n_rec > (int64_t)nnz_p) {
            if (tid == 0) atomicOr(&a.st[p].error, 2);
            return false;
        }
        if (tid * wpt < words) {
            for (int j = 0; j < wpt; ++j) {
                const int w = tid * wpt + j;
                uint32_t x = s_bits[w];
                int at = base_u + (int)s_pre[w];
                const uint32_t key0 = key_lo + lo + (uint32_t)w * 32u;
                while (x) {
                    const int bit = __ffs(x) - 1;
                    x &= x - 1;
                    uq[at++] = key0 + bit;
                }
            }
        }
        if (!FROM_IDS) {                                   // rank samples beside the bitmap, for the inverse kernel
            for (uint32_t u = (tw0 + 2u) / 3u + tid; 3u * u < tw0 + (uint32_t)words; u += NTH)
                bmw[4u * u + 3u] = (uint32_t)(base_u + (int)s_pre[3u * u - tw0]);
        }
        if (is_last && tid == 0) {
            a.st[p].n_unique = base_u + n_u;
            seg[base_u + n_u] = nnz_p;
            if (FROM_IDS) a.st[p].error = (int32_t)flags;
            else if (flags) atomicOr(&a.st[p].error, (int32_t)flags);
        }
        PK_PT(a, slice, 5);
        return true;
    };
    if (n_u == 0) {
        (void)after_lookback();
        return;
    }

    // ---- occurrences per distinct key, segment offsets, headers of the backward tiles, and every
    //      occurrence's gradient place at its key's next free position; a round handles RANKS keys ----
    const int tp = a.tp, dim = k.dim;
    const bool wide = k.has_mean != 0;                     // the pack's entries carry the bag length
    uint32_t* __restrict__ ent = a.ent_all + (size_t)pstart * a.ent_mult;
    const size_t tbase = (size_t)(pstart / tp + p);
    int4* th = a.tile_hdr + tbase;
    double* gh = a.ghot + tbase * a.dmax;
    const int32_t* __restrict__ po = a.packed_offsets + (int64_t)k.first_slot * B + p;
    auto rank_of = [&](uint32_t kl) {
        return (int)(s_pre[kl >> 5] + __popc(s_bits[kl >> 5] & ((1u << (kl & 31)) - 1u)));
    };
    const int rounds_cap = cached ? RANKS - 3 * CACHE : RANKS;      // cached occurrences take the upper counters' room
    int placed = 0;                                        // occurrences of the keys of earlier rounds
    for (int r0 = 0; r0 < n_u; r0 += rounds_cap) {
        const int width = min(rounds_cap, n_u - r0);
        __syncthreads();
        for (int i = tid; i < width; i += NTH) s_cnt[i] = 0;
        __syncthreads();
        for_records([&](const SliceRec& r, bool on) {
            const uint32_t rr = (uint32_t)(rank_of(r.kl) - r0);
            if (GROUPED) (void)lds_inc_grouped(s_cnt, rr, on && rr < (uint32_t)width);
            else if (on && rr < (uint32_t)width) atomicAdd(&s_cnt[rr], 1);
        });
        __syncthreads();
        PK_PT(a, slice, 6);
        const int per = (width + NTH - 1) / NTH;           // consecutive counters per thread
        int sum = 0;
        for (int j = 0; j < per; ++j) {
            const int i = tid * per + j;
            sum += i < width ? s_cnt[i] : 0;
        }
        int tot;
        const int ex_occ = block_excl_scan<NTH>(sum, &tot);
        if (r0 == 0 && !after_lookback()) return;          // the same for every thread
        int s0 = rec_before + placed + ex_occ;
        for (int j = 0; j < per; ++j) {
            const int i = tid * per + j;
            if (i < width) {
                const int len = s_cnt[i];
                const int u = base_u + r0 + i;
                seg[u] = s0;
                s_cnt[i] = s0;                             // from here on: the segment's next free position
                // headers of the backward tiles the segment overlaps: x = the key that holds the
                // tile's first position, y = the key that holds its last one, z = where the
                // tile's decoded window ends (its last key is decoded to its end unless it is long)
                for (int tt = s0 / tp; (int64_t)tt * tp < (int64_t)s0 + len; ++tt) {
                    const int t_first = tt * tp, t_end = min(t_first + tp, nnz_p);
                    if (t_first >= s0) th[tt].x = u;
                    if (t_end - 1 < s0 + len) {
                        th[tt].y = u;
                        th[tt].z = len <= kWarmMax ? s0 + len : t_end;
                    }
                }
                if (len > kWarmMax && s0 / tp != (s0 + len - 1) / tp) {
                    const int slot = s0 / tp;              // one such key at most starts in a tile
                    for (int d = 0; d < dim; ++d) gh[(size_t)slot * dim + d] = 0.0;
                }
                s0 += len;
            }
        }
        __syncthreads();
        PK_PT(a, slice, 7);
        for_records([&](const SliceRec& r, bool on) {
            const int rk = rank_of(r.kl);
            const uint32_t rr = (uint32_t)(rk - r0);
            on = on && rr < (uint32_t)width;
            int pos = 0;
            if (GROUPED) pos = lds_inc_grouped(s_cnt, rr, on);
            if (!on) return;
            if (!GROUPED) pos = atomicAdd(&s_cnt[rr], 1);
            uint32_t ref, len = 1u;
            if (FROM_IDS) {
                int L = r.L, b = r.b;
                if (b < 0) b = bag_of(r.x, r.q, &L);
                ref = (uint32_t)((int64_t)b * out_dim + s_tf[kSliceTfWords * r.x + 3]);
                if ((s_tf[kSliceTfWords * r.x + 4] & 1) == PK_MEAN && L > 0) len = (uint32_t)L;
                const int qp = r.q + s_tf[kSliceTfWords * r.x + 2];
                if ((unsigned)qp < (unsigned)a.nnz) {
                    a.keys[qp] = key_lo + lo + r.kl;
                    a.inverse[qp] = base_u + rk;
                }
            } else {
                ref = (uint32_t)r.x;                       // the record holds the place of the gradient chunk
                if (wide) {
                    len = (uint32_t)r.L;
                    if (len == 0) {                        // a bag too long for the record's bits: its length from the bag
                        const uint32_t b = ref / (uint32_t)out_dim, col = ref - b * (uint32_t)out_dim;
                        int j = 0;
                        while (j + 1 < nf && (uint32_t)s_tf[kSliceTfWords * j + 3] != col) ++j;
                        const uint32_t g = (uint32_t)s_tf[kSliceTfWords * j] * (uint32_t)B + b;
                        len = (uint32_t)max(po[g + 1] - po[g], 1);
                    }
                }
            }
            if ((unsigned)pos < (unsigned)nnz_p) {
                if (wide) reinterpret_cast<uint2*>(ent)[pos] = make_uint2(ref, len);
                else ent[pos] = ref;
            }
        });
        placed += tot;
    }

    __syncthreads();
    PK_PT(a, slice, 8);
}

// Large batches: one block per slice, in two launches with a scan between them.
constexpr int kFineThreads = 256, kFineRanks = 2048;
constexpr int kSliceThreads = 1024, kSliceRanks = 8192;

template <int MODE>
__global__ void __launch_bounds__(kFineThreads, 8)
pk_slices_kernel(SliceArgs a)
{
    extern __shared__ int32_t s_dyn[];
    __shared__ int32_t s_main[slice_lds_words(kSliceLogFine, kFineRanks)];
    slice_body<MODE, kFineThreads, kSliceLogFine, kFineRanks>(a, blockIdx.x, s_main, s_dyn);
}

// ... the listed slices with many records: four times the threads, same cut
template <int MODE>
__global__ void __launch_bounds__(kSliceThreads)
pk_slices_big_kernel(SliceArgs a)
{
    extern __shared__ int32_t s_dyn[];
    __shared__ int32_t s_main[slice_lds_words(kSliceLogFine, kSliceRanks)];
    if ((int)blockIdx.x >= min(*a.n_big, kBigSlicesMax)) return;
    slice_body<MODE, kSliceThreads, kSliceLogFine, kSliceRanks, true>(a, a.big_list[blockIdx.x], s_main, s_dyn);
}

// ... and the shape for calls with a table too long for slices of 32 K keys
template <int MODE>
__global__ void __launch_bounds__(kSliceThreads)
pk_slices_wide_kernel(SliceArgs a)
{
    extern __shared__ int32_t s_dyn[];
    __shared__ int32_t s_main[slice_lds_words(kSliceLogMax, kSliceRanks)];
    slice_body<MODE, kSliceThreads, kSliceLogMax, kSliceRanks>(a, blockIdx.x, s_main, s_dyn);
}

// Large batches: the slices' numbers of distinct keys become running sums, in place (exclusive, over all
// packs; a slice takes the difference to its pack's first slice).  Blocks as in the scan of the records.
__global__ void __launch_bounds__(kScanThreads)
pk_unique_scan_kernel(int32_t* __restrict__ slice_nu, int n_slices, int32_t* __restrict__ sums)
{
    const int base = blockIdx.x * kScanThreads;
    int before = 0;
    for (int i = threadIdx.x; i < base; i += kScanThreads) before += slice_nu[i];
    int carry;
    (void)block_excl_scan<kScanThreads>(before, &carry);
    const int s = base + (int)threadIdx.x;
    const int c = s < n_slices ? slice_nu[s] : 0;
    int tot;
    const int ex = block_excl_scan<kScanThreads>(c, &tot);
    if (s < n_slices) sums[s] = carry + ex;
}

// Small batches: the blocks beside the slice blocks that write what is per bag and per pack:
// packed bag offsets and the packs' sizes.  (The slice blocks check the offsets.)
__device__ __forceinline__ void meta_body(const SliceArgs& a, int block, int nblocks, int32_t* s_main)
{
    const int F = a.F, B = a.B, P = a.P, tid = threadIdx.x;
    int32_t* s_fb = s_main;
    int32_t* s_delta = s_fb + (F + 1);
    int32_t* s_slotpos = s_delta + F;
    const int bad = field_scan<kSliceThreads>(a.offsets, B, F, a.nnz, a.slot_field, s_fb, s_delta, s_slotpos);
    if (block == 0) {
        for (int p = tid; p < P; p += kSliceThreads) {
            const PackMeta k = a.pm[p];
            const int start = s_slotpos[k.first_slot];
            const int n = s_slotpos[k.first_slot + k.n_fields] - start;
            a.st[p].nnz = n;
            a.st[p].start = start;
            a.st[p].first_slice = 0;
            if (k.n_stables == 0) {                        // no slice block writes these
                a.st[p].n_unique = 0;
                a.st[p].error = bad ? 1 : 0;
                a.seg_all[start + p] = 0;
            }
            a.packed_offsets[(int64_t)k.first_slot * B + p + (int64_t)k.n_fields * B] = n;
        }
    }
    if (bad) return;
    int32_t* po = a.packed_offsets;
    const int64_t n_bags = (int64_t)F * B;
    for (int64_t g = (int64_t)block * kSliceThreads + tid; g < n_bags; g += (int64_t)nblocks * kSliceThreads) {
        const int f = (int)(g / B);
        const int b = (int)(g - (int64_t)f * B);
        const FieldMeta m = a.fmeta[f];
        const PackMeta k = a.pm[m.pack];
        const int o = min(max(a.offsets[g], s_fb[f]), s_fb[f + 1]);
        po[(int64_t)k.first_slot * B + m.pack + (int64_t)m.slot * B + b] = o + s_delta[f] - s_slotpos[k.first_slot];
    }
}

// ---------------------------------------------------------------------------
// Large batches: inverse[q] = number of distinct keys of the pack below key[q]: the rank sample that
// stands beside the key's three bitmap words (written by the slice kernel) plus the set bits before
// the key among them: one 16-byte read per position.  Tiles of KT consecutive positions of the packed order (all packs in one launch); which
// table a position belongs to follows from where its field's occurrences start, staged in LDS with
// the table's first key and the place of its bitmap.
// ---------------------------------------------------------------------------
template <int KT>
__global__ void __launch_bounds__(NT)
pk_inverse_kernel(int F, const int32_t* __restrict__ fscan, const SlotMeta* __restrict__ slot_meta,
                  const PackState* __restrict__ st, const uint32_t* __restrict__ keys,
                  const uint4* __restrict__ bitmap4, int32_t* __restrict__ inverse)
{
    extern __shared__ int32_t s_dyn[];                     // field scan | per slot: first key, bitmap place, rows, the pack's error word
    int32_t* s_fb = s_dyn;
    int32_t* s_slotpos = s_fb + (F + 1) + F;
    uint32_t* s_klo = reinterpret_cast<uint32_t*>(s_slotpos + (F + 1));
    uint32_t* s_wb = s_klo + F;
    uint32_t* s_rows = s_wb + F;
    int32_t* s_pack = reinterpret_cast<int32_t*>(s_rows + F);
    for (int j = threadIdx.x; j < F; j += NT) {
        const SlotMeta m = slot_meta[j];
        s_klo[j] = m.key_lo; s_wb[j] = m.word_base; s_rows[j] = m.rows; s_pack[j] = st[m.pack].error;   // (the error word, final by now)
    }
    if (field_scan_load<NT>(fscan, F, s_fb)) return;
    const int n = s_slotpos[F];
    const int n_tiles = (n + KT - 1) / KT;
    for (XcdTiles it(n_tiles); it.valid(); it.next()) {
        uint32_t key[KT / NT];
#pragma unroll
        for (int k = 0; k < KT / NT; ++k) {
            const int q = it.tile * KT + k * NT + (int)threadIdx.x;
            key[k] = q < n ? keys[q] : 0;
        }
        // the lookups of the tile's positions are all asked for before any is used
        int j = -1;
        uint32_t kk[KT / NT];
        uint4 x[KT / NT];
        bool ok[KT / NT];
#pragma unroll
        for (int k = 0; k < KT / NT; ++k) {
            const int q = it.tile * KT + k * NT + (int)threadIdx.x;
            ok[k] = q < n;
            kk[k] = 0;
            x[k] = make_uint4(0, 0, 0, 0);
            if (ok[k]) {
                if (j < 0 || q >= s_slotpos[j + 1]) j = upper_bound_i32(s_slotpos, F + 1, q) - 1;   // the slot of this position
                kk[k] = key[k] - s_klo[j];
                // no lookup for a pack with rejected offsets, nor for a key that is none of its table (only possible then)
                ok[k] = s_pack[j] == 0 && kk[k] < s_rows[j];
                if (ok[k]) x[k] = bitmap4[(size_t)s_wb[j] / 4 + (kk[k] >> 5) / 3u];
            }
        }
#pragma unroll
        for (int k = 0; k < KT / NT; ++k) {
            const int q = it.tile * KT + k * NT + (int)threadIdx.x;
            const uint32_t tw = kk[k] >> 5;
            const int wi = (int)(tw - tw / 3u * 3u);
            const uint32_t w[3] = {x[k].x, x[k].y, x[k].z};
            int r = (int)x[k].w;                           // the rank of the 16 bytes' first key
            uint32_t cur = 0;
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                if (i < wi) r += __popc(w[i]);
                if (i == wi) cur = w[i];
            }
            r += __popc(cur & ((1u << (kk[k] & 31)) - 1u));
            if (ok[k]) inverse[q] = r;
        }
    }
}

// ---------------------------------------------------------------------------
// Partition (Sec. II-D operator list; Sec. III-B fuses it with Unique): one GPU's share of it.  With the
// rows of a packed table dealt to n workers by row mod n, the distinct keys of a pack are regrouped by
// owner -- owner 0 first, ascending inside an owner -- with the place of every key in `unique` beside it
// (what Stitch needs for the rows that come back) and the offsets of the owners' groups.  A counting
// sort in three small launches: counts per chunk of 512 keys and owner, a scan in owner-major order,
// and the placing pass (a wavefront per chunk, so that the order inside an owner is the key order).
// ---------------------------------------------------------------------------
constexpr int kPartChunk = 512;
constexpr int kPartOwnersMax = 64;

__global__ void __launch_bounds__(NT)
pk_partition_count_kernel(const PackState* __restrict__ st, int p, const uint32_t* __restrict__ unique_all,
                          int n_owners, int32_t* __restrict__ chunk_counts)
{
    __shared__ int s_cnt[kPartOwnersMax];
    const int U = st[p].n_unique;
    const uint32_t* uq = unique_all + st[p].start;
    const int n_chunks = (U + kPartChunk - 1) / kPartChunk;
    for (int ch = blockIdx.x; ch < n_chunks; ch += gridDim.x) {
        __syncthreads();
        if (threadIdx.x < kPartOwnersMax) s_cnt[threadIdx.x] = 0;
        __syncthreads();
        for (int i = ch * kPartChunk + threadIdx.x; i < min((ch + 1) * kPartChunk, U); i += NT)
            atomicAdd(&s_cnt[uq[i] % (uint32_t)n_owners], 1);
        __syncthreads();
        if ((int)threadIdx.x < n_owners) chunk_counts[(size_t)threadIdx.x * n_chunks + ch] = s_cnt[threadIdx.x];   // owner-major
    }
}

// exclusive scan of the owner-major counts, in place; the owners' offsets on the way (one block)
__global__ void __launch_bounds__(kScanThreads)
pk_partition_scan_kernel(const PackState* __restrict__ st, int p, int n_owners, int32_t* chunk_counts,
                         int32_t* __restrict__ offsets)
{
    const int U = st[p].n_unique;
    const int n_chunks = (U + kPartChunk - 1) / kPartChunk;
    const int total = n_owners * n_chunks;
    int carry = 0;
    for (int base = 0; base < total; base += kScanThreads) {
        const int i = base + (int)threadIdx.x;
        const int c = i < total ? chunk_counts[i] : 0;
        int tot;
        const int ex = block_excl_scan<kScanThreads>(c, &tot);
        if (i < total) {
            chunk_counts[i] = carry + ex;
            if (i % n_chunks == 0) offsets[i / n_chunks] = carry + ex;
        }
        carry += tot;
    }
    if (threadIdx.x == 0) {
        offsets[n_owners] = U;
        if (n_chunks == 0) for (int o = 0; o < n_owners; ++o) offsets[o] = 0;
    }
}

__global__ void __launch_bounds__(64)
pk_partition_place_kernel(const PackState* __restrict__ st, int p, const uint32_t* __restrict__ unique_all,
                          int n_owners, const int32_t* __restrict__ chunk_offsets, uint32_t* __restrict__ part_keys,
                          int32_t* __restrict__ part_index)
{
    const int U = st[p].n_unique, lane = threadIdx.x;
    const uint32_t* uq = unique_all + st[p].start;
    const int n_chunks = (U + kPartChunk - 1) / kPartChunk;
    const uint64_t below = (1ull << lane) - 1ull;
    for (int ch = blockIdx.x; ch < n_chunks; ch += gridDim.x) {
        int cur = lane < n_owners ? chunk_offsets[(size_t)lane * n_chunks + ch] : 0;   // lane o: owner o's next place
        for (int base = ch * kPartChunk; base < min((ch + 1) * kPartChunk, U); base += 64) {
            const int i = base + lane;
            const bool on = i < U;
            const uint32_t key = on ? uq[i] : 0u;
            const int o = on ? (int)(key % (uint32_t)n_owners) : -1;
            int rank = 0, add = 0;
            for (int ov = 0; ov < n_owners; ++ov) {        // lanes are in key order: rank among the owner's lanes
                const uint64_t m = __ballot(o == ov);
                if (o == ov) rank = __popcll(m & below);
                if (lane == ov) add = __popcll(m);
            }
            const int at = __shfl(cur, on ? o : 0, 64) + rank;
            if (on) {
                part_keys[at] = key;
                part_index[at] = i;
            }
            cur += add;
        }
    }
}
