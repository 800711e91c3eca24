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

// s_first [T+1]: the first slice of every table, in table-list order (slices are numbered over all packs)
template <int NTH>
__device__ __forceinline__ void table_scan(const TableMeta* __restrict__ tmeta, int T, int F, int64_t nnz, int target,
                                           int32_t* s_first)
{
    int carry = 0;
    for (int base = 0; base < T; base += NTH) {
        const int t = base + (int)threadIdx.x;
        int n = 0;
        if (t < T) {
            const TableMeta tm = tmeta[t];
            n = slice_geom(tm.rows, tm.field_end - tm.field_begin, F, nnz, target).n;
        }
        int tot;
        const int ex = block_excl_scan<NTH>(n, &tot);
        if (t < T) s_first[t] = carry + ex;
        carry += tot;
    }
    if (threadIdx.x == 0) s_first[T] = carry;
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

__global__ void __launch_bounds__(NT)
pk_clear_kernel(uint4* p, int64_t n4)
{
    const uint4 z = make_uint4(0, 0, 0, 0);
    for (int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x; i < n4; i += (int64_t)gridDim.x * NT) p[i] = z;
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
pk_keys_kernel(const int64_t* __restrict__ ids, const int32_t* __restrict__ offsets, int B, int F, int P, int T,
               int64_t nnz, int target, const FieldMeta* __restrict__ fmeta, const PackMeta* __restrict__ pm,
               const TableMeta* __restrict__ tmeta, const int32_t* __restrict__ slot_field, PackState* st,
               uint32_t* __restrict__ keys, int32_t* __restrict__ packed_offsets, int32_t* slice_total,
               int32_t* __restrict__ seg_all)
{
    extern __shared__ int32_t s_dyn[];                     // field scan | first slices | the tile's counts
    __shared__ int32_t s_po[BT + 1];
    __shared__ int s_flag;
    int32_t* s_fb = s_dyn;
    int32_t* s_delta = s_fb + (F + 1);
    int32_t* s_slotpos = s_delta + F;
    int32_t* s_first = s_slotpos + (F + 1);
    int32_t* s_hist = s_first + (T + 1);
    const int tid = threadIdx.x;
    const int bad = field_scan<NT>(offsets, B, F, nnz, slot_field, s_fb, s_delta, s_slotpos);
    table_scan<NT>(tmeta, T, F, nnz, target, s_first);
    if (blockIdx.x == 0) {
        for (int p = tid; p < P; p += NT) {
            const PackMeta k = pm[p];
            const int start = s_slotpos[k.first_slot];
            const int n = s_slotpos[k.first_slot + k.n_fields] - start;
            st[p].nnz = n;
            st[p].start = start;
            st[p].first_slice = s_first[k.first_stable];
            if (bad) atomicOr(&st[p].error, 1);            // the clearing kernel zeroed the word
            if (k.n_stables == 0) seg_all[start + p] = 0;  // no table that a field reads: no slice writes the end of its segments
            packed_offsets[(int64_t)k.first_slot * B + p + (int64_t)k.n_fields * B] = n;
        }
    }
    if (bad) return;
    const int tpf = (B + BT - 1) / BT;
    const int64_t n_tiles = (int64_t)F * tpf;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const TileOf tl(tile, tpf, B, BT);
        const int f = tl.f;
        const FieldMeta m = fmeta[f];
        const PackMeta k = pm[m.pack];
        const TableMeta tm = tmeta[m.stable];
        const SliceGeom g = slice_geom(tm.rows, tm.field_end - tm.field_begin, F, nnz, target);
        const int64_t g0 = (int64_t)f * B + tl.b0;
        __syncthreads();                                   // the previous tile's LDS is consumed
        for (int t = tid; t <= tl.nb; t += NT) s_po[t] = offsets[g0 + t];
        for (int s = tid; s < g.n; s += NT) s_hist[s] = 0;
        if (tid == 0) s_flag = 0;
        __syncthreads();
        for (int t = tid; t < tl.nb; t += NT)
            if (s_po[t] > s_po[t + 1] || s_po[t] < s_fb[f] || s_po[t + 1] > s_fb[f + 1]) s_flag = 1;
        __syncthreads();
        if (s_flag) {
            if (tid == 0) atomicOr(&st[m.pack].error, 1);
            continue;
        }
        const int dl = s_delta[f];
        const int pbase = s_slotpos[k.first_slot];
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
                const uint32_t kk = on ? fold_id(idv[j], m.rows) : 0u;
                if (on) keys[i + dl] = m.base_row + kk;
                (void)lds_inc_grouped(s_hist, kk >> g.log_keys, on);
            }
        }
        __syncthreads();
        const int slice0 = s_first[m.stable];
        for (int s = tid; s < g.n; s += NT) {
            const int c = s_hist[s];
            if (c) atomicAdd(&slice_total[slice0 + s], c);
        }
    }
}

// Large batches: the slices' totals become places (one block: there are a few thousand slices).
// Every slice gets its table, its index in the table, the place of its first record and the number
// of records; the cursors of the scatter kernel start at those places.
constexpr int kScanThreads = 1024;
__global__ void __launch_bounds__(kScanThreads)
pk_slice_scan_kernel(const TableMeta* __restrict__ tmeta, int T, int F, int64_t nnz, int target,
                     const int32_t* __restrict__ slice_total, int32_t* __restrict__ slice_cursor,
                     SliceInfo* __restrict__ slice_info, int n_slices)
{
    extern __shared__ int32_t s_first[];                   // [T+1]
    table_scan<kScanThreads>(tmeta, T, F, nnz, target, s_first);
    int carry = 0;
    for (int base = 0; base < n_slices; base += kScanThreads) {
        const int s = base + (int)threadIdx.x;
        const int c = s < n_slices ? slice_total[s] : 0;
        int tot;
        const int ex = block_excl_scan<kScanThreads>(c, &tot);
        if (s < n_slices) {
            const int t = upper_bound_i32(s_first, T + 1, s) - 1;
            SliceInfo si;
            si.table = t; si.idx = s - s_first[t]; si.start = carry + ex; si.count = c;
            slice_info[s] = si;
            slice_cursor[s] = carry + ex;
        }
        carry += tot;
    }
}

// Large batches: one record per occurrence, (key inside its slice, bag inside its pack), written to
// the slice's place.  A tile counts its occurrences per slice in LDS, reserves room in every
// touched slice with one global add, and then places its records from block-local cursors.
template <int BT>
__global__ void __launch_bounds__(NT)
pk_scatter_kernel(const int32_t* __restrict__ offsets, int B, int F, int T, int64_t nnz, int target,
                  const FieldMeta* __restrict__ fmeta, const PackMeta* __restrict__ pm,
                  const TableMeta* __restrict__ tmeta, const int32_t* __restrict__ slot_field,
                  const PackState* __restrict__ st, const uint32_t* __restrict__ keys, int32_t* slice_cursor,
                  uint2* __restrict__ rec, int hist_words)
{
    extern __shared__ int32_t s_dyn[];                     // field scan | first slices | counts | places
    __shared__ int32_t s_po[BT + 1];
    int32_t* s_fb = s_dyn;
    int32_t* s_delta = s_fb + (F + 1);
    int32_t* s_slotpos = s_delta + F;
    int32_t* s_first = s_slotpos + (F + 1);
    int32_t* s_hist = s_first + (T + 1);
    int32_t* s_place = s_hist + hist_words;
    const int tid = threadIdx.x;
    const int bad = field_scan<NT>(offsets, B, F, nnz, slot_field, s_fb, s_delta, s_slotpos);
    table_scan<NT>(tmeta, T, F, nnz, target, s_first);
    if (bad) return;
    const int tpf = (B + BT - 1) / BT;
    const int64_t n_tiles = (int64_t)F * tpf;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const TileOf tl(tile, tpf, B, BT);
        const int f = tl.f;
        const FieldMeta m = fmeta[f];
        if (st[m.pack].error) continue;                    // the keys kernel rejected offsets of this pack
        const TableMeta tm = tmeta[m.stable];
        const SliceGeom g = slice_geom(tm.rows, tm.field_end - tm.field_begin, F, nnz, target);
        const int64_t g0 = (int64_t)f * B + tl.b0;
        __syncthreads();
        for (int t = tid; t <= tl.nb; t += NT) s_po[t] = offsets[g0 + t];
        for (int s = tid; s < g.n; s += NT) s_hist[s] = 0;
        __syncthreads();
        const int dl = s_delta[f];
        const int q_lo = s_po[0], q_hi = s_po[tl.nb];
        for (int base = q_lo; base < q_hi; base += NT) {
            const int i = base + tid;
            const uint32_t s = i < q_hi ? (keys[i + dl] - m.base_row) >> g.log_keys : 0xFFFFFFFFu;
            (void)lds_inc_grouped(s_hist, s, s < (uint32_t)g.n);
        }
        __syncthreads();
        const int slice0 = s_first[m.stable];
        for (int s = tid; s < g.n; s += NT) {
            const int c = s_hist[s];
            s_place[s] = c ? atomicAdd(&slice_cursor[slice0 + s], c) : 0;
            s_hist[s] = 0;
        }
        __syncthreads();
        const uint32_t bag0 = (uint32_t)m.slot * (uint32_t)B + (uint32_t)tl.b0;
        for (int base = q_lo; base < q_hi; base += NT) {
            const int i = base + tid;
            const uint32_t kk = i < q_hi ? keys[i + dl] - m.base_row : 0xFFFFFFFFu;
            const uint32_t s = kk >> g.log_keys;
            const bool on = i < q_hi && s < (uint32_t)g.n;
            const int at_local = lds_inc_grouped(s_hist, s, on);
            if (!on) continue;
            const int t = upper_bound_i32(s_po, tl.nb + 1, i) - 1;
            const int64_t at = (int64_t)s_place[s] + at_local;
            if ((uint64_t)at < (uint64_t)nnz) rec[at] = make_uint2(kk - (s << g.log_keys), bag0 + (uint32_t)t);
        }
    }
}

// ---------------------------------------------------------------------------
// The slice kernel's body.
// ---------------------------------------------------------------------------
constexpr int kSliceThreads = 1024;

struct SliceArgs {
    const TableMeta* tmeta; const int32_t* table_fields; int T;
    const FieldMeta* fmeta; const PackMeta* pm; const int32_t* slot_field; PackState* st; int P;
    int F, B; int64_t nnz; int target;
    const int64_t* ids; const int32_t* offsets;                 // small batches: the block finds its occurrences itself
    const SliceInfo* slice_info; const uint2* rec;              // large batches: the slice's records
    int32_t* packed_offsets;
    uint32_t* keys; int32_t* inverse;                           // written here for small batches only
    uint32_t* bitmap; int32_t* rank;                            // written here for large batches only
    uint32_t* unique; int32_t* seg_all; uint32_t* ent_all; int ent_mult;
    int4* tile_hdr; int tp; double* ghot; int dmax;
    uint64_t* desc; int32_t* done; int n_slices;                // small batches: descriptors the library owns, cleaned by the last block
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

// LDS of a slice block: bitmap words | their popcount prefix | counters of a round of distinct keys.
// The same words first hold the set-up scans (first slices of the tables, then the field scan).
constexpr int kSliceLds = 2 * kSliceWordsMax + kSliceRanks;
static_assert(kSliceLds >= 3 * 4096 + 2 && kSliceLds >= 4096 + 1, "set-up scans must fit the slice block's LDS");

// one occurrence of a slice: its key inside the slice and where it comes from
struct SliceRec {
    uint32_t kl;       // key minus the slice's first key
    int32_t x;         // small batches: the field's index in the table's field list; large: the bag inside the pack
    int32_t q;         // small batches: position in ids
};

template <bool FROM_IDS>
__device__ __forceinline__ void slice_body(const SliceArgs& a, int slice, int32_t* s_main, int32_t* s_tf)
{
    const int tid = threadIdx.x;
    uint32_t* s_bits = reinterpret_cast<uint32_t*>(s_main);
    uint32_t* s_pre = s_bits + kSliceWordsMax;
    int32_t* s_cnt = s_main + 2 * kSliceWordsMax;
    __shared__ uint32_t s_bc[4];
    const int F = a.F, B = a.B, T = a.T;
    const int64_t out_dim = a.out_dim;

    PK_PT(a, slice, 0);
    // ---- which slice, of which table; where the pack's arrays start ----
    int t, idx, pack_first, is_last, pstart, nnz_p, rec_start = 0, rec_count = 0;
    if (FROM_IDS) {
        table_scan<kSliceThreads>(a.tmeta, T, F, a.nnz, a.target, s_main);
        t = upper_bound_i32(s_main, T + 1, slice) - 1;
        idx = slice - s_main[t];
        const PackMeta k0 = a.pm[a.tmeta[t].pack];
        pack_first = s_main[k0.first_stable];
        is_last = slice + 1 == s_main[k0.first_stable + k0.n_stables];
        __syncthreads();
    } else {
        const SliceInfo si = a.slice_info[slice];
        t = si.table; idx = si.idx; rec_start = si.start; rec_count = si.count;
        pack_first = 0; is_last = 0;
    }
    const TableMeta tm = a.tmeta[t];
    const int p = tm.pack;
    const PackMeta k = a.pm[p];
    const int nf = tm.field_end - tm.field_begin;
    const SliceGeom geo = slice_geom(tm.rows, nf, F, a.nnz, a.target);
    const int lg = geo.log_keys;
    uint32_t own_flags = 0;
    if (FROM_IDS) {
        int32_t* s_fb = s_main;
        int32_t* s_delta = s_fb + (F + 1);
        int32_t* s_slotpos = s_delta + F;
        const int bad = field_scan<kSliceThreads>(a.offsets, B, F, a.nnz, a.slot_field, s_fb, s_delta, s_slotpos);
        pstart = s_slotpos[k.first_slot];
        nnz_p = s_slotpos[k.first_slot + k.n_fields] - pstart;
        for (int j = tid; j < nf; j += kSliceThreads) {
            const int f = a.table_fields[tm.field_begin + j];
            s_tf[3 * j] = s_fb[f];
            s_tf[3 * j + 1] = s_fb[f + 1];
            s_tf[3 * j + 2] = s_delta[f];
        }
        __syncthreads();
        if (bad) {                                         // every block sees the same boundaries: nobody publishes, nobody waits
            if (is_last && tid == 0) { a.st[p].n_unique = 0; a.st[p].error = 1; }
            return;
        }
        // the offsets of this slice's share of the table's bags: inside the field and not decreasing
        int viol = 0;
        const int b_lo = (int)((int64_t)B * idx / geo.n), b_hi = (int)((int64_t)B * (idx + 1) / geo.n);
        for (int j = 0; j < nf; ++j) {
            const int f = a.table_fields[tm.field_begin + j];
            const int32_t* offs = a.offsets + (int64_t)f * B;
            for (int b = b_lo + tid; b < b_hi; b += kSliceThreads) {
                const int o0 = offs[b], o1 = offs[b + 1];
                viol |= o0 > o1 || o0 < s_tf[3 * j] || o1 > s_tf[3 * j + 1];
            }
        }
        if (__syncthreads_or(viol)) own_flags |= 1u;
    } else {
        pstart = a.st[p].start;
        nnz_p = a.st[p].nnz;
        pack_first = a.st[p].first_slice;
        is_last = t == k.first_stable + k.n_stables - 1 && idx + 1 == geo.n;   // last slice of the pack's last table
        if (a.st[p].error) return;                         // offsets of this pack were rejected: no block of it publishes or waits
    }

    PK_PT(a, slice, 1);
    const uint32_t lo = (uint32_t)idx << lg;               // first key of the slice inside its table
    const uint32_t nkeys = min((uint32_t)1 << lg, tm.rows - lo);
    const int words = 1 << (lg - 5);
    const int32_t* __restrict__ tf = a.table_fields + tm.field_begin;

    // all occurrences of the slice, in any order: fn(SliceRec, on).  Every lane makes the same trips and
    // calls fn every time, with on = false where it has no occurrence, so that fn may combine lanes.
    auto for_records = [&](auto&& fn) {
        if (FROM_IDS) {
            for (int j = 0; j < nf; ++j) {
                const int q0 = s_tf[3 * j], q1 = s_tf[3 * j + 1];
                for (int base = q0; base < q1; base += 4 * kSliceThreads) {
                    int64_t idv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int i = base + tid + u * kSliceThreads;
                        idv[u] = i < q1 ? a.ids[i] : 0;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int i = base + tid + u * kSliceThreads;
                        const uint32_t kk = i < q1 ? fold_id(idv[u], tm.rows) : 0xFFFFFFFFu;
                        const bool on = i < q1 && (kk >> lg) == (uint32_t)idx;
                        fn(SliceRec{on ? kk - lo : 0u, j, i}, on);
                    }
                }
            }
        } else {
            const uint2* __restrict__ rec = a.rec + rec_start;
            for (int base = 0; base < rec_count; base += 4 * kSliceThreads) {
                uint2 r[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = base + tid + u * kSliceThreads;
                    r[u] = i < rec_count ? rec[i] : make_uint2(0xFFFFFFFFu, 0);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const bool on = r[u].x < nkeys;
                    fn(SliceRec{on ? r[u].x : 0u, (int32_t)r[u].y, 0}, on);
                }
            }
        }
    };

    // ---- which keys occur ----
    for (int w = tid; w < words; w += kSliceThreads) s_bits[w] = 0;
    __syncthreads();
    int mine = 0;
    for_records([&](const SliceRec& r, bool on) {
        if (!on) return;
        const uint32_t bit = 1u << (r.kl & 31);
        if (!(s_bits[r.kl >> 5] & bit)) atomicOr(&s_bits[r.kl >> 5], bit);
        ++mine;
    });
    int n_rec;
    (void)block_excl_scan<kSliceThreads>(mine, &n_rec);    // its barriers also complete the bitmap
    PK_PT(a, slice, 2);
    if (!FROM_IDS) n_rec = rec_count;
    // popcount prefix of the words: thread i owns words [i * wpt, (i + 1) * wpt)
    const int wpt = max(1, words / kSliceThreads);
    int c = 0;
    if (tid * wpt < words)
        for (int j = 0; j < wpt; ++j) c += __popc(s_bits[tid * wpt + j]);
    int n_u;
    const int ex = block_excl_scan<kSliceThreads>(c, &n_u);
    if (tid * wpt < words) {
        int run = ex;
        for (int j = 0; j < wpt; ++j) {
            s_pre[tid * wpt + j] = (uint32_t)run;
            run += __popc(s_bits[tid * wpt + j]);
        }
    }
    PK_PT(a, slice, 3);
    // ---- distinct keys and occurrences of the pack's slices before this one ----
    if (tid < 64) {
        uint32_t pa = 0, pb = 0, pf = 0;
        if (slice == pack_first) {
            if (tid == 0) publish_desc(a.desc + slice, make_desc(kDescPfx, (uint32_t)n_u, (uint32_t)n_rec, own_flags));
        } else {
            if (tid == 0) publish_desc(a.desc + slice, make_desc(kDescAgg, (uint32_t)n_u, (uint32_t)n_rec, own_flags));
            lookback(a.desc, pack_first, slice, &pa, &pb, &pf);
            if (tid == 0)
                publish_desc(a.desc + slice, make_desc(kDescPfx, pa + (uint32_t)n_u, pb + (uint32_t)n_rec, pf | own_flags));
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
    const int base_u = (int)s_bc[0];
    const int rec_before = FROM_IDS ? (int)s_bc[1] : rec_start - pstart;
    const uint32_t flags = s_bc[2];
    if (FROM_IDS && s_bc[3]) {
        for (int i = tid; i < a.n_slices; i += kSliceThreads) publish_desc(a.desc + i, 0);
        if (tid == 0) *a.done = 0;
    }

    // whatever the descriptors held, no write below leaves the pack's arrays
    if (base_u < 0 || rec_before < 0 || (int64_t)base_u + n_u > (int64_t)nnz_p || (int64_t)rec_before + n_rec > (int64_t)nnz_p) {
        if (tid == 0) atomicOr(&a.st[p].error, 2);
        return;
    }

    // ---- the slice's distinct keys, ascending; bitmap and rank samples for the inverse kernel ----
    uint32_t* __restrict__ uq = a.unique + pstart;
    int32_t* __restrict__ seg = a.seg_all + pstart + p;
    if (tid * wpt < words) {
        for (int j = 0; j < wpt; ++j) {
            const int w = tid * wpt + j;
            uint32_t x = s_bits[w];
            int at = base_u + (int)s_pre[w];
            const uint32_t key0 = tm.key_lo + lo + (uint32_t)w * 32u;
            while (x) {
                const int bit = __ffs(x) - 1;
                x &= x - 1;
                uq[at++] = key0 + bit;
            }
        }
    }
    if (!FROM_IDS) {
        const size_t w0 = (size_t)tm.word_base + (size_t)idx * words;
        for (int w = tid; w < words; w += kSliceThreads) {
            a.bitmap[w0 + w] = s_bits[w];
            if ((w & (kRankWords - 1)) == 0) a.rank[(w0 + w) / kRankWords] = base_u + (int)s_pre[w];
        }
    }
    if (is_last && tid == 0) {
        a.st[p].n_unique = base_u + n_u;
        seg[base_u + n_u] = nnz_p;
        if (FROM_IDS) a.st[p].error = (int32_t)flags;
        else if (flags) atomicOr(&a.st[p].error, (int32_t)flags);
    }

    PK_PT(a, slice, 5);
    // ---- occurrences per distinct key, segment offsets, headers of the backward tiles, and every
    //      occurrence's gradient place at its key's next free position; a round handles kSliceRanks keys ----
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
    int placed = 0;                                        // occurrences of the keys of earlier rounds
    for (int r0 = 0; r0 < n_u; r0 += kSliceRanks) {
        const int width = min(kSliceRanks, n_u - r0);
        __syncthreads();
        for (int i = tid; i < width; i += kSliceThreads) s_cnt[i] = 0;
        __syncthreads();
        for_records([&](const SliceRec& r, bool on) {
            const uint32_t rr = (uint32_t)(rank_of(r.kl) - r0);
            (void)lds_inc_grouped(s_cnt, rr, on && rr < (uint32_t)width);
        });
        __syncthreads();
        PK_PT(a, slice, 6);
        constexpr int per = kSliceRanks / kSliceThreads;   // consecutive counters per thread
        int sum = 0;
#pragma unroll
        for (int j = 0; j < per; ++j) {
            const int i = tid * per + j;
            sum += i < width ? s_cnt[i] : 0;
        }
        int tot;
        int s0 = rec_before + placed + block_excl_scan<kSliceThreads>(sum, &tot);
#pragma unroll
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
            const int pos = lds_inc_grouped(s_cnt, rr, on);
            if (!on) return;
            uint32_t ref, len;
            if (FROM_IDS) {
                const int f = tf[r.x];
                const FieldMeta m = a.fmeta[f];
                const int32_t* offs = a.offsets + (int64_t)f * B;
                const int b = find_bag(offs, B, r.q, r.q - s_tf[3 * r.x]);
                const int L = offs[b + 1] - offs[b];
                ref = (uint32_t)((int64_t)b * out_dim + m.col);
                len = (m.pool == PK_MEAN && L > 0) ? (uint32_t)L : 1u;
                const int qp = r.q + s_tf[3 * r.x + 2];
                if ((unsigned)qp < (unsigned)a.nnz) {
                    a.keys[qp] = tm.key_lo + lo + r.kl;
                    a.inverse[qp] = base_u + rk;
                }
            } else {
                const uint32_t g = (uint32_t)r.x;
                const uint32_t slot = g / (uint32_t)B, b = g - slot * (uint32_t)B;
                const int f = slot < (uint32_t)k.n_fields ? a.slot_field[k.first_slot + (int)slot] : a.slot_field[k.first_slot];
                const FieldMeta m = a.fmeta[f];
                ref = (uint32_t)((int64_t)b * out_dim + m.col);
                len = 1u;
                if (wide && m.pool == PK_MEAN && slot < (uint32_t)k.n_fields) {
                    const int L = po[g + 1] - po[g];
                    if (L > 0) len = (uint32_t)L;
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

// Large batches: one block per slice.  (Block i takes slice i; see the look-back's note on order.)
__global__ void __launch_bounds__(kSliceThreads)
pk_slices_kernel(SliceArgs a)
{
    __shared__ int32_t s_main[kSliceLds];
    slice_body<false>(a, blockIdx.x, s_main, nullptr);
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
// Large batches: inverse[q] = number of distinct keys of the pack below key[q]: the rank sample of
// the key's 256-key block (written by the slice kernel) plus the set bits before the key inside
// the block.  Tiles as in the keys kernel: bags of one field, hence one table.
// ---------------------------------------------------------------------------
template <int BT>
__global__ void __launch_bounds__(NT)
pk_inverse_kernel(const int32_t* __restrict__ offsets, int B, int F, int64_t nnz, const FieldMeta* __restrict__ fmeta,
                  const TableMeta* __restrict__ tmeta, const int32_t* __restrict__ slot_field,
                  const PackState* __restrict__ st, const uint32_t* __restrict__ keys,
                  const uint4* __restrict__ bitmap4, const int32_t* __restrict__ rank, int32_t* __restrict__ inverse)
{
    extern __shared__ int32_t s_dyn[];
    int32_t* s_fb = s_dyn;
    int32_t* s_delta = s_fb + (F + 1);
    int32_t* s_slotpos = s_delta + F;
    const int tid = threadIdx.x;
    if (field_scan<NT>(offsets, B, F, nnz, slot_field, s_fb, s_delta, s_slotpos)) return;
    const int tpf = (B + BT - 1) / BT;
    const int64_t n_tiles = (int64_t)F * tpf;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const TileOf tl(tile, tpf, B, BT);
        const int f = tl.f;
        const FieldMeta m = fmeta[f];
        if (st[m.pack].error) continue;
        const TableMeta tm = tmeta[m.stable];
        const int64_t g0 = (int64_t)f * B + tl.b0;
        const int q_lo = min(max(offsets[g0], s_fb[f]), s_fb[f + 1]) + s_delta[f];
        const int q_hi = min(max(offsets[g0 + tl.nb], s_fb[f]), s_fb[f + 1]) + s_delta[f];
        const uint4* bm = bitmap4 + (size_t)tm.word_base / 4;
        const int32_t* rk = rank + (size_t)tm.word_base / kRankWords;
        for (int q0 = q_lo + tid; q0 < q_hi; q0 += 4 * NT) {
            uint32_t kk[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int q = q0 + j * NT;
                kk[j] = q < q_hi ? keys[q] - tm.key_lo : 0;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int q = q0 + j * NT;
                if (q >= q_hi || kk[j] >= tm.rows) continue;
                const uint32_t blk = kk[j] >> 8;
                const int wi = (kk[j] >> 5) & 7;
                const uint4 x = bm[2 * (size_t)blk], y = bm[2 * (size_t)blk + 1];
                const uint32_t w[8] = {x.x, x.y, x.z, x.w, y.x, y.y, y.z, y.w};
                int r = rk[blk];
                uint32_t cur = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if (i < wi) r += __popc(w[i]);
                    if (i == wi) cur = w[i];
                }
                r += __popc(cur & ((1u << (kk[j] & 31)) - 1u));
                inverse[q] = r;
            }
        }
    }
}
