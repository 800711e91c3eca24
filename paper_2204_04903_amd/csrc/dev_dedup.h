// H1 and H2: packed keys, the bitmap of the rows that occur, its one-pass scan (distinct keys and rank
// samples), the inverse index, and the per-key occurrence lists (LDS counting sort).
// Part of pk_device.hip: included there, in this order, inside its anonymous namespace.

// ---------------------------------------------------------------------------
// H1: packed keys (Sec. III-B: one packed ID tensor per pack), packed bag
// offsets, and for every occurrence the place of its bag's gradient chunk.
// A block takes BT consecutive bags (field-major, so their IDs are contiguous),
// keeps their offsets in LDS and finds each occurrence's bag there.
//
// Where a field's occurrences go in the packed order follows from the field
// boundaries alone, so every block derives it for itself (a scan over the
// fields in (pack, slot) order) instead of waiting for a set-up launch; block 0
// also stores it for the later kernels.  All blocks share the clearing of the
// scan descriptors.
// ---------------------------------------------------------------------------
struct KeysArgs {
    const int64_t* ids; const int32_t* offsets; int B, F, P; int64_t nnz;
    const FieldMeta* fmeta; const PackMeta* pm; const int32_t* slot_field; PackState* st;
    int32_t* fb_out; int32_t* delta_out;
    uint32_t* keys; uint32_t* bagref; uint32_t* baglen; int32_t* packed_offsets;
    int64_t out_dim; uint4* clear4; int64_t n_clear4;
};

// LDS words of keys_body: per bag (a flag, the offsets of BT bags and five values per bag) and
// per field (the scan of the field boundaries)
template <int BT>
constexpr int keys_bag_words() { return 1 + (BT + 1) + 5 * BT; }
constexpr size_t keys_field_words(int F) { return (size_t)(3 * F + 2); }

// `block` of `nblocks` blocks of NTH threads.  (The arrays come as restrict-qualified parameters
// of their own: the compiler orders the loads and stores of the inner loop far better when it
// knows that they do not overlap.)
template <int BT, int NTH>
__device__ __forceinline__ void keys_core(const int64_t* __restrict__ ids, const int32_t* __restrict__ offsets,
                                          const FieldMeta* __restrict__ fmeta, const PackMeta* __restrict__ pm,
                                          const int32_t* __restrict__ slot_field, uint32_t* __restrict__ keys,
                                          uint32_t* __restrict__ bagref, uint32_t* __restrict__ baglen,
                                          int32_t* __restrict__ packed_offsets, const KeysArgs& a, int block,
                                          int nblocks, int32_t* lds_bag, int32_t* lds_field)
{
    const int B = a.B, F = a.F, P = a.P;
    const int64_t nnz = a.nnz;
    const int64_t out_dim = a.out_dim;
    int32_t* s_po = lds_bag;                  // [BT+1] offsets of the tile's bags
    uint32_t* s_base = reinterpret_cast<uint32_t*>(s_po + (BT + 1));   // [BT] each
    uint32_t* s_rows = s_base + BT;
    uint32_t* s_ref = s_rows + BT;
    int32_t* s_dl = reinterpret_cast<int32_t*>(s_ref + BT);
    uint32_t* s_len = reinterpret_cast<uint32_t*>(s_dl + BT);
    int32_t* s_badp = reinterpret_cast<int32_t*>(s_len + BT);
    int32_t* s_fb = lds_field;                // [F+1] field boundaries in ids
    int32_t* s_delta = s_fb + (F + 1);        // [F]   packed position minus position in ids
    int32_t* s_slotpos = s_delta + F;         // [F+1] packed position of each (pack, slot)
    const int tid = threadIdx.x;
    {
        const uint4 z = make_uint4(0, 0, 0, 0);
        const int64_t stride = (int64_t)nblocks * NTH;
        for (int64_t i = (int64_t)block * NTH + tid; i < a.n_clear4; i += stride) a.clear4[i] = z;
    }
    if (tid == 0) *s_badp = 0;
    for (int f = tid; f <= F; f += NTH) s_fb[f] = offsets[(int64_t)f * B];
    __syncthreads();
    for (int f = tid; f < F; f += NTH)
        if (s_fb[f + 1] < s_fb[f]) *s_badp = 1;
    if (tid == 0 && (s_fb[0] != 0 || (int64_t)s_fb[F] != nnz)) *s_badp = 1;
    __syncthreads();
    const int bad = *s_badp;
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
    if (block == 0) {
        for (int f = tid; f <= F; f += NTH) a.fb_out[f] = s_fb[f];
        for (int f = tid; f < F; f += NTH) a.delta_out[f] = s_delta[f];
        for (int p = tid; p < P; p += NTH) {
            const PackMeta k = pm[p];
            const int start = s_slotpos[k.first_slot];
            PackState s;
            s.nnz = s_slotpos[k.first_slot + k.n_fields] - start;
            s.start = start; s.n_unique = 0; s.error = (p == 0) ? bad : 0;
            s.pad[0] = s.pad[1] = s.pad[2] = s.pad[3] = 0;
            a.st[p] = s;
            packed_offsets[(int64_t)k.first_slot * B + p + (int64_t)k.n_fields * B] = s.nnz;
        }
    }
    if (bad) return;
    const int64_t n_bags = (int64_t)F * B;
    const int64_t n_tiles = (n_bags + BT - 1) / BT;
    for (int64_t tile = block; tile < n_tiles; tile += nblocks) {
        const int64_t g0 = tile * BT;
        const int nb = (int)min((int64_t)BT, n_bags - g0);
        __syncthreads();                               // the previous tile's LDS is consumed
        for (int t = tid; t <= nb; t += NTH) s_po[t] = (int32_t)min((int64_t)max(offsets[g0 + t], 0), nnz);
        __syncthreads();
        for (int t = tid; t < nb; t += NTH) {
            const int64_t g = g0 + t;
            const int f = (int)(g / B);
            const int b = (int)(g - (int64_t)f * B);
            const FieldMeta m = fmeta[f];
            const PackMeta k = pm[m.pack];
            s_base[t] = m.base_row;
            s_rows[t] = m.rows;
            s_dl[t] = s_delta[f];
            s_ref[t] = (uint32_t)((int64_t)b * out_dim + m.col);
            const int L = s_po[t + 1] - s_po[t];
            s_len[t] = (m.pool == PK_MEAN && L > 0) ? (uint32_t)L : 1u;     // what the gradient is divided by
            packed_offsets[(int64_t)k.first_slot * B + m.pack + (int64_t)m.slot * B + b] =
                s_po[t] + s_delta[f] - s_slotpos[k.first_slot];
        }
        __syncthreads();
        const int q_lo = s_po[0], q_hi = s_po[nb];
        for (int i0 = q_lo + tid; i0 < q_hi; i0 += 4 * NTH) {
            int64_t idv[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {              // the loads of four rounds in flight together
                const int i = i0 + k * NTH;
                idv[k] = i < q_hi ? ids[i] : 0;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = i0 + k * NTH;
                if (i >= q_hi) continue;
                const int t = upper_bound_i32(s_po, nb + 1, i) - 1;
                if ((unsigned)t >= (unsigned)nb) continue;
                const int64_t q = (int64_t)i + s_dl[t];
                if ((uint64_t)q >= (uint64_t)nnz) continue;
                keys[q] = s_base[t] + fold_id(idv[k], s_rows[t]);
                bagref[q] = s_ref[t];
                if (baglen) baglen[q] = s_len[t];
            }
        }
    }
}

template <int BT>
__global__ void __launch_bounds__(NT)
pk_keys_kernel(const int64_t* __restrict__ ids, const int32_t* __restrict__ offsets, int B, int F, int P, int64_t nnz,
               const FieldMeta* __restrict__ fmeta, const PackMeta* __restrict__ pm,
               const int32_t* __restrict__ slot_field, PackState* st, int32_t* fb_out, int32_t* delta_out,
               uint32_t* __restrict__ keys, uint32_t* __restrict__ bagref, uint32_t* __restrict__ baglen,
               int32_t* __restrict__ packed_offsets, int64_t out_dim, uint4* clear4, int64_t n_clear4)
{
    extern __shared__ int32_t s_dyn[];                     // keys_field_words(F)
    __shared__ int32_t s_bag[keys_bag_words<BT>()];
    const KeysArgs a{ids, offsets, B, F, P, nnz, fmeta, pm, slot_field, st, fb_out, delta_out, keys, bagref, baglen,
                     packed_offsets, out_dim, clear4, n_clear4};
    keys_core<BT, NT>(ids, offsets, fmeta, pm, slot_field, keys, bagref, baglen, packed_offsets, a, blockIdx.x,
                      gridDim.x, s_bag, s_dyn);
}

// ---------------------------------------------------------------------------
// H2, first half: which rows occur.  Global atomics run at a fixed, low rate on
// this GPU whatever their address, so the bitmap is not built with them: a block
// owns a slice of a pack's key space, keeps the slice's bits in LDS, scans the
// keys of the fields whose tables overlap the slice (they are contiguous in the
// packed order) and stores the finished words with plain coalesced writes.
// Every bitmap word is written by exactly one block, so nothing needs clearing.
// ---------------------------------------------------------------------------
constexpr int kMarkThreads = 1024;
constexpr int kMarkUnroll = 8;

struct MarkArgs {
    const MarkItem* items; const int32_t* item_fields; const PackMeta* pm; const PackState* st;
    const int32_t* fb; const int32_t* delta; const uint32_t* keys; uint32_t* bitmap; int64_t nnz;
};

// set bit k of the slice if it is inside (one LDS read where the bit is already there)
__device__ __forceinline__ void mark_bit(uint32_t* s_bits, uint32_t k, uint32_t span)
{
    if (k < span) {
        const uint32_t bit = 1u << (k & 31);
        if (!(s_bits[k >> 5] & bit)) atomicOr(&s_bits[k >> 5], bit);
    }
}

// One slice.  FROM_IDS: the keys are formed here from the IDs of the fields (the same hash
// as in keys_body), so that this does not have to wait for the keys kernel and can share
// its launch; `ka` is then that kernel's argument block.
template <bool FROM_IDS>
__device__ __forceinline__ void mark_body(const MarkArgs& ma, const KeysArgs& ka, int item, uint32_t* s_bits)
{
    int mine = 0;
    if (FROM_IDS) {                                        // the checks of keys_body, which runs beside this
        for (int f = threadIdx.x; f < ka.F; f += kMarkThreads)
            mine |= ka.offsets[(int64_t)(f + 1) * ka.B] < ka.offsets[(int64_t)f * ka.B];
        if (threadIdx.x == 0) mine |= ka.offsets[0] != 0 || (int64_t)ka.offsets[(int64_t)ka.F * ka.B] != ka.nnz;
    }
    const MarkItem it = ma.items[item];
    for (int w = threadIdx.x; w < it.n_words; w += kMarkThreads) s_bits[w] = 0;
    const uint32_t span = (uint32_t)it.n_words * 32u;
    int bad;
    if (FROM_IDS) {
        bad = __syncthreads_or(mine);
    } else {
        __syncthreads();
        bad = ma.st[0].error;
    }
    if (!bad) {
        for (int fi = it.field_begin; fi < it.field_end; ++fi) {
            const int f = ma.item_fields[fi];
            if (FROM_IDS) {
                const FieldMeta m = ka.fmeta[f];
                const int64_t q0 = ka.offsets[(int64_t)f * ka.B], q1 = ka.offsets[(int64_t)(f + 1) * ka.B];
                const uint32_t base = m.base_row - it.key_lo;      // modulo 2^32, like the subtraction below
                int64_t q = q0 + threadIdx.x;
                for (; q + (kMarkUnroll - 1) * kMarkThreads < q1; q += kMarkUnroll * kMarkThreads) {
                    int64_t id[kMarkUnroll];
#pragma unroll
                    for (int j = 0; j < kMarkUnroll; ++j) id[j] = ka.ids[q + j * kMarkThreads];
#pragma unroll
                    for (int j = 0; j < kMarkUnroll; ++j) mark_bit(s_bits, base + fold_id(id[j], m.rows), span);
                }
                for (; q < q1; q += kMarkThreads) mark_bit(s_bits, base + fold_id(ka.ids[q], m.rows), span);
            } else {
                const int64_t q0 = (int64_t)ma.fb[f] + ma.delta[f], q1 = (int64_t)ma.fb[f + 1] + ma.delta[f];
                if (q0 < 0 || q1 > ma.nnz) continue;
                int64_t q = q0 + threadIdx.x;
                for (; q + (kMarkUnroll - 1) * kMarkThreads < q1; q += kMarkUnroll * kMarkThreads) {
                    uint32_t k[kMarkUnroll];
#pragma unroll
                    for (int j = 0; j < kMarkUnroll; ++j) k[j] = ma.keys[q + j * kMarkThreads] - it.key_lo;   // loads in flight together
#pragma unroll
                    for (int j = 0; j < kMarkUnroll; ++j) mark_bit(s_bits, k[j], span);
                }
                for (; q < q1; q += kMarkThreads) mark_bit(s_bits, ma.keys[q] - it.key_lo, span);
            }
        }
    }
    __syncthreads();
    uint4* dst = reinterpret_cast<uint4*>(ma.bitmap + (size_t)ma.pm[it.pack].first_tile * kTileWords + it.key_lo / 32);
    const uint4* src = reinterpret_cast<const uint4*>(s_bits);
    for (int w = threadIdx.x; w < it.n_words / 4; w += kMarkThreads) dst[w] = src[w];
}

__global__ void __launch_bounds__(kMarkThreads)
pk_mark_kernel(MarkArgs ma)
{
    __shared__ uint32_t s_bits[kMarkWords];
    mark_body<false>(ma, KeysArgs{}, blockIdx.x, s_bits);
}

// Small batches: the keys and the bitmap in one launch.  Blocks [0, mark_blocks) take the
// slices and form the keys they need themselves; the others are the keys kernel.  (With few
// occurrences every launch is mostly latency, and the second one would wait for the first.)
constexpr int kFusedKeysBags = 1024;       // bags per block iteration of the keys part
template <int BT>
__global__ void __launch_bounds__(kMarkThreads)
pk_keys_mark_kernel(const int64_t* __restrict__ ids, const int32_t* __restrict__ offsets, int B, int F, int P,
                    int64_t nnz, const FieldMeta* __restrict__ fmeta, const PackMeta* __restrict__ pm,
                    const int32_t* __restrict__ slot_field, PackState* st, int32_t* fb_out, int32_t* delta_out,
                    uint32_t* __restrict__ keys, uint32_t* __restrict__ bagref, uint32_t* __restrict__ baglen,
                    int32_t* __restrict__ packed_offsets, int64_t out_dim, uint4* clear4, int64_t n_clear4,
                    MarkArgs ma, int mark_blocks)
{
    __shared__ uint32_t s_raw[kMarkWords];                 // either role's LDS
    const KeysArgs ka{ids, offsets, B, F, P, nnz, fmeta, pm, slot_field, st, fb_out, delta_out, keys, bagref, baglen,
                      packed_offsets, out_dim, clear4, n_clear4};
    if ((int)blockIdx.x < mark_blocks)
        mark_body<true>(ma, ka, blockIdx.x, s_raw);
    else
        keys_core<BT, kMarkThreads>(ids, offsets, fmeta, pm, slot_field, keys, bagref, baglen, packed_offsets, ka,
                                    (int)blockIdx.x - mark_blocks, (int)gridDim.x - mark_blocks,
                                    reinterpret_cast<int32_t*>(s_raw),
                                    reinterpret_cast<int32_t*>(s_raw) + keys_bag_words<BT>());
}

// ---------------------------------------------------------------------------
// H2 (Unique, Sec. II-D) via a bitmap over the pack's rows: the ascending
// distinct keys are the set bits in order, and the index of a key among them is
// the number of set bits before it.  One pass: popcount per 256-bit block,
// prefix over all blocks of the pack, rank samples, distinct keys written out.
// ---------------------------------------------------------------------------
// A block iteration scans a run of K tiles of one pack (K * kTileWords bitmap words, every
// thread K consecutive 256-bit blocks): with several thousand tiles, fewer and larger steps
// keep the chain of prefixes short.
template <int K>
__global__ void __launch_bounds__(NT, 4)   // four blocks per CU must fit: 1024 blocks resident at once
pk_tiles_kernel(const uint4* __restrict__ bitmap4, uint64_t* tile_desc, int n_runs_total,
                const PackMeta* __restrict__ pm, PackState* st, int P,
                int32_t* __restrict__ rank, uint32_t* __restrict__ unique)
{
    __shared__ uint32_t s_pre;
    // Block b takes runs b, b+G, b+2G, ...: a run waits for the runs before it, those of
    // other blocks' earlier rounds included; the launch keeps G small enough for all blocks
    // to be resident, so the waits end.
    int p = 0, first = 0;                                  // the pack of the run, the pack's first run
    for (int run = blockIdx.x; run < n_runs_total; run += gridDim.x) {
        while (p + 1 < P && run >= first + (pm[p].n_tiles + K - 1) / K) {
            first += (pm[p].n_tiles + K - 1) / K;
            ++p;
        }
        const int n_blocks = pm[p].n_tiles * NT;           // 256-bit blocks of the pack
        const int b0 = ((run - first) * NT + (int)threadIdx.x) * K;   // this thread's first one
        const size_t t0 = (size_t)pm[p].first_tile * NT + b0;
        uint32_t w[K][8];
        int c[K], mine = 0;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            uint4 a = make_uint4(0, 0, 0, 0), b = a;
            if (b0 + k < n_blocks) { a = bitmap4[2 * (t0 + k)]; b = bitmap4[2 * (t0 + k) + 1]; }
            w[k][0] = a.x; w[k][1] = a.y; w[k][2] = a.z; w[k][3] = a.w;
            w[k][4] = b.x; w[k][5] = b.y; w[k][6] = b.z; w[k][7] = b.w;
            c[k] = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) c[k] += __popc(w[k][i]);
            mine += c[k];
        }
        int tot;
        const int ex = block_excl_scan<NT>(mine, &tot);    // its barriers also fence s_pre between rounds
        if (threadIdx.x < 64) {
            if (run == first) {
                if (threadIdx.x == 0) { publish_desc(tile_desc + run, make_desc(kDescPfx, (uint32_t)tot, 0)); s_pre = 0; }
            } else {
                if (threadIdx.x == 0) publish_desc(tile_desc + run, make_desc(kDescAgg, (uint32_t)tot, 0));
                uint32_t pa, pb;
                lookback(tile_desc, first, run, &pa, &pb, &st[0].error);
                if (threadIdx.x == 0) {
                    publish_desc(tile_desc + run, make_desc(kDescPfx, pa + (uint32_t)tot, 0));
                    s_pre = pa;
                }
            }
        }
        __syncthreads();
        int pre = (int)s_pre + ex;
        if (run == first + (pm[p].n_tiles + K - 1) / K - 1 && threadIdx.x == 0) st[p].n_unique = (int)s_pre + tot;
        uint32_t* uq = unique + st[p].start;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (b0 + k >= n_blocks) break;
            rank[t0 + k] = pre;
            if (c[k] != 0) {
                const uint32_t key0 = (uint32_t)(b0 + k) * 256u;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    uint32_t x = w[k][i];
                    while (x) {
                        const int bit = __ffs(x) - 1;
                        x &= x - 1;
                        uq[pre] = key0 + i * 32 + bit;
                        ++pre;
                    }
                }
            }
        }
    }
}

// inverse[q] = number of distinct keys below key[q]: the rank sample of the key's
// 256-bit block plus the set bits before it inside the block.
template <int KT>
__global__ void __launch_bounds__(NT)
pk_inverse_kernel(const PackMeta* __restrict__ pm, const PackState* __restrict__ st,
                  const uint32_t* __restrict__ keys, const uint4* __restrict__ bitmap4,
                  const int32_t* __restrict__ rank, int32_t* __restrict__ inverse)
{
    const int p = blockIdx.y;
    const int n = st[p].nnz, start = st[p].start;
    const size_t rb = (size_t)pm[p].first_tile * NT;          // rank blocks before this pack
    const uint4* bm = bitmap4 + 2 * rb;
    const int32_t* rk = rank + rb;
    const int n_tiles = (n + KT - 1) / KT;
    for (XcdTiles it(n_tiles); it.valid(); it.next()) {
        uint32_t key[KT / NT];
#pragma unroll
        for (int k = 0; k < KT / NT; ++k) {
            const int q = it.tile * KT + k * NT + threadIdx.x;
            key[k] = q < n ? keys[start + q] : 0;
        }
#pragma unroll
        for (int k = 0; k < KT / NT; ++k) {
            const int q = it.tile * KT + k * NT + threadIdx.x;
            if (q < n) {
                const uint32_t blk = key[k] >> 8;
                const int wi = (key[k] >> 5) & 7;
                const uint4 a = bm[2 * (size_t)blk], b = bm[2 * (size_t)blk + 1];
                const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
                int r = rk[blk];
                uint32_t cur = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if (i < wi) r += __popc(w[i]);
                    if (i == wi) cur = w[i];
                }
                r += __popc(cur & ((1u << (key[k] & 31)) - 1u));
                inverse[start + q] = r;
            }
        }
    }
}

// number of distinct keys of the pack below `key` (key may be absent, or one past the last row)
__device__ __forceinline__ int rank_of_key(const uint4* __restrict__ bm, const int32_t* __restrict__ rk,
                                           uint64_t key64, uint64_t key_end, int n_unique)
{
    if (key64 >= key_end) return n_unique;
    const uint32_t key = (uint32_t)key64;
    const uint32_t blk = key >> 8;
    const int wi = (key >> 5) & 7;
    const uint4 a = bm[2 * (size_t)blk], b = bm[2 * (size_t)blk + 1];
    const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    int r = rk[blk];
    uint32_t cur = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (i < wi) r += __popc(w[i]);
        if (i == wi) cur = w[i];
    }
    return r + __popc(cur & ((1u << (key & 31)) - 1u));
}

// H2, last part: the occurrences grouped by distinct key (a counting sort by
// rank), the segment offsets, and what the backward pass needs to cut its work
// by occurrences -- in one kernel and without global atomics.
//
// A table's distinct keys are a contiguous range of ranks, and its occurrences
// are the occurrences of the fields that read it (contiguous in the packed
// order).  A work item is one table and up to kSortCap of its ranks; which items
// exist depends on the batch, so every block derives the list for itself from
// the rank samples.  An item
//   1. counts the occurrences of each of its ranks in LDS,
//   2. scans the counts, learns the number of occurrences before it from the
//      items before it (descriptor look-back), and writes the segment offsets,
//      for each backward tile the key that holds the tile's first position, and
//      zeroed partial sums for keys that are long and cross a tile boundary,
//   3. passes over the occurrences again and stores each one's gradient place
//      (and mean-pooling scale) at its segment's next free position.
// Block b takes items b, b+G, ...: an item only waits for lower items, which are
// in earlier rounds or in lower blocks of this round; G is small enough for all
// blocks to be resident, so the waits end.
constexpr int kSortThreads = 1024;
constexpr int kSortUnroll2 = 4;       // occurrences per thread in flight in the placing pass

struct SortArgs {
    const TableMeta* tmeta; const int32_t* table_fields; int T;
    const PackMeta* pm; PackState* st; int P;
    const int32_t* fb; const int32_t* delta;
    const uint4* bitmap4; const int32_t* rank;
    const int32_t* inverse; const uint32_t* bagref; const uint32_t* baglen;
    int32_t* seg_all; uint32_t* ent_all; int ent_mult;
    int4* tile_hdr; int tp; uint64_t* desc; double* ghot; int dmax;
    int64_t nnz;
};

// What a work item (a table's ranks [c0, c0 + width), width counters in s_cnt) needs to know
struct SortItem {
    TableMeta tm;
    int p;               // pack
    int dim, wide;       // the pack's dimension; its entries carry the bag length (mean pooling)
    int n, start;        // occurrences of the pack, position of its first one in the packed order
    int c0;
    uint32_t width;
};

// Step 1 of an item: occurrences per rank, counted in LDS.  Returns this thread's share of
// the counters (`per` consecutive ones starting at tid * per), scanned over the block.
__device__ __forceinline__ int sort_count(const SortArgs& sa, const SortItem& it, int32_t* s_cnt, int* per_out,
                                          int* n_item)
{
    const int tid = threadIdx.x;
    const int32_t* inverse = sa.inverse;
    __syncthreads();                               // the previous use of s_cnt is over
    for (int i = tid; i < (int)it.width; i += kSortThreads) s_cnt[i] = 0;
    __syncthreads();
    for (int fi = it.tm.field_begin; fi < it.tm.field_end; ++fi) {
        const int f = sa.table_fields[fi];
        const int64_t q0 = (int64_t)sa.fb[f] + sa.delta[f], q1 = (int64_t)sa.fb[f + 1] + sa.delta[f];
        if (q0 < 0 || q1 > sa.nnz) continue;
        int64_t q = q0 + tid;
        for (; q + (kMarkUnroll - 1) * kSortThreads < q1; q += kMarkUnroll * kSortThreads) {
            uint32_t r[kMarkUnroll];
#pragma unroll
            for (int j = 0; j < kMarkUnroll; ++j) r[j] = (uint32_t)(inverse[q + j * kSortThreads] - it.c0);
#pragma unroll
            for (int j = 0; j < kMarkUnroll; ++j)
                if (r[j] < it.width) atomicAdd(&s_cnt[r[j]], 1);
        }
        for (; q < q1; q += kSortThreads) {
            const uint32_t r0 = (uint32_t)(inverse[q] - it.c0);
            if (r0 < it.width) atomicAdd(&s_cnt[r0], 1);
        }
    }
    __syncthreads();
    const int per = ((int)it.width + kSortThreads - 1) / kSortThreads;   // consecutive counters per thread
    int mine = 0;
    for (int j = 0; j < per; ++j) {
        const int i = tid * per + j;
        mine += i < (int)it.width ? s_cnt[i] : 0;
    }
    *per_out = per;
    return block_excl_scan<kSortThreads>(mine, n_item);
}

// Steps 2 and 3 of an item, given the occurrences of the pack before it: segment offsets,
// headers of the backward tiles, zeroed partial sums for long keys that cross tile
// boundaries; then every occurrence's gradient place goes to its segment's cursor.
__device__ __forceinline__ void sort_place(const SortArgs& sa, const SortItem& it, int32_t* s_cnt, int before,
                                           int ex, int per)
{
    const int tid = threadIdx.x;
    const int tp = sa.tp, n = it.n;
    const int32_t* inverse = sa.inverse;
    int32_t* seg = sa.seg_all + it.start + it.p;
    uint32_t* ent = sa.ent_all + (size_t)it.start * sa.ent_mult;
    const size_t tbase = (size_t)(it.start / tp + it.p);
    int4* th = sa.tile_hdr + tbase;
    double* gh = sa.ghot + tbase * sa.dmax;
    const bool wide = it.wide != 0;
    int s0 = before + ex;
    for (int j = 0; j < per; ++j) {
        const int i = tid * per + j;
        if (i < (int)it.width) {
            const int len = s_cnt[i];
            seg[it.c0 + i] = s0;
            s_cnt[i] = s0;                                 // from here on: the segment's next free position
            // headers of the backward tiles the segment overlaps: x = the key that holds the
            // tile's first position, y = the key that holds its last one, z = where the
            // tile's decoded window ends (its last key is decoded to its end unless it is long)
            for (int tt = s0 / tp; (int64_t)tt * tp < (int64_t)s0 + len; ++tt) {
                const int t_first = tt * tp, t_end = min(t_first + tp, n);
                if (t_first >= s0) th[tt].x = it.c0 + i;
                if (t_end - 1 < s0 + len) {
                    th[tt].y = it.c0 + i;
                    th[tt].z = len <= kWarmMax ? s0 + len : t_end;
                }
            }
            if (len > kWarmMax && s0 / tp != (s0 + len - 1) / tp) {
                const int slot = s0 / tp;                  // one such key at most starts in a tile
                for (int d = 0; d < it.dim; ++d) gh[(size_t)slot * it.dim + d] = 0.0;
            }
            s0 += len;
        }
    }
    __syncthreads();
    for (int fi = it.tm.field_begin; fi < it.tm.field_end; ++fi) {
        const int f = sa.table_fields[fi];
        const int64_t q0 = (int64_t)sa.fb[f] + sa.delta[f], q1 = (int64_t)sa.fb[f + 1] + sa.delta[f];
        if (q0 < 0 || q1 > sa.nnz) continue;
        int64_t q = q0 + tid;
        for (; q + (kSortUnroll2 - 1) * kSortThreads < q1; q += kSortUnroll2 * kSortThreads) {
            uint32_t r[kSortUnroll2], e[kSortUnroll2], c[kSortUnroll2];
#pragma unroll
            for (int j = 0; j < kSortUnroll2; ++j) {
                r[j] = (uint32_t)(inverse[q + j * kSortThreads] - it.c0);
                e[j] = sa.bagref[q + j * kSortThreads];
                c[j] = wide ? sa.baglen[q + j * kSortThreads] : 1u;
            }
#pragma unroll
            for (int j = 0; j < kSortUnroll2; ++j)
                if (r[j] < it.width) {
                    const int pos = atomicAdd(&s_cnt[r[j]], 1);
                    if ((unsigned)pos < (unsigned)n) {
                        if (wide) reinterpret_cast<uint2*>(ent)[pos] = make_uint2(e[j], c[j]);
                        else ent[pos] = e[j];
                    }
                }
        }
        for (; q < q1; q += kSortThreads) {
            const uint32_t r0 = (uint32_t)(inverse[q] - it.c0);
            if (r0 < it.width) {
                const int pos = atomicAdd(&s_cnt[r0], 1);
                if ((unsigned)pos < (unsigned)n) {
                    if (wide) reinterpret_cast<uint2*>(ent)[pos] = make_uint2(sa.bagref[q], sa.baglen[q]);
                    else ent[pos] = sa.bagref[q];
                }
            }
        }
    }
}

// `block` of `nblocks` blocks of kSortThreads threads; s_dyn: (4 T + 1) ints of LDS
__device__ __forceinline__ void sort_body(const SortArgs& sa, int block, int nblocks, int32_t* s_dyn)
{
    const TableMeta* __restrict__ tmeta = sa.tmeta;
    const int T = sa.T, P = sa.P;
    const PackMeta* __restrict__ pm = sa.pm;
    PackState* st = sa.st;
    const int32_t* __restrict__ fb = sa.fb;
    const uint4* __restrict__ bitmap4 = sa.bitmap4;
    const int32_t* __restrict__ rank = sa.rank;
    int32_t* s_rlo = s_dyn;                  // [T]   first rank of each table inside its pack
    int32_t* s_u = s_dyn + T;                // [T]   distinct keys of each table
    int32_t* s_first = s_u + T;              // [T+1] first work item of each table
    int32_t* s_occ = s_first + T + 1;        // [T]   occurrences in the tables before (all packs)
    __shared__ int32_t s_cnt[kSortCap];
    __shared__ uint32_t s_base;
    const int tid = threadIdx.x;
    if (st[0].error) return;
    int carry = 0, carry_occ = 0;
    for (int base = 0; base < T; base += kSortThreads) {
        const int t = base + tid;
        int chunks = 0, occ = 0;
        if (t < T) {
            const TableMeta tm = tmeta[t];
            for (int fi = tm.field_begin; fi < tm.field_end; ++fi) {
                const int f = sa.table_fields[fi];
                occ += fb[f + 1] - fb[f];
            }
            const PackMeta k = pm[tm.pack];
            const size_t rb = (size_t)k.first_tile * NT;
            const uint64_t key_end = (uint64_t)k.n_tiles * (uint64_t)(kTileWords * 32);
            const int nu = st[tm.pack].n_unique;
            const int r_lo = rank_of_key(bitmap4 + 2 * rb, rank + rb, tm.key_lo, key_end, nu);
            const int r_hi = rank_of_key(bitmap4 + 2 * rb, rank + rb, (uint64_t)tm.key_lo + tm.rows, key_end, nu);
            s_rlo[t] = r_lo;
            s_u[t] = r_hi - r_lo;
            chunks = (r_hi - r_lo + kSortCap - 1) / kSortCap;
        }
        int tot, tot_occ;
        const int ex = block_excl_scan<kSortThreads>(chunks, &tot);
        const int ex_occ = block_excl_scan<kSortThreads>(occ, &tot_occ);
        if (t < T) { s_first[t] = carry + ex; s_occ[t] = carry_occ + ex_occ; }
        carry += tot;
        carry_occ += tot_occ;
    }
    if (tid == 0) s_first[T] = carry;
    for (int p = block; p < P; p += nblocks)     // the entry after the last segment of each pack
        if (tid == 0) {
            const PackState ps = st[p];
            sa.seg_all[ps.start + p + ps.n_unique] = ps.nnz;
        }
    __syncthreads();
    const int total = s_first[T];
    for (int item = block; item < total; item += nblocks) {
        const int t = upper_bound_i32(s_first, T + 1, item) - 1;
        SortItem it;
        it.tm = tmeta[t];
        it.p = it.tm.pack;
        const PackMeta k = pm[it.p];
        it.dim = k.dim; it.wide = k.has_mean;
        it.n = st[it.p].nnz; it.start = st[it.p].start;
        const int chunk = item - s_first[t];
        it.c0 = s_rlo[t] + chunk * kSortCap;
        it.width = (uint32_t)min(kSortCap, s_rlo[t] + s_u[t] - it.c0);
        const uint32_t occ_before = (uint32_t)(s_occ[t] - s_occ[k.first_stable]);   // in the pack's earlier tables
        const int first_item = s_first[t];             // the table's first item: its start is known
        int per, n_item;
        const int ex = sort_count(sa, it, s_cnt, &per, &n_item);
        // occurrences before the item: those of the pack's earlier tables (known from the field
        // boundaries) plus those of the table's earlier items (descriptor look-back inside the table)
        if (tid < 64) {
            if (chunk == 0) {
                if (tid == 0) { publish_desc(sa.desc + item, make_desc(kDescPfx, (uint32_t)n_item, 0)); s_base = occ_before; }
            } else {
                if (tid == 0) publish_desc(sa.desc + item, make_desc(kDescAgg, (uint32_t)n_item, 0));
                uint32_t pa, pb;
                lookback(sa.desc, first_item, item, &pa, &pb, &st[0].error);
                if (tid == 0) {
                    publish_desc(sa.desc + item, make_desc(kDescPfx, pa + (uint32_t)n_item, 0));
                    s_base = occ_before + pa;
                }
            }
        }
        __syncthreads();
        sort_place(sa, it, s_cnt, (int)s_base, ex, per);
    }
}

__global__ void __launch_bounds__(kSortThreads, 8)
pk_sort_kernel(SortArgs sa)
{
    extern __shared__ int32_t s_dyn[];
    sort_body(sa, blockIdx.x, gridDim.x, s_dyn);
}
