// Device code and launch logic of the packed multi-field embedding layer for
// gfx950 (wave64).  The path is gather / reduce / scatter and is bound by HBM
// bandwidth, so there is no MFMA here: the work is in keeping every access
// coalesced across the embedding dimension, in touching each distinct row once
// (the point of Unique, Sec. II-D), and in launching once per pack instead of
// once per field (D-Packing, Sec. III-B).
//
// Stages of one step (all packs of the plan share the integer stages):
//   keys      H1: key = base_row + (uint64)id mod rows in packed order, packed bag offsets,
//             per occurrence the place of its bag's gradient chunk (and the bag length)
//   pool      H3-H5: per pack, gather rows by key, pool per bag, write concatenated
//   mark      H2: which rows occur (bitmap slices built in LDS)
//   tiles     H2: one-pass popcount scan of the bitmap -> rank samples, distinct keys (ascending)
//   inverse   H2: inverse[q] = rank(key[q])
//   sort      H2: occurrences grouped by distinct key (LDS counting sort), segment offsets,
//             headers of the backward tiles; small batches: pooling shares this launch
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

// ---------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------
namespace {

constexpr int NT = 256;   // threads per block of the streaming kernels

#ifndef PK_ADA_WAVES
#define PK_ADA_WAVES 6    // wavefronts per SIMD the backward kernel is compiled for (register budget)
#endif
#ifndef PK_ADA_WAVES_MEAN
#define PK_ADA_WAVES_MEAN 6
#endif
#ifndef PK_ADA_UNROLL
#define PK_ADA_UNROLL 4   // gradient chunks a lane group keeps in flight
#endif
#ifndef PK_ADA_UNROLL_MEAN
#define PK_ADA_UNROLL_MEAN 2
#endif

template <int NTHREADS>
__device__ __forceinline__ int block_excl_scan(int v, int* total)
{
    __shared__ int wsum[NTHREADS / 64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
    }
    __syncthreads();   // readers of the previous call are done with wsum
    if (lane == 63) wsum[w] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NTHREADS / 64; ++i) {
        int s = wsum[i];
        if (i < w) base += s;
        tot += s;
    }
    *total = tot;
    return base + inc - v;
}

__device__ __forceinline__ uint32_t fold_id(int64_t id, uint32_t rows)
{
    const uint64_t u = (uint64_t)id;
    return u < rows ? (uint32_t)u : (uint32_t)(u % (uint64_t)rows);
}

// first index in [0, n) whose value exceeds x, for a non-decreasing array
template <typename P>
__device__ __forceinline__ int upper_bound_i32(P a, int n, int x)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (a[mid] <= x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// ---------------------------------------------------------------------------
// single-pass multi-block prefix sums: every tile publishes a 64-bit
// descriptor (state | value b | value a) and sums the descriptors of the tiles
// before it.  A block takes tiles b, b + G, ...; a tile of a later round waits
// for tiles of the round before, of every block, so the wait ends when all G
// blocks are resident together: the launches keep G below what the chip holds
// of that kernel alone.  (Two such kernels side by side on one GPU can hold
// each other's places; calls of this library on one device are meant to follow
// one another.)  The wait is bounded all the same: running out of patience sets
// bit 1 of the error word, the kernels after it skip their work and the tables
// stay as they are.
// ---------------------------------------------------------------------------
constexpr uint64_t kDescAgg = 1, kDescPfx = 2;
constexpr int kSpinLimit = 1 << 22;

__device__ __forceinline__ uint64_t make_desc(uint64_t state, uint32_t a, uint32_t b)
{
    return (state << 62) | ((uint64_t)b << 31) | (uint64_t)a;
}

__device__ __forceinline__ void publish_desc(uint64_t* d, uint64_t v)
{
    __hip_atomic_store(d, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Sum of (a, b) over tiles [first, me).  Called by all 64 lanes of one wave.
__device__ __forceinline__ void lookback(uint64_t* desc, int first, int me, uint32_t* out_a, uint32_t* out_b,
                                         int32_t* error_word)
{
    const int lane = threadIdx.x & 63;
    uint32_t acc_a = 0, acc_b = 0;
    int hi = me;
    bool done = false;
    while (hi > first && !done) {
        const int idx = hi - 1 - lane;
        const bool valid = idx >= first;
        uint64_t d = make_desc(kDescPfx, 0, 0);
        int spins = 0;
        while (true) {
            if (valid) d = __hip_atomic_load(desc + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const bool ready = (d >> 62) != 0;
            if (__ballot(ready) == ~0ull) break;
            if (++spins > kSpinLimit) {
                if (lane == 0) atomicOr(error_word, 2);
                d = make_desc(kDescPfx, 0, 0);
                break;
            }
            __builtin_amdgcn_s_sleep(2);
        }
        const uint64_t pfx_mask = __ballot((d >> 62) == kDescPfx);
        int last = 64;                                   // lanes [0, last] contribute
        if (pfx_mask) { last = __ffsll((unsigned long long)pfx_mask) - 1; done = true; }
        if (lane <= last) {
            acc_a += (uint32_t)(d & 0x7FFFFFFFull);
            acc_b += (uint32_t)((d >> 31) & 0x7FFFFFFFull);
        }
        hi -= 64;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        acc_a += __shfl_xor(acc_a, o, 64);
        acc_b += __shfl_xor(acc_b, o, 64);
    }
    *out_a = acc_a;
    *out_b = acc_b;
}

// Workgroups are handed to the 8 XCDs round-robin and each XCD has its own L2.
// Giving XCD x the x-th contiguous eighth of the tiles keeps the irregular
// accesses of neighbouring tiles (same table, same gradient columns) in one L2.
// Only locality depends on this; any placement gives the same results.
struct XcdTiles {
    int tile, hi, step;
    __device__ __forceinline__ XcdTiles(int n_tiles)
    {
        const int x = blockIdx.x & 7, i = blockIdx.x >> 3;
        const int chunk = (n_tiles + 7) >> 3;
        step = (gridDim.x + 7) >> 3;
        tile = x * chunk + i;
        hi = min((x + 1) * chunk, n_tiles);
    }
    __device__ __forceinline__ bool valid() const { return tile < hi; }
    __device__ __forceinline__ void next() { tile += step; }
};

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

// ---------------------------------------------------------------------------
// row access: VEC consecutive elements of a table row as floats
// ---------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);      // round to nearest, ties to even (finite inputs)
    return u >> 16;
}

template <typename WT, int VEC> struct Row;

template <> struct Row<float, 4> {
    static __device__ __forceinline__ void load(const float* p, float* v)
    { const float4 x = *reinterpret_cast<const float4*>(p); v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; }
    static __device__ __forceinline__ void store(float* p, const float* v)
    { *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]); }
};
template <> struct Row<float, 1> {
    static __device__ __forceinline__ void load(const float* p, float* v) { v[0] = *p; }
    static __device__ __forceinline__ void store(float* p, const float* v) { *p = v[0]; }
};
template <> struct Row<uint16_t, 8> {
    static __device__ __forceinline__ void load(const uint16_t* p, float* v)
    {
        const uint4 x = *reinterpret_cast<const uint4*>(p);
        v[0] = bf16_to_f32(x.x & 0xFFFFu); v[1] = bf16_to_f32(x.x >> 16);
        v[2] = bf16_to_f32(x.y & 0xFFFFu); v[3] = bf16_to_f32(x.y >> 16);
        v[4] = bf16_to_f32(x.z & 0xFFFFu); v[5] = bf16_to_f32(x.z >> 16);
        v[6] = bf16_to_f32(x.w & 0xFFFFu); v[7] = bf16_to_f32(x.w >> 16);
    }
    static __device__ __forceinline__ void store(uint16_t* p, const float* v)
    {
        uint4 x;
        x.x = f32_to_bf16(v[0]) | (f32_to_bf16(v[1]) << 16);
        x.y = f32_to_bf16(v[2]) | (f32_to_bf16(v[3]) << 16);
        x.z = f32_to_bf16(v[4]) | (f32_to_bf16(v[5]) << 16);
        x.w = f32_to_bf16(v[6]) | (f32_to_bf16(v[7]) << 16);
        *reinterpret_cast<uint4*>(p) = x;
    }
};
template <> struct Row<uint16_t, 1> {
    static __device__ __forceinline__ void load(const uint16_t* p, float* v) { v[0] = bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(uint16_t* p, const float* v) { *p = (uint16_t)f32_to_bf16(v[0]); }
};

// VEC consecutive floats of out / grad_out / the accumulators.  The vector
// kernels (VEC a multiple of 4) are only launched when the host has checked that
// every such address is 16-byte aligned; otherwise the one-element-per-lane
// kernels run.
template <int VEC>
__device__ __forceinline__ void load_f32(const float* p, float* v)
{
    if constexpr (VEC % 4 == 0) {
#pragma unroll
        for (int i = 0; i < VEC; i += 4) {
            const float4 x = *reinterpret_cast<const float4*>(p + i);
            v[i] = x.x; v[i + 1] = x.y; v[i + 2] = x.z; v[i + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = p[i];
    }
}

template <int VEC>
__device__ __forceinline__ void store_f32(float* p, const float* v)
{
    if constexpr (VEC % 4 == 0) {
#pragma unroll
        for (int i = 0; i < VEC; i += 4)
            *reinterpret_cast<float4*>(p + i) = make_float4(v[i], v[i + 1], v[i + 2], v[i + 3]);
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) p[i] = v[i];
    }
}

// ---------------------------------------------------------------------------
// Where a row lives.  Plain tables: row r of the pack's table.  With HybridHash
// (Sec. III-D) the table passed to the kernel is the Cold-storage (every row) and
// the frequently queried rows live, and are updated, in a small Hot-storage:
// slot_of[r] >= 0 names the row's slot there.  slot_of == nullptr: no Hot-storage.
// ---------------------------------------------------------------------------
struct HotView {
    const int32_t* slot_of;
    void* W_hot;
    float* A_hot;
};

template <typename WT, bool HYB>
__device__ __forceinline__ WT* row_of(WT* cold, const HotView& hv, uint32_t row, int D)
{
    if constexpr (HYB) {
        const int s = hv.slot_of[row];
        if (s >= 0) return static_cast<WT*>(hv.W_hot) + (size_t)s * D;
    }
    return cold + (size_t)row * D;
}

// the row's weights and its accumulator
template <typename WT>
__device__ __forceinline__ void rows_of(WT* W, float* A, const HotView& hv, uint32_t row, int D, WT** wrow, float** arow)
{
    if (hv.slot_of) {
        const int s = hv.slot_of[row];
        if (s >= 0) {
            *wrow = static_cast<WT*>(hv.W_hot) + (size_t)s * D;
            *arow = hv.A_hot + (size_t)s * D;
            return;
        }
    }
    *wrow = W + (size_t)row * D;
    *arow = A + (size_t)row * D;
}

// ---------------------------------------------------------------------------
// H3+H4+H5: Gather and SegmentReduction (Sec. II-D) fused (K-Packing, Sec.
// III-B: both are memory-bound), one launch per pack.  A group of LPR lanes owns
// one bag; each lane covers VEC (x NCH) columns, so a row is read with one
// coalesced access.  The concatenation of the fields of a sample is the write
// address.
// ---------------------------------------------------------------------------
// `block` of `nblocks` blocks of `nthreads` threads; HYB: rows may live in a Hot-storage;
// DEEP: eight rows of a bag in flight instead of four (the kernel that shares the sort's
// launch has no registers for that)
template <typename WT, int VEC, int LPR, int NCH, bool HYB, bool DEEP>
__device__ __forceinline__ void pool_body(const WT* __restrict__ W, const uint32_t* __restrict__ keys_all,
                                          const int32_t* __restrict__ po, const PackState* __restrict__ st,
                                          const FieldMeta* __restrict__ fmeta, const int32_t* __restrict__ slot_field,
                                          int B, int D, int64_t n_bags, float* __restrict__ out, int64_t out_stride,
                                          int block, int nblocks, int nthreads, const HotView hv)
{
    const int GPB = nthreads / LPR;
    const int li = threadIdx.x % LPR, gi = threadIdx.x / LPR;
    const int n = st->nnz;
    const uint32_t* keys = keys_all + st->start;
    for (int64_t bag = (int64_t)block * GPB + gi; bag < n_bags; bag += (int64_t)nblocks * GPB) {
        const int j = (int)(bag / B);
        const int b = (int)(bag - (int64_t)j * B);
        const FieldMeta m = fmeta[slot_field[j]];
        const int q0 = min(max(po[bag], 0), n);
        const int q1 = min(max(po[bag + 1], q0), n);
        float acc[NCH][VEC];
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[c][v] = 0.f;
        int q = q0;
        if (DEEP) {                                        // eight rows in flight where the registers allow it
            for (; q + 8 <= q1; q += 8) {
                const WT* r[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) r[k] = row_of<const WT, HYB>(W, hv, keys[q + k], D);
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    const int d0 = (c * LPR + li) * VEC;
                    if (d0 < D) {
                        float x[8][VEC];
#pragma unroll
                        for (int k = 0; k < 8; ++k) Row<WT, VEC>::load(r[k] + d0, x[k]);
#pragma unroll
                        for (int v = 0; v < VEC; ++v) {        // the order of additions of two rounds of four
                            acc[c][v] += (x[0][v] + x[1][v]) + (x[2][v] + x[3][v]);
                            acc[c][v] += (x[4][v] + x[5][v]) + (x[6][v] + x[7][v]);
                        }
                    }
                }
            }
        }
        for (; q + 4 <= q1; q += 4) {
            const WT* r0 = row_of<const WT, HYB>(W, hv, keys[q], D);
            const WT* r1 = row_of<const WT, HYB>(W, hv, keys[q + 1], D);
            const WT* r2 = row_of<const WT, HYB>(W, hv, keys[q + 2], D);
            const WT* r3 = row_of<const WT, HYB>(W, hv, keys[q + 3], D);
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int d0 = (c * LPR + li) * VEC;
                if (d0 < D) {
                    float x0[VEC], x1[VEC], x2[VEC], x3[VEC];
                    Row<WT, VEC>::load(r0 + d0, x0);
                    Row<WT, VEC>::load(r1 + d0, x1);
                    Row<WT, VEC>::load(r2 + d0, x2);
                    Row<WT, VEC>::load(r3 + d0, x3);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[c][v] += (x0[v] + x1[v]) + (x2[v] + x3[v]);
                }
            }
        }
        for (; q < q1; ++q) {
            const WT* r0 = row_of<const WT, HYB>(W, hv, keys[q], D);
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int d0 = (c * LPR + li) * VEC;
                if (d0 < D) {
                    float x0[VEC];
                    Row<WT, VEC>::load(r0 + d0, x0);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[c][v] += x0[v];
                }
            }
        }
        const float scale = (m.pool == PK_MEAN && q1 > q0) ? 1.0f / (float)(q1 - q0) : 1.0f;
        float* o = out + (size_t)b * out_stride + m.col;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int d0 = (c * LPR + li) * VEC;
            if (d0 < D) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[c][v] *= scale;
                store_f32<VEC>(o + d0, acc[c]);
            }
        }
    }
}

template <typename WT, int VEC, int LPR, int NCH, bool HYB>
__global__ void __launch_bounds__(NT)
pk_pool_kernel(const WT* __restrict__ W, const uint32_t* __restrict__ keys_all, const int32_t* __restrict__ po,
               const PackState* __restrict__ st, const FieldMeta* __restrict__ fmeta,
               const int32_t* __restrict__ slot_field, int B, int D, int64_t n_bags,
               float* __restrict__ out, int64_t out_stride, const HotView hv)
{
    pool_body<WT, VEC, LPR, NCH, HYB, true>(W, keys_all, po, st, fmeta, slot_field, B, D, n_bags, out, out_stride,
                                      blockIdx.x, gridDim.x, NT, hv);
}

// Small batches: the sort kernel has few work items (one per table) and leaves most of the
// chip idle, and the pooling of all packs depends on the keys only, so both run in ONE
// launch: the first `sort_blocks` blocks sort, the others pool.  (Side streams do the same
// for large batches; for small ones a cross-stream dependency costs more than it hides.)
constexpr int kFusedPacks = 16;
struct PoolPack {
    const void* W; const int32_t* po; const int32_t* slot_field;
    int64_t n_bags; int32_t D; int32_t variant; int32_t block_begin; int32_t pad;   // pad: the pack's index
};
struct PoolJob {
    PoolPack pack[kFusedPacks];
    int32_t n_packs; int32_t B; int32_t n_blocks; int32_t pad;
    const uint32_t* keys; const PackState* st; const FieldMeta* fmeta; float* out; int64_t out_stride;
};

// variant = 12 * dtype + shape; the shapes in the order of the host's dispatch
#define PK_POOL_SHAPES(WT, VECW, base)                                                          \
    case base + 0:  pool_body<WT, VECW, 1, 1, false, false>(PK_POOL_ARGS); break;                       \
    case base + 1:  pool_body<WT, VECW, 2, 1, false, false>(PK_POOL_ARGS); break;                       \
    case base + 2:  pool_body<WT, VECW, 4, 1, false, false>(PK_POOL_ARGS); break;                       \
    case base + 3:  pool_body<WT, VECW, 8, 1, false, false>(PK_POOL_ARGS); break;                       \
    case base + 4:  pool_body<WT, VECW, 16, 1, false, false>(PK_POOL_ARGS); break;                      \
    case base + 5:  pool_body<WT, VECW, 32, 1, false, false>(PK_POOL_ARGS); break;                      \
    case base + 6:  pool_body<WT, VECW, 64, 1, false, false>(PK_POOL_ARGS); break;                      \
    case base + 7:  pool_body<WT, 1, 4, 1, false, false>(PK_POOL_ARGS); break;                          \
    case base + 8:  pool_body<WT, 1, 16, 1, false, false>(PK_POOL_ARGS); break;                         \
    case base + 9:  pool_body<WT, 1, 64, 1, false, false>(PK_POOL_ARGS); break;                         \
    case base + 10: pool_body<WT, 1, 64, 2, false, false>(PK_POOL_ARGS); break;                         \
    case base + 11: pool_body<WT, 1, 64, 4, false, false>(PK_POOL_ARGS); break;
#define PK_POOL_ARGS                                                                            \
    static_cast<const WT_*>(k.W), pj.keys, k.po, pj.st + k.pad, pj.fmeta, k.slot_field, pj.B, k.D, k.n_bags, pj.out,  \
        pj.out_stride, local, n_local, kSortThreads, HotView{nullptr, nullptr, nullptr}

__global__ void __launch_bounds__(kSortThreads, 8)
pk_sort_pool_kernel(SortArgs sa, PoolJob pj, int sort_blocks)
{
    extern __shared__ int32_t s_dyn[];
    if ((int)blockIdx.x < sort_blocks) {
        sort_body(sa, blockIdx.x, sort_blocks, s_dyn);
        return;
    }
    const int pb = (int)blockIdx.x - sort_blocks;
    int p = 0;
    while (p + 1 < pj.n_packs && pb >= pj.pack[p + 1].block_begin) ++p;
    const PoolPack k = pj.pack[p];
    const int local = pb - k.block_begin;
    const int n_local = (p + 1 < pj.n_packs ? pj.pack[p + 1].block_begin : pj.n_blocks) - k.block_begin;
    switch (k.variant) {
        {
            using WT_ = float;
            PK_POOL_SHAPES(float, 4, 0)
        }
        {
            using WT_ = uint16_t;
            PK_POOL_SHAPES(uint16_t, 8, 12)
        }
    }
}

// ---------------------------------------------------------------------------
// H6+H7: per distinct key, the gradients of its occurrences are reduced in
// double (mirror of the forward pooling, Sec. II-D) and the row takes one
// Adagrad step in place.  Fused so the reduced gradient never goes to memory.
//
// Work is cut by OCCURRENCES, not by keys, because the ID distribution is
// heavily skewed (Sec. II-B): a block takes a tile of consecutive positions of
// the key-sorted occurrence list and handles the keys that start there.
//   up to kColdMax occurrences: one lane group per key;
//   up to kWarmMax, or inside
//   one tile:                   one wavefront per key, groups stride over it;
//   longer, across tiles:       the whole block reduces the tile's piece of the key and
//                               adds it with double atomics to the key's row of partial
//                               sums (indexed by the tile the key starts in);
//                               pk_adagrad_hot_kernel then applies the update.
// ---------------------------------------------------------------------------
// The gradient chunks of a tile's occurrences: element offsets into grad_out and
// mean-pooling scales, decoded once per tile, in parallel, into LDS.
template <bool MEAN>
struct GradSrc {
    const float* grad;
    const uint32_t* s_addr;      // LDS: positions [t0, ...)
    const double* s_scl;         // LDS: 1/L per position (packs with mean pooling only)
    int t0;
    __device__ __forceinline__ void fetch(int s, uint32_t* addr, double* scale) const
    {
        *addr = s_addr[s - t0];
        *scale = MEAN ? s_scl[s - t0] : 1.0;
    }
};

// acc += sum over positions s, s+step, ... < s_end of scale * grad chunk.  Packs with
// mean pooling carry a double per chunk in flight, so they keep fewer in flight.
template <int VEC, int LPR, int NCH, bool MEAN>
__device__ __forceinline__ void accum_range(double (&acc)[NCH][VEC], const GradSrc<MEAN>& g, int D, int li,
                                            int s, int s_end, int step)
{
    constexpr int UN = MEAN ? PK_ADA_UNROLL_MEAN : PK_ADA_UNROLL;
    for (; s + (UN - 1) * step < s_end; s += UN * step) {
        uint32_t a[UN];
        double c[UN];
#pragma unroll
        for (int k = 0; k < UN; ++k) g.fetch(s + k * step, &a[k], &c[k]);
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const int d0 = (ch * LPR + li) * VEC;
            if (d0 < D) {
                float x[UN][VEC];
#pragma unroll
                for (int k = 0; k < UN; ++k) load_f32<VEC>(g.grad + a[k] + d0, x[k]);
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    double t = 0.0;
#pragma unroll
                    for (int k = 0; k < UN; ++k) t += MEAN ? c[k] * (double)x[k][v] : (double)x[k][v];
                    acc[ch][v] += t;
                }
            }
        }
    }
    for (; s < s_end; s += step) {
        uint32_t a0;
        double c0;
        g.fetch(s, &a0, &c0);
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const int d0 = (ch * LPR + li) * VEC;
            if (d0 < D) {
                float x0[VEC];
                load_f32<VEC>(g.grad + a0 + d0, x0);
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[ch][v] += MEAN ? c0 * (double)x0[v] : (double)x0[v];
            }
        }
    }
}

// the row's current weights and accumulators (issued before the gradient
// reduction so that both sets of loads are in flight together)
template <typename WT, int VEC, int LPR, int NCH>
__device__ __forceinline__ void row_load(const WT* wrow, const float* arow, int D, int li,
                                         float (&w)[NCH][VEC], float (&a)[NCH][VEC])
{
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int d0 = (c * LPR + li) * VEC;
        if (d0 < D) {
            Row<WT, VEC>::load(wrow + d0, w[c]);
            load_f32<VEC>(arow + d0, a[c]);
        }
    }
}

// one Adagrad step of the row: a += g^2 ; w -= lr * g / (sqrt(a) + eps)
template <typename WT, int VEC, int LPR, int NCH>
__device__ __forceinline__ void row_step(WT* wrow, float* arow, int D, int li,
                                         const double (&acc)[NCH][VEC], float (&w)[NCH][VEC],
                                         float (&a)[NCH][VEC], float lr, float eps)
{
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int d0 = (c * LPR + li) * VEC;
        if (d0 < D) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const float g = (float)acc[c][v];
                a[c][v] = a[c][v] + g * g;
                w[c][v] = w[c][v] - lr * g / (sqrtf(a[c][v]) + eps);
            }
            store_f32<VEC>(arow + d0, a[c]);
            Row<WT, VEC>::store(wrow + d0, w[c]);
        }
    }
}

// sum over the lane groups of a wavefront (butterfly); every lane ends with the total
template <int VEC, int LPR, int NCH>
__device__ __forceinline__ void wave_group_sum(double (&acc)[NCH][VEC])
{
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1)
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[c][v] += __shfl_xor(acc[c][v], o, 64);
}

template <typename WT, int VEC, int LPR, int NCH, bool MEAN>
__global__ void __launch_bounds__(NT, VEC > 4 ? 1 : (MEAN ? PK_ADA_WAVES_MEAN : PK_ADA_WAVES))   // 8-wide rows need their registers
pk_adagrad_kernel(WT* W, float* A, const PackState* __restrict__ st, int p,
                  const uint32_t* __restrict__ unique_all, const int32_t* __restrict__ seg_all,
                  double* ghot_all, int dmax, const int4* __restrict__ tile_hdr, int tp, int n_host,
                  const uint32_t* __restrict__ seg_ent_all, int ent_mult,
                  const float* __restrict__ grad, int64_t gstride, int64_t out_dim, uint32_t addr_max, int D,
                  float lr, float eps, const HotView hv)
{
    constexpr int GPB = NT / LPR;          // lane groups per block
    constexpr int GPW = 64 / LPR;          // lane groups per wavefront
    __shared__ int s_nwarm, s_nhot;
    __shared__ int s_warm[kPosTileMax / (kColdMax + 1) + 2];
    __shared__ int s_hot[kPosTileMax / (kWarmMax + 1) + 4];
    __shared__ double s_red[NT / 64][LPR][NCH][VEC];   // per-wavefront partial sums of a hot piece
    __shared__ int s_seg[kPosTileMax + 2];          // segment offsets of the tile's keys
    __shared__ uint32_t s_row[kPosTileMax + 1];     // their table rows
    __shared__ uint32_t s_addr[kPosTileMax + kWarmMax];   // decoded positions of the tile and its tail
    __shared__ double s_scl[MEAN ? kPosTileMax + kWarmMax : 1];   // 1/L of mean pooling, in double: see the decode below
    const int li = threadIdx.x % LPR, gi = threadIdx.x / LPR;
    const int wv = threadIdx.x >> 6, gw = (threadIdx.x & 63) / LPR;
    // A plan with one pack has all occurrences in it, so the host knows the sizes and the first
    // tile header can be requested without waiting for the pack's state; the state is still
    // checked.  A forward pass that raised the error word (input rejected, or a scan that ran
    // out of patience) left no lists worth reading: the tables are then left alone.
    const int n = n_host >= 0 ? n_host : st->nnz, start = n_host >= 0 ? 0 : st->start;
    const bool state_ok = (n_host < 0 || st->nnz == n_host) && (st - p)->error == 0;
    const int32_t* seg = seg_all + start + p;
    const uint32_t* uq = unique_all + start;
    const size_t tbase = (size_t)(start / tp + p);
    double* gh = ghot_all + tbase * dmax;
    const int4* th = tile_hdr + tbase;
    const uint32_t* ent = seg_ent_all + (size_t)start * ent_mult;
    GradSrc<MEAN> g{grad, s_addr, s_scl, 0};
    const int n_tiles = (n + tp - 1) / tp;
    for (XcdTiles it(n_tiles); it.valid(); it.next()) {
        const int tile = it.tile;
        const int t0 = tile * tp, t1 = min(t0 + tp, n);
        // keys whose segments overlap [t0, t1), and the decode window: the tile, plus the tail
        // of its last key unless that key is a long one (long keys are cut at the tile's end).
        // The clamps keep the LDS arrays in bounds whatever the header holds.
        const int4 hdr = th[tile];
        if (!state_ok) return;
        const int u_lo = hdr.x;
        const int nseg = min(max(hdr.y - u_lo + 1, 0), tp);
        const int w_end = min(max(hdr.z, t1), t1 + kWarmMax);
        __syncthreads();                                   // the previous tile's LDS is consumed
        for (int i = threadIdx.x; i <= nseg; i += NT) s_seg[i] = seg[u_lo + i];
        for (int i = threadIdx.x; i < nseg; i += NT) s_row[i] = uq[u_lo + i];
        for (int i = threadIdx.x; i < w_end - t0; i += NT) {
            // The 1/L of mean pooling is formed and applied in double.  The first Adagrad step
            // of a row moves a weight by lr*g/(|g|+eps): where the gradients of a key cancel
            // (|g| near eps) an error of 1e-8 in g is an error of lr in the weight, and a
            // float 1/L alone is off by 6e-8 of every term.
            uint32_t a;
            double c = 1.0;
            if (MEAN) {
                const uint2 e = reinterpret_cast<const uint2*>(ent)[t0 + i];
                a = e.x;
                c = 1.0 / (double)max(e.y, 1u);
            } else {
                a = ent[t0 + i];
            }
            if (gstride != out_dim) {                      // padded gradient rows
                const uint32_t b = a / (uint32_t)out_dim;
                a = b * (uint32_t)gstride + (a - b * (uint32_t)out_dim);
            }
            if (a > addr_max) { a = 0; c = 0.0; }          // never leave grad_out, whatever the list holds
            s_addr[i] = a;
            if (MEAN) s_scl[i] = c;
        }
        if (threadIdx.x == 0) { s_nwarm = 0; s_nhot = 0; }
        g.t0 = t0;
        __syncthreads();
        // cold keys that start here are finished on the spot; the others are listed
        for (int k = gi; k < nseg; k += GPB) {
            const int s0 = s_seg[k], s1 = s_seg[k + 1];
            const int len = s1 - s0;
            if (len <= kColdMax) {
                if (s0 >= t0) {
                    WT* wrow;
                    float* arow;
                    rows_of<WT>(W, A, hv, s_row[k], D, &wrow, &arow);
                    float w[NCH][VEC], a[NCH][VEC];
                    row_load<WT, VEC, LPR, NCH>(wrow, arow, D, li, w, a);
                    double acc[NCH][VEC];
#pragma unroll
                    for (int c = 0; c < NCH; ++c)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) acc[c][v] = 0.0;
                    accum_range<VEC, LPR, NCH, MEAN>(acc, g, D, li, s0, s1, 1);
                    row_step<WT, VEC, LPR, NCH>(wrow, arow, D, li, acc, w, a, lr, eps);
                }
            } else if (len <= kWarmMax || (s0 >= t0 && s1 <= t1)) {   // fits the decoded window
                if (s0 >= t0 && li == 0) s_warm[atomicAdd(&s_nwarm, 1)] = k;
            } else if (li == 0) {
                s_hot[atomicAdd(&s_nhot, 1)] = k;
            }
        }
        __syncthreads();
        // warm keys that start here: one wavefront each
        const int n_warm = s_nwarm;
        for (int i = wv; i < n_warm; i += NT / 64) {
            const int k = s_warm[i];
            const int s0 = s_seg[k], s1 = s_seg[k + 1];
            WT* wrow;
            float* arow;
            rows_of<WT>(W, A, hv, s_row[k], D, &wrow, &arow);
            float w[NCH][VEC], a[NCH][VEC];
            if (gw == 0) row_load<WT, VEC, LPR, NCH>(wrow, arow, D, li, w, a);
            double acc[NCH][VEC];
#pragma unroll
            for (int c = 0; c < NCH; ++c)
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[c][v] = 0.0;
            accum_range<VEC, LPR, NCH, MEAN>(acc, g, D, li, s0 + gw, s1, GPW);
            wave_group_sum<VEC, LPR, NCH>(acc);
            if (gw == 0) row_step<WT, VEC, LPR, NCH>(wrow, arow, D, li, acc, w, a, lr, eps);
        }
        // long keys that cross tile boundaries: the tile's piece is split over the block's
        // wavefronts, reduced in LDS and added to the key's partial sums;
        // pk_adagrad_hot_kernel finishes those keys.
        const int n_hot_here = s_nhot;
        for (int i = 0; i < n_hot_here; ++i) {
            const int k = s_hot[i];
            const int s0 = s_seg[k], s1 = s_seg[k + 1];
            const int a0 = max(s0, t0), b0 = min(s1, t1);
            const int share = (b0 - a0 + NT / 64 - 1) / (NT / 64);
            const int c0 = a0 + wv * share, c1 = min(c0 + share, b0);
            double acc[NCH][VEC];
#pragma unroll
            for (int c = 0; c < NCH; ++c)
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[c][v] = 0.0;
            accum_range<VEC, LPR, NCH, MEAN>(acc, g, D, li, c0 + gw, c1, GPW);
            wave_group_sum<VEC, LPR, NCH>(acc);
            __syncthreads();                               // s_red of the previous piece is consumed
            if (gw == 0) {
#pragma unroll
                for (int c = 0; c < NCH; ++c)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) s_red[wv][li][c][v] = acc[c][v];
            }
            __syncthreads();
            if (wv == 0 && gw == 0) {
#pragma unroll
                for (int c = 0; c < NCH; ++c)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        double t = 0.0;
#pragma unroll
                        for (int w2 = 0; w2 < NT / 64; ++w2) t += s_red[w2][li][c][v];
                        acc[c][v] = t;
                    }
                {
                    double* prow = gh + (size_t)(s0 / tp) * D; // partial sums, indexed by the tile the key starts in
#pragma unroll
                    for (int c = 0; c < NCH; ++c) {
                        const int d0 = (c * LPR + li) * VEC;
                        if (d0 < D) {
#pragma unroll
                            for (int v = 0; v < VEC; ++v) atomicAdd(prow + d0 + v, acc[c][v]);
                        }
                    }
                }
            }
        }
    }
}

// Keys that are long and cross tile boundaries: their partial sums are complete
// once pk_adagrad_kernel has ended; apply the update.  One wavefront per tile
// looks at the key that runs out of the tile's end and takes it if it starts in
// this tile (so every such key is taken exactly once).  All packs in one launch;
// there are few such keys, so a row is handled one element per lane.
struct HotPacks {
    void* W[16];
    float* A[16];
    HotView hv[16];
};

__global__ void __launch_bounds__(NT)
pk_adagrad_hot_kernel(HotPacks ptrs, int p0, const PackMeta* __restrict__ pm, const PackState* __restrict__ st,
                      const uint32_t* __restrict__ unique_all, const int32_t* __restrict__ seg_all,
                      const double* __restrict__ ghot_all, int dmax, const int4* __restrict__ tile_hdr, int tp,
                      float lr, float eps)
{
    const int p = p0 + blockIdx.y;
    const PackMeta k = pm[p];
    if (st[0].error) return;                               // as in pk_adagrad_kernel
    const int n = st[p].nnz, start = st[p].start, D = k.dim;
    const int32_t* seg = seg_all + start + p;
    const size_t tbase = (size_t)(start / tp + p);
    const double* gh = ghot_all + tbase * dmax;
    const int4* th = tile_hdr + tbase;
    const int n_tiles = (n + tp - 1) / tp;
    const int lane = threadIdx.x & 63;
    for (int t = blockIdx.x * (NT / 64) + (threadIdx.x >> 6); t + 1 < n_tiles; t += gridDim.x * (NT / 64)) {
        const int u = th[t + 1].x;                             // the key that holds the next tile's first position
        const int s0 = seg[u], s1 = seg[u + 1];
        if (s0 < t * tp || s0 >= (t + 1) * tp || s1 - s0 <= kWarmMax) continue;
        const uint32_t row = unique_all[start + u];
        if (k.dtype == PK_F32) {
            float* wrow;
            float* arow;
            rows_of<float>(static_cast<float*>(ptrs.W[blockIdx.y]), ptrs.A[blockIdx.y], ptrs.hv[blockIdx.y], row, D, &wrow, &arow);
            for (int d = lane; d < D; d += 64) {
                const float g = (float)gh[(size_t)t * D + d];
                const float a = arow[d] + g * g;
                arow[d] = a;
                wrow[d] = wrow[d] - lr * g / (sqrtf(a) + eps);
            }
        } else {
            uint16_t* wrow;
            float* arow;
            rows_of<uint16_t>(static_cast<uint16_t*>(ptrs.W[blockIdx.y]), ptrs.A[blockIdx.y], ptrs.hv[blockIdx.y], row, D, &wrow, &arow);
            for (int d = lane; d < D; d += 64) {
                const float g = (float)gh[(size_t)t * D + d];
                const float a = arow[d] + g * g;
                arow[d] = a;
                wrow[d] = (uint16_t)f32_to_bf16(bf16_to_f32(wrow[d]) - lr * g / (sqrtf(a) + eps));
            }
        }
    }
}

// ---------------------------------------------------------------------------
// HybridHash (Sec. III-D, Alg. 1): bookkeeping of the Hot-storage.
// ---------------------------------------------------------------------------
constexpr int kHhBins = 65536;         // histogram of FCounter values; larger counts share the last bin
constexpr int kHhTile = 2048;          // rows per block of the selection kernels

// FCounter(id) += 1 for the distinct rows the batch queried; hits = those found in the Hot-storage
__global__ void __launch_bounds__(NT)
pk_hh_count_kernel(const PackState* __restrict__ st, int p, const uint32_t* __restrict__ unique_all,
                   const int32_t* __restrict__ slot_of, uint32_t* __restrict__ fcounter,
                   unsigned long long* counters)
{
    __shared__ int s_hits[NT / 64];
    const int U = st[p].n_unique;
    const uint32_t* uq = unique_all + st[p].start;
    int hits = 0;
    for (int u = blockIdx.x * NT + threadIdx.x; u < U; u += gridDim.x * NT) {
        const uint32_t row = uq[u];
        fcounter[row] += 1;                      // the distinct rows are distinct: no two threads share one
        hits += slot_of[row] >= 0;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) hits += __shfl_xor(hits, o, 64);
    if ((threadIdx.x & 63) == 0) s_hits[threadIdx.x >> 6] = hits;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
        for (int i = 0; i < NT / 64; ++i) t += s_hits[i];
        if (t) atomicAdd(&counters[2 * p + 1], (unsigned long long)t);
        if (blockIdx.x == 0) counters[2 * p] = (unsigned long long)U;
    }
}

// Rows leaving the Hot-storage are written back to the Cold-storage (one wavefront per row,
// lanes over its elements) ...
template <typename WT>
__global__ void __launch_bounds__(NT)
pk_hh_evict_kernel(WT* W_cold, float* A_cold, const WT* __restrict__ W_hot, const float* __restrict__ A_hot,
                   const uint32_t* __restrict__ hot_row, int32_t* slot_of, const int32_t* __restrict__ evict_slot,
                   const uint32_t* __restrict__ counts, int D)
{
    const int n = (int)counts[0], lane = threadIdx.x & 63;
    for (int i = blockIdx.x * (NT / 64) + (threadIdx.x >> 6); i < n; i += gridDim.x * (NT / 64)) {
        const size_t s = (size_t)evict_slot[i], row = hot_row[s];
        for (int d = lane; d < D; d += 64) { W_cold[row * D + d] = W_hot[s * D + d]; A_cold[row * D + d] = A_hot[s * D + d]; }
        if (lane == 0) slot_of[row] = -1;
    }
}

// ... and the rows entering it take the freed slots first, then unused ones.
template <typename WT>
__global__ void __launch_bounds__(NT)
pk_hh_insert_kernel(const WT* __restrict__ W_cold, const float* __restrict__ A_cold, WT* W_hot, float* A_hot,
                    uint32_t* hot_row, int32_t* slot_of, const int32_t* __restrict__ evict_slot,
                    const uint32_t* __restrict__ ins_row, const uint32_t* __restrict__ counts, int64_t n_hot_old,
                    int64_t cap, int D)
{
    const int n_evict = (int)counts[0], n_ins = (int)counts[1], lane = threadIdx.x & 63;
    for (int i = blockIdx.x * (NT / 64) + (threadIdx.x >> 6); i < n_ins; i += gridDim.x * (NT / 64)) {
        const size_t row = ins_row[i];
        const int64_t s = i < n_evict ? (int64_t)evict_slot[i] : n_hot_old + (i - n_evict);
        if (s >= cap) continue;
        for (int d = lane; d < D; d += 64) { W_hot[s * D + d] = W_cold[row * D + d]; A_hot[s * D + d] = A_cold[row * D + d]; }
        if (lane == 0) { slot_of[row] = (int32_t)s; hot_row[s] = (uint32_t)row; }
    }
}

// Histogram of the FCounter values of the rows that were ever queried.  Most of them share a
// few small counts, and contended global atomics are served one at a time, so small counts
// are tallied in LDS first.
constexpr int kHhLdsBins = 2048;

__global__ void __launch_bounds__(NT)
pk_hh_hist_kernel(const uint32_t* __restrict__ fcounter, int64_t rows, uint32_t* hist)
{
    __shared__ uint32_t s_hist[kHhLdsBins];
    for (int i = threadIdx.x; i < kHhLdsBins; i += NT) s_hist[i] = 0;
    __syncthreads();
    for (int64_t r = (int64_t)blockIdx.x * NT + threadIdx.x; r < rows; r += (int64_t)gridDim.x * NT) {
        const uint32_t c = fcounter[r];
        if (c == 0) continue;
        if (c < (uint32_t)kHhLdsBins) atomicAdd(&s_hist[c], 1u);
        else atomicAdd(&hist[min(c, (uint32_t)(kHhBins - 1))], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kHhLdsBins; i += NT)
        if (s_hist[i]) atomicAdd(&hist[i], s_hist[i]);
}

// class of a row for the selection: 2 = count above the threshold, 1 = equal to it, 0 = below
__device__ __forceinline__ int hh_class(uint32_t c, uint32_t thr)
{
    const uint32_t b = min(c, (uint32_t)(kHhBins - 1));
    return b > thr ? 2 : (b == thr ? 1 : 0);
}

// per tile of rows: how many rows have a count equal to the threshold
__global__ void __launch_bounds__(NT)
pk_hh_tilecount_kernel(const uint32_t* __restrict__ fcounter, int64_t rows, uint32_t thr, int32_t* __restrict__ tile_eq)
{
    const int64_t r0 = (int64_t)blockIdx.x * kHhTile;
    int eq = 0;
    for (int i = threadIdx.x; i < kHhTile; i += NT) {
        const int64_t r = r0 + i;
        if (r < rows) eq += hh_class(fcounter[r], thr) == 1;
    }
    int te;
    (void)block_excl_scan<NT>(eq, &te);
    if (threadIdx.x == 0) tile_eq[blockIdx.x] = te;
}

// exclusive scan of the per-tile array, in place (one block)
__global__ void __launch_bounds__(1024)
pk_hh_scan_kernel(int32_t* tile_eq, int n_tiles)
{
    int ce = 0;
    for (int base = 0; base < n_tiles; base += 1024) {
        const int i = base + threadIdx.x;
        const int e = i < n_tiles ? tile_eq[i] : 0;
        int te;
        const int xe = block_excl_scan<1024>(e, &te);
        if (i < n_tiles) tile_eq[i] = ce + xe;
        ce += te;
    }
}

// The new content of the Hot-storage: every row above the threshold and the first need_eq
// rows equal to it (ascending row order decides among those).  Compared with where the rows
// live now this gives the slots to free and the rows to bring in; rows that stay are not moved.
__global__ void __launch_bounds__(NT)
pk_hh_diff_kernel(const uint32_t* __restrict__ fcounter, int64_t rows, uint32_t thr, int need_eq,
                  const int32_t* __restrict__ eq_before, const int32_t* __restrict__ slot_of,
                  int32_t* __restrict__ evict_slot, uint32_t* __restrict__ ins_row, uint32_t* counts, int64_t cap)
{
    constexpr int PER = kHhTile / NT;                 // consecutive rows per thread
    const int64_t r0 = (int64_t)blockIdx.x * kHhTile + (int64_t)threadIdx.x * PER;
    int cl[PER];
    int eq = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        cl[j] = r0 + j < rows ? hh_class(fcounter[r0 + j], thr) : 0;
        eq += cl[j] == 1;
    }
    int te;
    int xe = block_excl_scan<NT>(eq, &te);
    const int eb = eq_before[blockIdx.x];
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const bool take = cl[j] == 2 || (cl[j] == 1 && eb + xe < need_eq);
        xe += cl[j] == 1;
        const bool live = r0 + j < rows;
        const int s = live ? slot_of[r0 + j] : -1;
        // one atomic per wavefront and list: contended atomics are served one at a time
        const bool ev = live && s >= 0 && !take, in = live && s < 0 && take;
        const unsigned long long m_ev = __ballot(ev), m_in = __ballot(in);
        const int lane = threadIdx.x & 63;
        const unsigned long long below = (1ull << lane) - 1ull;
        if (m_ev) {
            uint32_t base = 0;
            if (lane == __ffsll((unsigned long long)m_ev) - 1) base = atomicAdd(&counts[0], (uint32_t)__popcll(m_ev));
            base = __shfl(base, __ffsll((unsigned long long)m_ev) - 1, 64);
            const uint32_t i = base + (uint32_t)__popcll(m_ev & below);
            if (ev && (int64_t)i < cap) evict_slot[i] = s;
        }
        if (m_in) {
            uint32_t base = 0;
            if (lane == __ffsll((unsigned long long)m_in) - 1) base = atomicAdd(&counts[1], (uint32_t)__popcll(m_in));
            base = __shfl(base, __ffsll((unsigned long long)m_in) - 1, 64);
            const uint32_t i = base + (uint32_t)__popcll(m_in & below);
            if (in && (int64_t)i < cap) ins_row[i] = (uint32_t)(r0 + j);
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct DeviceState {
    int device = -1;
    void* blob = nullptr;
    FieldMeta* fmeta = nullptr;
    PackMeta* pmeta = nullptr;
    int32_t* slot_field = nullptr;
    MarkItem* mark_items = nullptr;
    int32_t* mark_fields = nullptr;
    TableMeta* sort_tables = nullptr;
    int32_t* table_fields = nullptr;
    std::mutex mu;
    // Side streams: packs (and the pooling of a pack vs the dedup chain) are independent
    // pieces of memory-bound work; running them side by side hides launch gaps and
    // latency tails (the interleaving of packed operations of Sec. III-C, on one GPU).
    static constexpr int kSide = 8;
    hipStream_t side[kSide] = {};
    hipEvent_t ev_fork = nullptr;
    hipEvent_t ev_join[kSide] = {};
    bool overlap = true;
    bool fuse = true;
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
    const size_t F = plan->fields.size(), P = plan->packs.size();
    std::vector<FieldMeta> fm(F);
    for (size_t f = 0; f < F; ++f) {
        const int32_t t = plan->fields[f].table;
        fm[f].base_row = (uint32_t)plan->table_base[t];
        fm[f].rows = (uint32_t)plan->tables[t].rows;
        fm[f].col = (int32_t)plan->field_col[f];
        fm[f].pack = plan->field_pack[f];
        fm[f].slot = plan->field_slot[f];
        fm[f].pool = plan->fields[f].pool;
    }
    std::vector<PackMeta> pmv(P);
    for (size_t p = 0; p < P; ++p) {
        const Pack& k = plan->packs[p];
        pmv[p].dim = k.dim; pmv[p].dtype = k.dtype; pmv[p].n_fields = (int32_t)k.fields.size();
        pmv[p].first_slot = k.first_slot; pmv[p].has_mean = k.has_mean ? 1 : 0;
        pmv[p].first_tile = k.first_tile; pmv[p].n_tiles = k.n_tiles; pmv[p].first_stable = k.first_stable;
    }
    auto pad = [](size_t b) { return (b + 255) / 256 * 256; };
    const size_t b_f = pad(F * sizeof(FieldMeta)), b_p = pad(P * sizeof(PackMeta)), b_s = pad(F * 4);
    const size_t b_i = pad(plan->mark_items.size() * sizeof(MarkItem)), b_m = pad(plan->mark_fields.size() * 4);
    const size_t b_t = pad(plan->sort_tables.size() * sizeof(TableMeta)), b_tf = pad(plan->table_fields.size() * 4);
    e = hipMalloc(&ds->blob, b_f + b_p + b_s + b_i + b_m + b_t + b_tf + 256);
    if (e != hipSuccess) { delete ds; return fail(PK_EHIP, hip_msg("hipMalloc(plan metadata)", e)); }
    {
        char* at = static_cast<char*>(ds->blob);
        ds->fmeta = reinterpret_cast<FieldMeta*>(at); at += b_f;
        ds->pmeta = reinterpret_cast<PackMeta*>(at); at += b_p;
        ds->slot_field = reinterpret_cast<int32_t*>(at); at += b_s;
        ds->mark_items = reinterpret_cast<MarkItem*>(at); at += b_i;
        ds->mark_fields = reinterpret_cast<int32_t*>(at); at += b_m;
        ds->sort_tables = reinterpret_cast<TableMeta*>(at); at += b_t;
        ds->table_fields = reinterpret_cast<int32_t*>(at);
    }
    auto up = [&](void* dst, const void* src, size_t bytes) {
        if (e == hipSuccess && bytes) e = hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice);
    };
    up(ds->fmeta, fm.data(), F * sizeof(FieldMeta));
    up(ds->pmeta, pmv.data(), P * sizeof(PackMeta));
    up(ds->slot_field, plan->slot_field.data(), F * 4);
    up(ds->mark_items, plan->mark_items.data(), plan->mark_items.size() * sizeof(MarkItem));
    up(ds->mark_fields, plan->mark_fields.data(), plan->mark_fields.size() * 4);
    up(ds->sort_tables, plan->sort_tables.data(), plan->sort_tables.size() * sizeof(TableMeta));
    up(ds->table_fields, plan->table_fields.data(), plan->table_fields.size() * 4);
    if (e != hipSuccess) { (void)hipFree(ds->blob); delete ds; return fail(PK_EHIP, hip_msg("hipMemcpy(plan metadata)", e)); }
    for (int i = 0; i < DeviceState::kSide && e == hipSuccess; ++i) {
        e = hipStreamCreateWithFlags(&ds->side[i], hipStreamNonBlocking);     // default priority
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ds->ev_join[i], hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ds->ev_fork, hipEventDisableTiming);
    if (e != hipSuccess) { (void)hipFree(ds->blob); delete ds; return fail(PK_EHIP, hip_msg("side stream setup", e)); }
    if (getenv("PK_TUNE_NO_OVERLAP")) ds->overlap = false;       // tuning aids
    if (getenv("PK_TUNE_NO_FUSE")) ds->fuse = false;
    plan->device_state = ds;
    *out = ds;
    return PK_OK;
}

// fork: side streams wait for what the caller's stream has enqueued so far
pk_status fork_streams(DeviceState* ds, hipStream_t main, int n)
{
    hipError_t e = hipEventRecord(ds->ev_fork, main);
    for (int i = 0; i < n && e == hipSuccess; ++i) e = hipStreamWaitEvent(ds->side[i], ds->ev_fork, 0);
    return e == hipSuccess ? PK_OK : fail(PK_EHIP, hip_msg("stream fork", e));
}

// join: the caller's stream waits for everything enqueued on the side streams
pk_status join_streams(DeviceState* ds, hipStream_t main, int n)
{
    hipError_t e = hipSuccess;
    for (int i = 0; i < n && e == hipSuccess; ++i) {
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
    const void* W; const uint32_t* keys; const int32_t* po; const PackState* st; const FieldMeta* fmeta;
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
                  static_cast<const WT*>(a.W), a.keys, a.po, a.st, a.fmeta, a.slot_field, a.B, a.D, a.n_bags, a.out,
                  a.out_stride, a.hv);
    else
        PK_LAUNCH("pk_pool", (pk_pool_kernel<WT, VEC, LPR, NCH, false>), dim3(grid), dim3(NT), 0,
                  static_cast<const WT*>(a.W), a.keys, a.po, a.st, a.fmeta, a.slot_field, a.B, a.D, a.n_bags, a.out,
                  a.out_stride, a.hv);
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

// shape of the pooling code for a pack, as numbered in pk_sort_pool_kernel, and its lanes per row
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

extern "C" {

// The forward pass, or one of its two stages (Sec. III-C, D-Interleaving runs them on different
// streams for different micro-batches): kDedup = H1 + H2, kPool = H3-H5 from a workspace that a
// dedup stage filled.  hot: per pack, where the rows of a Hot-storage live (HybridHash), or NULL.
enum { kDedup = 1, kPool = 2 };

static pk_status forward_impl(const pk_plan* plan, int stages, const char* who, void* const* W, const HotView* hot,
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
    DeviceState* ds = nullptr;
    rc = ensure_device_state(plan, &ds);
    if (rc != PK_OK) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    Ws ws{static_cast<char*>(workspace), make_layout(plan, B, nnz)};
    const Layout& L = ws.L;

    PackState* st = ws.at<PackState>(L.state);
    int32_t* fb = ws.at<int32_t>(L.fb);
    int32_t* delta = ws.at<int32_t>(L.delta);
    int32_t* packed_offsets = ws.at<int32_t>(L.packed_offsets);
    uint32_t* keys = ws.at<uint32_t>(L.keys);
    int32_t* inverse = ws.at<int32_t>(L.inverse);
    uint32_t* bagref = ws.at<uint32_t>(L.bagref);
    uint32_t* baglen = plan->any_mean ? ws.at<uint32_t>(L.baglen) : nullptr;
    uint32_t* seg_ent = ws.at<uint32_t>(L.seg_ent);
    int4* tile_hdr = ws.at<int4>(L.tile_hdr);
    uint32_t* unique = ws.at<uint32_t>(L.unique);
    int32_t* seg = ws.at<int32_t>(L.seg);
    double* ghot = ws.at<double>(L.ghot);
    uint32_t* bitmap = ws.at<uint32_t>(L.bitmap);
    uint64_t* tile_desc = ws.at<uint64_t>(L.tile_desc);
    uint64_t* sort_desc = ws.at<uint64_t>(L.sort_desc);
    int32_t* rank = ws.at<int32_t>(L.rank);
    const int64_t n_tiles = L.n_tiles_total;
    const int64_t n_clear4 = (int64_t)(L.clear_bytes / 16);
    const int T = (int)plan->sort_tables.size();

    // keys: BT bags per block iteration; fewer when bags are long, so that blocks stay comparable
    const int64_t n_bags = (int64_t)F * B;
    const bool long_bags = nnz / n_bags >= 16;
    const int bt = long_bags ? 32 : 256;
    const dim3 key_grid(blocks_for(n_bags, bt, 256 * 8));
    const MarkArgs ma{ds->mark_items, ds->mark_fields, ds->pmeta, st, fb, delta, keys, bitmap, nnz};
    const int n_mark = (int)plan->mark_items.size();
    // small batches: the keys and the bitmap in one launch (its LDS holds either role's arrays)
    const bool fuse_keys_mark = do_dedup && ds->fuse && nnz < (1 << 20) &&
                                keys_bag_words<kFusedKeysBags>() + keys_field_words(F) <= (size_t)kMarkWords;
    if (!do_dedup) {
    } else if (fuse_keys_mark) {
        if (long_bags)
            PK_LAUNCH("pk_keys_mark", pk_keys_mark_kernel<kFusedKeysBags / 8>,
                      dim3((unsigned)n_mark + blocks_for(n_bags, kFusedKeysBags / 8, 512)), dim3(kMarkThreads), 0, ids,
                      offsets, B, F, P, nnz, ds->fmeta, ds->pmeta, ds->slot_field, st, fb, delta, keys, bagref, baglen,
                      packed_offsets, plan->out_dim, reinterpret_cast<uint4*>(tile_desc), n_clear4, ma, n_mark);
        else
            PK_LAUNCH("pk_keys_mark", pk_keys_mark_kernel<kFusedKeysBags>,
                      dim3((unsigned)n_mark + blocks_for(n_bags, kFusedKeysBags, 512)), dim3(kMarkThreads), 0, ids,
                      offsets, B, F, P, nnz, ds->fmeta, ds->pmeta, ds->slot_field, st, fb, delta, keys, bagref, baglen,
                      packed_offsets, plan->out_dim, reinterpret_cast<uint4*>(tile_desc), n_clear4, ma, n_mark);
    } else if (long_bags) {
        PK_LAUNCH("pk_keys", pk_keys_kernel<32>, key_grid, dim3(NT), keys_field_words(F) * 4, ids, offsets, B, F, P, nnz,
                  ds->fmeta, ds->pmeta, ds->slot_field, st, fb, delta, keys, bagref, baglen, packed_offsets,
                  plan->out_dim, reinterpret_cast<uint4*>(tile_desc), n_clear4);
    } else {
        PK_LAUNCH("pk_keys", pk_keys_kernel<256>, key_grid, dim3(NT), keys_field_words(F) * 4, ids, offsets, B, F, P, nnz,
                  ds->fmeta, ds->pmeta, ds->slot_field, st, fb, delta, keys, bagref, baglen, packed_offsets,
                  plan->out_dim, reinterpret_cast<uint4*>(tile_desc), n_clear4);
    }

    // Pooling needs the keys only.  Large batches: it runs on side streams beside the rest of
    // the dedup chain.  Small ones: it shares the launch of the sort kernel (a cross-stream
    // dependency would cost more than a small pooling kernel takes).
    // Interleaving groups (Sec. III-C, K-Interleaving): pack p belongs to group p mod G; a
    // group's packed operations follow one another on the group's stream, the groups run side
    // by side.  G = 0 lets the size decide (up to 4 groups for large batches, none for small).
    const int G = plan->opts.interleave_groups;
    const bool overlap = ds->overlap && !ds->prof_on &&
                         (G >= 2 || (G == 0 && (P > 1 || nnz >= (1 << 20)) && nnz >= (1 << 18)));
    const int n_side = overlap && do_pool ? std::min<int>(P, G >= 2 ? G : 4) : 0;
    const bool fuse_pool = do_dedup && do_pool && !hot && !n_side && P <= kFusedPacks && T > 0 && nnz < (1 << 20) &&
                           ds->fuse;
    auto pool_aligned = [&](int p) {
        return cols_aligned(plan, p) && aligned16(out) && out_row_stride % 4 == 0 && aligned16(W[p]);
    };
    if (n_side) { rc = fork_streams(ds, stream, n_side); if (rc != PK_OK) return rc; }
    for (int p = 0; p < P && do_pool && !fuse_pool; ++p) {
        const Pack& k = plan->packs[p];
        if (k.fields.empty()) continue;
        PoolArgs a{W[p], keys, packed_offsets + po_off(plan, p, B), st + p, ds->fmeta, ds->slot_field + k.first_slot,
                   B, k.dim, (int64_t)k.fields.size() * B, out, out_row_stride, 256 * 32, pool_aligned(p),
                   hot ? hot[p] : HotView{nullptr, nullptr, nullptr}};
        hipStream_t ps = n_side ? ds->side[p % n_side] : stream;
        rc = k.dtype == PK_F32 ? dispatch_pool<float, 4>(ds, ps, k.dim, a)
                               : dispatch_pool<uint16_t, 8>(ds, ps, k.dim, a);
        if (rc != PK_OK) return rc;
    }

    if (!do_dedup) {
        if (n_side) { rc = join_streams(ds, stream, n_side); if (rc != PK_OK) return rc; }
        return PK_OK;
    }
    if (!fuse_keys_mark) PK_LAUNCH("pk_mark", pk_mark_kernel, dim3((unsigned)n_mark), dim3(kMarkThreads), 0, ma);
    // a grid that the chip holds at once (the scan's waits need that); with more tiles than that,
    // runs of four tiles per block iteration
    constexpr int kTilesGrid = 1024, kTileRun = 4;
    if (n_tiles <= kTilesGrid) {
        PK_LAUNCH("pk_tiles", pk_tiles_kernel<1>, dim3(blocks_for(n_tiles, 1, kTilesGrid)), dim3(NT), 0,
                  reinterpret_cast<const uint4*>(bitmap), tile_desc, (int)n_tiles, ds->pmeta, st, P, rank, unique);
    } else {
        int64_t n_runs = 0;
        for (const Pack& k : plan->packs) n_runs += (k.n_tiles + kTileRun - 1) / kTileRun;
        PK_LAUNCH("pk_tiles", pk_tiles_kernel<kTileRun>, dim3(blocks_for(n_runs, 1, kTilesGrid)), dim3(NT), 0,
                  reinterpret_cast<const uint4*>(bitmap), tile_desc, (int)n_runs, ds->pmeta, st, P, rank, unique);
    }
    const int kt = nnz < (1 << 20) ? 256 : 1024;      // occurrences per tile of the inverse kernel
    const unsigned xq = (blocks_for(nnz, kt, 256 * 16) + 7u) & ~7u;
    if (kt == 256)
        PK_LAUNCH("pk_inverse", pk_inverse_kernel<256>, dim3(xq, P), dim3(NT), 0, ds->pmeta, st, keys,
                  reinterpret_cast<const uint4*>(bitmap), rank, inverse);
    else
        PK_LAUNCH("pk_inverse", pk_inverse_kernel<1024>, dim3(xq, P), dim3(NT), 0, ds->pmeta, st, keys,
                  reinterpret_cast<const uint4*>(bitmap), rank, inverse);
    if (T > 0) {
        // at most nnz / kSortCap + T work items exist; the grid is kept small enough for every
        // block to be resident (two per CU when their LDS fits)
        const size_t sort_lds = (size_t)(4 * T + 1) * 4;
        const int64_t resident = 2 * (kSortCap * 4 + 256 + sort_lds) <= 160 * 1024 ? 512 : 256;
        const unsigned sgrid = (unsigned)std::max<int64_t>(1, std::min<int64_t>(nnz / kSortCap + T, resident));
        const SortArgs sa{ds->sort_tables, ds->table_fields, T, ds->pmeta, st, P, fb, delta,
                          reinterpret_cast<const uint4*>(bitmap), rank, inverse, bagref, baglen, seg, seg_ent,
                          plan->any_mean ? 2 : 1, tile_hdr, L.pos_tile, sort_desc, ghot, L.dmax, nnz};
        if (fuse_pool) {
            PoolJob pj{};
            int nb = 0, np = 0;
            for (int p = 0; p < P; ++p) {
                const Pack& k = plan->packs[p];
                if (k.fields.empty()) continue;
                int lpr = 1;
                PoolPack& q = pj.pack[np++];
                q.W = W[p]; q.po = packed_offsets + po_off(plan, p, B); q.slot_field = ds->slot_field + k.first_slot;
                q.n_bags = (int64_t)k.fields.size() * B; q.D = k.dim;
                q.variant = pool_variant(k.dtype, k.dim, pool_aligned(p), &lpr);
                q.block_begin = nb;
                // pj.st is indexed by pack: remember which pack this entry is
                q.pad = p;
                nb += (int)blocks_for(q.n_bags, kSortThreads / lpr, 2048);
            }
            pj.n_packs = np; pj.B = B; pj.n_blocks = nb; pj.keys = keys; pj.st = st; pj.fmeta = ds->fmeta;
            pj.out = out; pj.out_stride = out_row_stride;
            PK_LAUNCH("pk_sort_pool", pk_sort_pool_kernel, dim3(sgrid + (unsigned)nb), dim3(kSortThreads), sort_lds, sa,
                      pj, (int)sgrid);
        } else {
            PK_LAUNCH("pk_sort", pk_sort_kernel, dim3(sgrid), dim3(kSortThreads), sort_lds, sa);
        }
    }
    if (n_side) { rc = join_streams(ds, stream, n_side); if (rc != PK_OK) return rc; }
    return PK_OK;
}

pk_status pk_forward(const pk_plan* plan, void* const* W, const int64_t* ids, const int32_t* offsets, int32_t B,
                     int64_t nnz, float* out, int64_t out_row_stride, void* workspace, size_t ws_bytes,
                     void* hip_stream)
{
    return forward_impl(plan, kDedup | kPool, "pk_forward", W, nullptr, ids, offsets, B, nnz, out, out_row_stride,
                        workspace, ws_bytes, hip_stream);
}

pk_status pk_forward_dedup(const pk_plan* plan, const int64_t* ids, const int32_t* offsets, int32_t B, int64_t nnz,
                   void* workspace, size_t ws_bytes, void* hip_stream)
{
    return forward_impl(plan, kDedup, "pk_forward_dedup", nullptr, nullptr, ids, offsets, B, nnz, nullptr, 0, workspace,
                        ws_bytes, hip_stream);
}

pk_status pk_forward_pool(const pk_plan* plan, void* const* W, int32_t B, int64_t nnz, float* out, int64_t out_row_stride,
                  void* workspace, size_t ws_bytes, void* hip_stream)
{
    return forward_impl(plan, kPool, "pk_forward_pool", W, nullptr, nullptr, nullptr, B, nnz, out, out_row_stride, workspace,
                        ws_bytes, hip_stream);
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
    const int n_side = overlap ? std::min<int>(P, G >= 2 ? G : 4) : 0;
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
    return forward_impl(plan, kDedup | kPool, "pk_hh_forward", W.data(), hv.data(), ids, offsets, B, nnz, out,
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
    PackState s;
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(&s, workspace, sizeof(PackState), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(PK_EHIP, hip_msg("pk_ctx_error", e));
    *error_word = s.error;
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
