// Device code and launch logic of the packed multi-field embedding layer for
// gfx950 (wave64).  The path is gather / reduce / scatter and is bound by HBM
// bandwidth, so there is no MFMA here: the work is in keeping every access
// coalesced across the embedding dimension, in touching each distinct row once
// (the point of Unique, Sec. II-D), and in launching once per pack instead of
// once per field (D-Packing, Sec. III-B).
//
// Stages of one step (all packs of the plan share the integer stages):
//   setup     field boundaries, per-pack occurrence counts and positions, bitmap clear
//   keys      H1: key = base_row + (uint64)id mod rows, packed order, mark bitmap
//   pool      H3-H5: per pack, gather rows by key, pool per bag, write concatenated
//   tiles     H2: one-pass popcount scan of the bitmap -> rank samples, distinct keys (ascending)
//   inverse   H2: inverse[q] = rank(key[q]); occurrence counts per distinct key
//   segs      H2: one-pass exclusive scan of the counts -> segment offsets; list of hot keys
//   scatter   H2: occurrences grouped by distinct key (gradient addresses)
//   adagrad   H6+H7: per pack, per distinct key: reduce gradients, update row in place
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
// before it.  Tiles are handed out by an atomic ticket, so a tile only ever
// waits for tiles that are already running: the wait always ends.  The wait is
// bounded all the same; running out of patience sets error bit 1.
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
// setup: block 0 derives the per-field and per-pack positions; the other
// blocks clear the scan descriptors.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(1024)
pk_setup_kernel(const int32_t* __restrict__ offsets, int B, int F, int P, int64_t nnz,
                const PackMeta* __restrict__ pm, const int32_t* __restrict__ slot_field,
                PackState* st, int32_t* fb, int32_t* delta, int32_t* slot_start, int32_t* packed_offsets,
                uint4* clear4, int64_t n_clear4)
{
    if (blockIdx.x != 0) {
        const uint4 z = make_uint4(0, 0, 0, 0);
        const int64_t stride = (int64_t)(gridDim.x - 1) * blockDim.x;
        for (int64_t i = (int64_t)(blockIdx.x - 1) * blockDim.x + threadIdx.x; i < n_clear4; i += stride)
            clear4[i] = z;
        return;
    }
    __shared__ int bad;
    const int tid = threadIdx.x;
    if (tid == 0) bad = 0;
    __syncthreads();
    for (int f = tid; f <= F; f += 1024) fb[f] = offsets[(int64_t)f * B];
    __syncthreads();
    for (int f = tid; f < F; f += 1024)
        if (fb[f + 1] < fb[f]) bad = 1;
    if (tid == 0 && (fb[0] != 0 || (int64_t)fb[F] != nnz)) bad = 1;
    __syncthreads();
    const int is_bad = bad;
    int start = 0;
    for (int p = 0; p < P; ++p) {
        const int k = pm[p].n_fields, fs = pm[p].first_slot;
        int carry = 0;
        for (int base = 0; base < k; base += 1024) {
            const int j = base + tid;
            int len = 0, f = 0;
            if (j < k) {
                f = slot_field[fs + j];
                len = is_bad ? 0 : fb[f + 1] - fb[f];
            }
            int tot;
            const int ex = block_excl_scan<1024>(len, &tot);
            if (j < k) {
                slot_start[fs + p + j] = carry + ex;
                delta[f] = start + carry + ex - fb[f];
            }
            carry += tot;
        }
        if (tid == 0) {
            slot_start[fs + p + k] = carry;
            PackState s;
            s.nnz = carry; s.start = start; s.n_unique = 0; s.n_hot = 0; s.error = (p == 0) ? is_bad : 0;
            s.pad[0] = s.pad[1] = s.pad[2] = 0;
            st[p] = s;
            packed_offsets[(int64_t)fs * B + p + (int64_t)k * B] = carry;
        }
        start += carry;
    }
}

// ---------------------------------------------------------------------------
// H1: packed keys (Sec. III-B: one packed ID tensor per pack) and packed bag
// offsets.  Pure streaming: 8 bytes in, 4 bytes out per occurrence.
// ---------------------------------------------------------------------------
template <int KT>
__global__ void __launch_bounds__(NT)
pk_keys_kernel(const int64_t* __restrict__ ids, const int32_t* __restrict__ offsets, int B, int F, int64_t nnz,
               const FieldMeta* __restrict__ fmeta, const PackMeta* __restrict__ pm, const PackState* __restrict__ st,
               const int32_t* __restrict__ fb, const int32_t* __restrict__ delta,
               const int32_t* __restrict__ slot_start, uint32_t* __restrict__ keys,
               int32_t* __restrict__ packed_offsets, int use_lds)
{
    extern __shared__ int32_t s_fb[];
    if (st[0].error) return;
    if (use_lds) {
        for (int f = threadIdx.x; f <= F; f += NT) s_fb[f] = fb[f];
        __syncthreads();
    }
    const int n_tiles = (int)((nnz + KT - 1) / KT);
    for (XcdTiles it(n_tiles); it.valid(); it.next()) {
        const int64_t tile = it.tile;
        int64_t idv[KT / NT];
#pragma unroll
        for (int k = 0; k < KT / NT; ++k) {          // all loads of the tile in flight together
            const int64_t i = tile * KT + k * NT + threadIdx.x;
            idv[k] = i < nnz ? ids[i] : 0;
        }
#pragma unroll
        for (int k = 0; k < KT / NT; ++k) {
            const int64_t i = tile * KT + k * NT + threadIdx.x;
            if (i < nnz) {
                const int f = (use_lds ? upper_bound_i32(s_fb, F + 1, (int)i) : upper_bound_i32(fb, F + 1, (int)i)) - 1;
                const FieldMeta m = fmeta[f];
                const int64_t q = i + delta[f];
                if ((uint64_t)q < (uint64_t)nnz) keys[q] = m.base_row + fold_id(idv[k], m.rows);
            }
        }
    }
    const int64_t stride = (int64_t)gridDim.x * NT;
    const int64_t n_bags = (int64_t)F * B;
    for (int64_t g = (int64_t)blockIdx.x * NT + threadIdx.x; g < n_bags; g += stride) {
        const int f = (int)(g / B);
        const int b = (int)(g - (int64_t)f * B);
        const FieldMeta m = fmeta[f];
        const PackMeta k = pm[m.pack];
        packed_offsets[(int64_t)k.first_slot * B + m.pack + (int64_t)m.slot * B + b] =
            slot_start[k.first_slot + m.pack + m.slot] + offsets[g] - fb[f];
    }
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

__global__ void __launch_bounds__(kMarkThreads)
pk_mark_kernel(const MarkItem* __restrict__ items, const int32_t* __restrict__ item_fields,
               const PackMeta* __restrict__ pm, const PackState* __restrict__ st,
               const int32_t* __restrict__ fb, const int32_t* __restrict__ delta,
               const uint32_t* __restrict__ keys, uint32_t* __restrict__ bitmap, int64_t nnz)
{
    __shared__ uint32_t s_bits[kMarkWords];
    const MarkItem it = items[blockIdx.x];
    for (int w = threadIdx.x; w < kMarkWords; w += kMarkThreads) s_bits[w] = 0;
    __syncthreads();
    const uint32_t span = (uint32_t)it.n_words * 32u;
    if (!st[0].error) {
        for (int fi = it.field_begin; fi < it.field_end; ++fi) {
            const int f = item_fields[fi];
            const int64_t q0 = (int64_t)fb[f] + delta[f], q1 = (int64_t)fb[f + 1] + delta[f];
            if (q0 < 0 || q1 > nnz) continue;
            int64_t q = q0 + threadIdx.x;
            for (; q + (kMarkUnroll - 1) * kMarkThreads < q1; q += kMarkUnroll * kMarkThreads) {
                uint32_t k[kMarkUnroll];
#pragma unroll
                for (int j = 0; j < kMarkUnroll; ++j) k[j] = keys[q + j * kMarkThreads] - it.key_lo;   // loads in flight together
#pragma unroll
                for (int j = 0; j < kMarkUnroll; ++j)
                    if (k[j] < span) {
                        const uint32_t bit = 1u << (k[j] & 31);
                        if (!(s_bits[k[j] >> 5] & bit)) atomicOr(&s_bits[k[j] >> 5], bit);
                    }
            }
            for (; q < q1; q += kMarkThreads) {
                const uint32_t k0 = keys[q] - it.key_lo;
                if (k0 < span) {
                    const uint32_t bit = 1u << (k0 & 31);
                    if (!(s_bits[k0 >> 5] & bit)) atomicOr(&s_bits[k0 >> 5], bit);
                }
            }
        }
    }
    __syncthreads();
    uint4* dst = reinterpret_cast<uint4*>(bitmap + (size_t)pm[it.pack].first_tile * kTileWords + it.key_lo / 32);
    const uint4* src = reinterpret_cast<const uint4*>(s_bits);
    for (int w = threadIdx.x; w < it.n_words / 4; w += kMarkThreads) dst[w] = src[w];
}

// ---------------------------------------------------------------------------
// H2 (Unique, Sec. II-D) via a bitmap over the pack's rows: the ascending
// distinct keys are the set bits in order, and the index of a key among them is
// the number of set bits before it.  One pass: popcount per 256-bit block,
// prefix over all blocks of the pack, rank samples, distinct keys written out.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(NT)
pk_tiles_kernel(const uint4* __restrict__ bitmap4, uint64_t* tile_desc, int n_tiles_total,
                const PackMeta* __restrict__ pm, PackState* st, int P,
                int32_t* __restrict__ rank, uint32_t* __restrict__ unique, int32_t* __restrict__ cnt)
{
    __shared__ uint32_t s_pre;
    // Block b takes tiles b, b+G, b+2G, ...: a tile only waits for lower tiles, which
    // belong to earlier rounds or to lower blocks of this round; the launch keeps G
    // small enough for all blocks to be resident, so the waits end.
    int p = 0;
    for (int tile = blockIdx.x; tile < n_tiles_total; tile += gridDim.x) {
        while (p + 1 < P && tile >= pm[p + 1].first_tile) ++p;
        const int first = pm[p].first_tile;
        const size_t t = (size_t)tile * NT + threadIdx.x;
        const uint4 a = bitmap4[2 * t], b = bitmap4[2 * t + 1];
        const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        int c = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) c += __popc(w[i]);
        int tot;
        const int ex = block_excl_scan<NT>(c, &tot);      // its barriers also fence s_pre between rounds
        if (threadIdx.x < 64) {
            if (tile == first) {
                if (threadIdx.x == 0) { publish_desc(tile_desc + tile, make_desc(kDescPfx, (uint32_t)tot, 0)); s_pre = 0; }
            } else {
                if (threadIdx.x == 0) publish_desc(tile_desc + tile, make_desc(kDescAgg, (uint32_t)tot, 0));
                uint32_t pa, pb;
                lookback(tile_desc, first, tile, &pa, &pb, &st[0].error);
                if (threadIdx.x == 0) {
                    publish_desc(tile_desc + tile, make_desc(kDescPfx, pa + (uint32_t)tot, 0));
                    s_pre = pa;
                }
            }
        }
        __syncthreads();
        int pre = (int)s_pre + ex;
        rank[t] = pre;
        if (tile == first + pm[p].n_tiles - 1 && threadIdx.x == NT - 1) st[p].n_unique = pre + c;
        if (c != 0) {
            const int start = st[p].start;
            uint32_t* uq = unique + start;
            const uint32_t key0 = ((uint32_t)(tile - first) * NT + threadIdx.x) * 256u;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                uint32_t x = w[i];
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

// Occurrences per distinct key, and for each occurrence its slot inside its
// key's segment -- again without global atomics.  A table's distinct keys are a
// contiguous range of ranks; a block takes one table and kCountCap of its ranks,
// counts them in LDS over the occurrences of the fields that read the table, and
// stores the counts with plain writes.  (Work items exist for every chunk the
// table's row count allows; those beyond the batch's distinct keys exit at once.)
__global__ void __launch_bounds__(kMarkThreads)
pk_count_kernel(const int32_t* __restrict__ item_table, const int32_t* __restrict__ item_chunk,
                const TableMeta* __restrict__ tmeta, const int32_t* __restrict__ table_fields,
                const PackMeta* __restrict__ pm, const PackState* __restrict__ st,
                const int32_t* __restrict__ fb, const int32_t* __restrict__ delta,
                const uint4* __restrict__ bitmap4, const int32_t* __restrict__ rank,
                const int32_t* __restrict__ inverse, int32_t* __restrict__ occ_slot, int32_t* __restrict__ cnt,
                int64_t nnz)
{
    __shared__ int32_t s_cnt[kCountCap];
    if (st[0].error) return;
    const TableMeta tm = tmeta[item_table[blockIdx.x]];
    const PackMeta k = pm[tm.pack];
    const PackState ps = st[tm.pack];
    const size_t rb = (size_t)k.first_tile * NT;
    const uint4* bm = bitmap4 + 2 * rb;
    const int32_t* rk = rank + rb;
    const uint64_t key_end = (uint64_t)k.n_tiles * (uint64_t)(kTileWords * 32);    // keys the bitmap covers
    const int r_lo = rank_of_key(bm, rk, tm.key_lo, key_end, ps.n_unique);
    const int r_hi = rank_of_key(bm, rk, (uint64_t)tm.key_lo + tm.rows, key_end, ps.n_unique);
    const int c0 = r_lo + item_chunk[blockIdx.x] * kCountCap;
    if (c0 >= r_hi) return;
    const uint32_t width = (uint32_t)min(kCountCap, r_hi - c0);
    for (int i = threadIdx.x; i < (int)width; i += kMarkThreads) s_cnt[i] = 0;
    __syncthreads();
    for (int fi = tm.field_begin; fi < tm.field_end; ++fi) {
        const int f = table_fields[fi];
        const int64_t q0 = (int64_t)fb[f] + delta[f], q1 = (int64_t)fb[f + 1] + delta[f];
        if (q0 < 0 || q1 > nnz) continue;
        int64_t q = q0 + threadIdx.x;
        for (; q + (kMarkUnroll - 1) * kMarkThreads < q1; q += kMarkUnroll * kMarkThreads) {
            uint32_t r[kMarkUnroll];
#pragma unroll
            for (int j = 0; j < kMarkUnroll; ++j) r[j] = (uint32_t)(inverse[q + j * kMarkThreads] - c0);
#pragma unroll
            for (int j = 0; j < kMarkUnroll; ++j)
                if (r[j] < width) occ_slot[q + j * kMarkThreads] = atomicAdd(&s_cnt[r[j]], 1);
        }
        for (; q < q1; q += kMarkThreads) {
            const uint32_t r0 = (uint32_t)(inverse[q] - c0);
            if (r0 < width) occ_slot[q] = atomicAdd(&s_cnt[r0], 1);
        }
    }
    __syncthreads();
    int32_t* cn = cnt + ps.start + tm.pack;
    for (int i = threadIdx.x; i < (int)width; i += kMarkThreads) cn[c0 + i] = s_cnt[i];
}

// Exclusive scan of the occurrence counts of a pack's distinct keys, in place
// (counts -> segment offsets), in one pass.  Keys with more than kWarmMax
// occurrences are listed (ascending) and get a zeroed row of partial sums.  For
// the backward pass, tile_first[t] = the key whose segment holds position t*tp.
__global__ void __launch_bounds__(NT)
pk_segs_kernel(const PackMeta* __restrict__ pm, PackState* st, int32_t* cnt, uint64_t* seg_desc,
               int32_t* __restrict__ hot, int32_t* __restrict__ hot_of, double* __restrict__ ghot, int dmax,
               int32_t* __restrict__ tile_first, int tp)
{
    __shared__ uint32_t s_pa, s_pb;
    __shared__ unsigned long long s_w[NT / 64];
    const int p = blockIdx.y;
    const int U = st[p].n_unique, start = st[p].start, D = pm[p].dim;
    int32_t* cn = cnt + start + p;
    const size_t hbase = (size_t)(start / (kWarmMax + 1) + p);
    int32_t* hl = hot + hbase;
    double* gh = ghot + hbase * dmax;
    int32_t* tf = tile_first + start / tp + p;
    uint64_t* desc = seg_desc + start / kSegTile + p;
    const int n_tiles = (U + kSegTile - 1) / kSegTile;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        cn[U] = st[p].nnz;
        if (n_tiles == 0) st[p].n_hot = 0;
    }
    // Block b takes tiles b, b+G, ...; all G blocks are resident (G is small), so the
    // wait for lower tiles ends.
    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int base = tile * kSegTile;
        unsigned long long mine = 0;                     // low 32: occurrences, high 32: hot keys
#pragma unroll
        for (int k = 0; k < kSegTile / NT; ++k) {
            const int u = base + k * NT + threadIdx.x;
            const int v = u < U ? cn[u] : 0;
            mine += (unsigned long long)(uint32_t)v + ((unsigned long long)(v > kWarmMax) << 32);
        }
        unsigned long long x = mine;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
        __syncthreads();                                 // s_w, s_pa, s_pb of the previous round are consumed
        if (lane == 0) s_w[wv] = x;
        __syncthreads();
        unsigned long long tot = 0;
#pragma unroll
        for (int i = 0; i < NT / 64; ++i) tot += s_w[i];
        const uint32_t tot_a = (uint32_t)tot, tot_b = (uint32_t)(tot >> 32);
        if (threadIdx.x < 64) {
            if (tile == 0) {
                if (threadIdx.x == 0) { publish_desc(desc, make_desc(kDescPfx, tot_a, tot_b)); s_pa = 0; s_pb = 0; }
            } else {
                if (threadIdx.x == 0) publish_desc(desc + tile, make_desc(kDescAgg, tot_a, tot_b));
                uint32_t pa, pb;
                lookback(desc, 0, tile, &pa, &pb, &st[0].error);
                if (threadIdx.x == 0) {
                    publish_desc(desc + tile, make_desc(kDescPfx, pa + tot_a, pb + tot_b));
                    s_pa = pa; s_pb = pb;
                }
            }
        }
        __syncthreads();
        uint32_t carry_a = s_pa, carry_b = s_pb;
        if (tile == n_tiles - 1 && threadIdx.x == 0) st[p].n_hot = (int)(carry_b + tot_b);
        for (int k = 0; k < kSegTile / NT; ++k) {
            const int u = base + k * NT + threadIdx.x;
            const int v = u < U ? cn[u] : 0;
            const int is_hot = v > kWarmMax;
            int ta, tb;
            const int ea = block_excl_scan<NT>(v, &ta);
            const int eb = block_excl_scan<NT>(is_hot, &tb);
            if (u < U) {
                const int s0 = (int)carry_a + ea;
                cn[u] = s0;
                for (int t = (s0 + tp - 1) / tp; t * tp < s0 + v; ++t) tf[t] = u;
                if (is_hot) {
                    const size_t h = carry_b + eb;
                    hl[h] = u;
                    hot_of[start + p + u] = (int)h;
                    for (int d = 0; d < D; ++d) gh[h * D + d] = 0.0;
                }
            }
            carry_a += ta;
            carry_b += tb;
        }
    }
}

// Occurrences grouped by distinct key (counting sort): each entry says where the
// occurrence's gradient lives in grad_out (sample * out_dim + the field's
// column) and, in packs with mean pooling, carries the 1/L of its bag.  A block
// takes BT consecutive bags (fewer when bags are long), whose occurrences are
// contiguous, and finds each occurrence's bag in LDS.
template <int BT>
__global__ void __launch_bounds__(NT)
pk_scatter_kernel(int B, int64_t out_dim, const FieldMeta* __restrict__ fmeta, const PackMeta* __restrict__ pm,
                  const PackState* __restrict__ st, const int32_t* __restrict__ slot_field,
                  const int32_t* __restrict__ packed_offsets,
                  const int32_t* __restrict__ inverse, const int32_t* __restrict__ occ_slot,
                  const int32_t* __restrict__ cnt, uint32_t* __restrict__ seg_ent, int ent_mult)
{
    __shared__ int32_t s_po[BT + 1];
    __shared__ uint32_t s_ent[BT];
    __shared__ float s_scl[BT];
    const int p = blockIdx.y;
    const int n = st[p].nnz, start = st[p].start;
    const PackMeta k = pm[p];
    const int32_t* po = packed_offsets + (int64_t)k.first_slot * B + p;
    const int32_t* sf = slot_field + k.first_slot;
    const int32_t* cn = cnt + start + p;
    uint32_t* ent = seg_ent + (size_t)start * ent_mult;
    const int64_t n_bags = (int64_t)k.n_fields * B;
    const int n_tiles = (int)((n_bags + BT - 1) / BT);
    for (XcdTiles it(n_tiles); it.valid(); it.next()) {
        const int64_t bag0 = (int64_t)it.tile * BT;
        const int nb = (int)min((int64_t)BT, n_bags - bag0);
        __syncthreads();
        for (int t = threadIdx.x; t <= nb; t += NT) s_po[t] = min(max(po[bag0 + t], 0), n);
        if (threadIdx.x < nb) {
            const int64_t g = bag0 + threadIdx.x;
            const int j = (int)(g / B);
            const int b = (int)(g - (int64_t)j * B);
            const FieldMeta m = fmeta[sf[j]];
            s_ent[threadIdx.x] = (uint32_t)((int64_t)b * out_dim + m.col);
            float sc = 1.0f;
            if (m.pool == PK_MEAN) {
                const int L = po[g + 1] - po[g];
                if (L > 0) sc = 1.0f / (float)L;
            }
            s_scl[threadIdx.x] = sc;
        }
        __syncthreads();
        const int q_lo = s_po[0], q_hi = s_po[nb];
        for (int q = q_lo + threadIdx.x; q < q_hi; q += NT) {
            const int t = upper_bound_i32(s_po, nb + 1, q) - 1;
            if ((unsigned)t >= (unsigned)nb) continue;
            const int pos = cn[inverse[start + q]] + occ_slot[start + q];
            if ((unsigned)pos < (unsigned)n) {
                if (k.has_mean) reinterpret_cast<uint2*>(ent)[pos] = make_uint2(s_ent[t], __float_as_uint(s_scl[t]));
                else ent[pos] = s_ent[t];
            }
        }
    }
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
// H3+H4+H5: Gather and SegmentReduction (Sec. II-D) fused (K-Packing, Sec.
// III-B: both are memory-bound), one launch per pack.  A group of LPR lanes owns
// one bag; each lane covers VEC (x NCH) columns, so a row is read with one
// coalesced access.  The concatenation of the fields of a sample is the write
// address.
// ---------------------------------------------------------------------------
template <typename WT, int VEC, int LPR, int NCH>
__global__ void __launch_bounds__(NT)
pk_pool_kernel(const WT* __restrict__ W, const uint32_t* __restrict__ keys_all, const int32_t* __restrict__ po,
               const PackState* __restrict__ st, const FieldMeta* __restrict__ fmeta,
               const int32_t* __restrict__ slot_field, int B, int D, int64_t n_bags,
               float* __restrict__ out, int64_t out_stride)
{
    constexpr int GPB = NT / LPR;
    const int li = threadIdx.x % LPR, gi = threadIdx.x / LPR;
    const int n = st->nnz;
    const uint32_t* keys = keys_all + st->start;
    for (int64_t bag = (int64_t)blockIdx.x * GPB + gi; bag < n_bags; bag += (int64_t)gridDim.x * GPB) {
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
        for (; q + 4 <= q1; q += 4) {
            const size_t r0 = (size_t)keys[q] * D, r1 = (size_t)keys[q + 1] * D;
            const size_t r2 = (size_t)keys[q + 2] * D, r3 = (size_t)keys[q + 3] * D;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int d0 = (c * LPR + li) * VEC;
                if (d0 < D) {
                    float x0[VEC], x1[VEC], x2[VEC], x3[VEC];
                    Row<WT, VEC>::load(W + r0 + d0, x0);
                    Row<WT, VEC>::load(W + r1 + d0, x1);
                    Row<WT, VEC>::load(W + r2 + d0, x2);
                    Row<WT, VEC>::load(W + r3 + d0, x3);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[c][v] += (x0[v] + x1[v]) + (x2[v] + x3[v]);
                }
            }
        }
        for (; q < q1; ++q) {
            const size_t r0 = (size_t)keys[q] * D;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int d0 = (c * LPR + li) * VEC;
                if (d0 < D) {
                    float x0[VEC];
                    Row<WT, VEC>::load(W + r0 + d0, x0);
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

// ---------------------------------------------------------------------------
// H6+H7: per distinct key, the gradients of its occurrences are reduced in
// double (mirror of the forward pooling, Sec. II-D) and the row takes one
// Adagrad step in place.  Fused so the reduced gradient never goes to memory.
//
// Work is cut by OCCURRENCES, not by keys, because the ID distribution is
// heavily skewed (Sec. II-B): a block takes a tile of consecutive positions of
// the key-sorted occurrence list and handles the keys that start there.
//   up to kColdMax occurrences: one lane group per key;
//   up to kWarmMax:             one wavefront per key, groups stride over it;
//   more:                       every tile reduces its piece of the key and adds
//                               it (double atomics) to the key's partial-sum row;
//                               pk_adagrad_hot_kernel then applies the update.
// ---------------------------------------------------------------------------
// The gradient chunks of a tile's occurrences: element offsets into grad_out and
// mean-pooling scales, decoded once per tile, in parallel, into LDS.
struct GradSrc {
    const float* grad;
    const uint32_t* s_addr;      // LDS: positions [t0, ...)
    const float* s_scl;
    int t0;
    __device__ __forceinline__ void fetch(int s, uint32_t* addr, float* scale) const
    {
        *addr = s_addr[s - t0];
        *scale = s_scl[s - t0];
    }
};

// acc += sum over positions s, s+step, ... < s_end of scale * grad chunk
template <int VEC, int LPR, int NCH>
__device__ __forceinline__ void accum_range(double (&acc)[NCH][VEC], const GradSrc& g, int D, int li,
                                            int s, int s_end, int step)
{
    for (; s + 3 * step < s_end; s += 4 * step) {
        uint32_t a[4];
        float c[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) g.fetch(s + k * step, &a[k], &c[k]);
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const int d0 = (ch * LPR + li) * VEC;
            if (d0 < D) {
                float x[4][VEC];
#pragma unroll
                for (int k = 0; k < 4; ++k) load_f32<VEC>(g.grad + a[k] + d0, x[k]);
#pragma unroll
                for (int v = 0; v < VEC; ++v)
                    acc[ch][v] += ((double)(c[0] * x[0][v]) + (double)(c[1] * x[1][v])) +
                                  ((double)(c[2] * x[2][v]) + (double)(c[3] * x[3][v]));
            }
        }
    }
    for (; s < s_end; s += step) {
        uint32_t a0;
        float c0;
        g.fetch(s, &a0, &c0);
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const int d0 = (ch * LPR + li) * VEC;
            if (d0 < D) {
                float x0[VEC];
                load_f32<VEC>(g.grad + a0 + d0, x0);
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[ch][v] += (double)(c0 * x0[v]);
            }
        }
    }
}

// the row's current weights and accumulators (issued before the gradient
// reduction so that both sets of loads are in flight together)
template <typename WT, int VEC, int LPR, int NCH>
__device__ __forceinline__ void row_load(const WT* W, const float* A, size_t row, int D, int li,
                                         float (&w)[NCH][VEC], float (&a)[NCH][VEC])
{
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int d0 = (c * LPR + li) * VEC;
        if (d0 < D) {
            Row<WT, VEC>::load(W + row * D + d0, w[c]);
            load_f32<VEC>(A + row * D + d0, a[c]);
        }
    }
}

// one Adagrad step of the row: a += g^2 ; w -= lr * g / (sqrt(a) + eps)
template <typename WT, int VEC, int LPR, int NCH>
__device__ __forceinline__ void row_step(WT* W, float* A, size_t row, int D, int li,
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
            store_f32<VEC>(A + row * D + d0, a[c]);
            Row<WT, VEC>::store(W + row * D + d0, w[c]);
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

template <typename WT, int VEC, int LPR, int NCH>
__global__ void __launch_bounds__(NT)
pk_adagrad_kernel(WT* W, float* A, const PackState* __restrict__ st, int p,
                  const uint32_t* __restrict__ unique_all, const int32_t* __restrict__ cnt,
                  const int32_t* __restrict__ hot_all, double* ghot_all, int dmax,
                  const int32_t* __restrict__ hot_of_all, const int32_t* __restrict__ tile_first, int tp, int hot_chunk,
                  const uint32_t* __restrict__ seg_ent_all, int ent_mult, int has_mean,
                  const float* __restrict__ grad, int64_t gstride, int64_t out_dim, int D, float lr, float eps)
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
    __shared__ float s_scl[kPosTileMax + kWarmMax];
    const int li = threadIdx.x % LPR, gi = threadIdx.x / LPR;
    const int wv = threadIdx.x >> 6, gw = (threadIdx.x & 63) / LPR;
    const int n = st->nnz, U = st->n_unique, start = st->start;
    const int32_t* seg = cnt + start + p;
    const uint32_t* uq = unique_all + start;
    const size_t hbase = (size_t)(start / (kWarmMax + 1) + p);
    double* gh = ghot_all + hbase * dmax;
    const int32_t* tf = tile_first + start / tp + p;
    const int32_t* hot_of = hot_of_all + start + p;
    const uint32_t* ent = seg_ent_all + (size_t)start * ent_mult;
    GradSrc g{grad, s_addr, s_scl, 0};
    const int n_tiles = (n + tp - 1) / tp;
    for (XcdTiles it(n_tiles); it.valid(); it.next()) {
        const int tile = it.tile;
        const int t0 = tile * tp, t1 = min(t0 + tp, n);
        // keys whose segments overlap [t0, t1)
        const int u_lo = tf[tile];
        int u_hi = U - 1;
        if (tile + 1 < n_tiles) {
            u_hi = tf[tile + 1];
            if (seg[u_hi] >= t1) --u_hi;
        }
        const int nseg = u_hi - u_lo + 1;
        // decode window: the tile, plus the tail of its last key unless that key is a hot one
        // (hot keys are cut at the tile's end)
        int w_end = t1;
        {
            const int e0 = seg[u_hi], e1 = seg[u_hi + 1];
            if (e1 - e0 <= kWarmMax) w_end = e1;
        }
        __syncthreads();                                   // the previous tile's LDS is consumed
        for (int i = threadIdx.x; i <= nseg; i += NT) s_seg[i] = seg[u_lo + i];
        for (int i = threadIdx.x; i < nseg; i += NT) s_row[i] = uq[u_lo + i];
        for (int i = threadIdx.x; i < w_end - t0; i += NT) {
            uint32_t a;
            float c = 1.0f;
            if (has_mean) {
                const uint2 e = reinterpret_cast<const uint2*>(ent)[t0 + i];
                a = e.x;
                c = __uint_as_float(e.y);
            } else {
                a = ent[t0 + i];
            }
            if (gstride != out_dim) {                      // padded gradient rows
                const uint32_t b = a / (uint32_t)out_dim;
                a = b * (uint32_t)gstride + (a - b * (uint32_t)out_dim);
            }
            s_addr[i] = a;
            s_scl[i] = c;
        }
        if (threadIdx.x == 0) { s_nwarm = 0; s_nhot = 0; }
        g.t0 = t0;
        __syncthreads();
        // cold keys that start here are finished on the spot
        for (int k = gi; k < nseg; k += GPB) {
            const int s0 = s_seg[k], s1 = s_seg[k + 1];
            const int len = s1 - s0;
            if (len <= kColdMax) {
                if (s0 >= t0) {
                    const size_t row = s_row[k];
                    float w[NCH][VEC], a[NCH][VEC];
                    row_load<WT, VEC, LPR, NCH>(W, A, row, D, li, w, a);
                    double acc[NCH][VEC];
#pragma unroll
                    for (int c = 0; c < NCH; ++c)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) acc[c][v] = 0.0;
                    accum_range<VEC, LPR, NCH>(acc, g, D, li, s0, s1, 1);
                    row_step<WT, VEC, LPR, NCH>(W, A, row, D, li, acc, w, a, lr, eps);
                }
            } else if (len <= kWarmMax) {
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
            const size_t row = s_row[k];
            float w[NCH][VEC], a[NCH][VEC];
            if (gw == 0) row_load<WT, VEC, LPR, NCH>(W, A, row, D, li, w, a);
            double acc[NCH][VEC];
#pragma unroll
            for (int c = 0; c < NCH; ++c)
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[c][v] = 0.0;
            accum_range<VEC, LPR, NCH>(acc, g, D, li, s0 + gw, s1, GPW);
            wave_group_sum<VEC, LPR, NCH>(acc);
            if (gw == 0) row_step<WT, VEC, LPR, NCH>(W, A, row, D, li, acc, w, a, lr, eps);
        }
        // hot keys: this tile's piece is split over the block's wavefronts, reduced in LDS and
        // added once to the key's partial sums
        const int n_hot_here = s_nhot;
        for (int i = 0; i < n_hot_here; ++i) {
            const int k = s_hot[i];
            const int a0 = max(s_seg[k], t0), b0 = min(s_seg[k + 1], t1);
            const int share = (b0 - a0 + NT / 64 - 1) / (NT / 64);
            const int c0 = a0 + wv * share, c1 = min(c0 + share, b0);
            double acc[NCH][VEC];
#pragma unroll
            for (int c = 0; c < NCH; ++c)
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[c][v] = 0.0;
            accum_range<VEC, LPR, NCH>(acc, g, D, li, c0 + gw, c1, GPW);
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
                double* prow = gh + (size_t)hot_of[u_lo + k] * D;   // the key's row of partial sums
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    const int d0 = (c * LPR + li) * VEC;
                    if (d0 < D) {
#pragma unroll
                        for (int v = 0; v < VEC; ++v) {
                            double t = 0.0;
#pragma unroll
                            for (int w2 = 0; w2 < NT / 64; ++w2) t += s_red[w2][li][c][v];
                            atomicAdd(prow + d0 + v, t);
                        }
                    }
                }
            }
        }
    }
}

// hot keys: partial sums are complete, apply the update (one lane group per key)
template <typename WT, int VEC, int LPR, int NCH>
__global__ void __launch_bounds__(NT)
pk_adagrad_hot_kernel(WT* W, float* A, const PackState* __restrict__ st, int p,
                      const uint32_t* __restrict__ unique_all, const int32_t* __restrict__ hot_all,
                      const double* __restrict__ ghot_all, int dmax, int D, float lr, float eps)
{
    constexpr int GPB = NT / LPR;
    const int li = threadIdx.x % LPR, gi = threadIdx.x / LPR;
    const int start = st->start, n_hot = st->n_hot;
    const size_t hbase = (size_t)(start / (kWarmMax + 1) + p);
    const int32_t* hl = hot_all + hbase;
    const double* gh = ghot_all + hbase * dmax;
    for (int h = blockIdx.x * GPB + gi; h < n_hot; h += gridDim.x * GPB) {
        double acc[NCH][VEC];
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int d0 = (c * LPR + li) * VEC;
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[c][v] = d0 < D ? gh[(size_t)h * D + d0 + v] : 0.0;
        }
        const size_t row = unique_all[start + hl[h]];
        float w[NCH][VEC], a[NCH][VEC];
        row_load<WT, VEC, LPR, NCH>(W, A, row, D, li, w, a);
        row_step<WT, VEC, LPR, NCH>(W, A, row, D, li, acc, w, a, lr, eps);
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
    TableMeta* table_meta = nullptr;
    int32_t* table_fields = nullptr;
    int32_t* count_item_table = nullptr;
    int32_t* count_item_chunk = nullptr;
    std::mutex mu;
    // Side streams: packs (and the pooling of a pack vs the dedup chain) are independent
    // pieces of memory-bound work; running them side by side hides launch gaps and
    // latency tails (the interleaving of packed operations of Sec. III-C, on one GPU).
    static constexpr int kSide = 4;
    hipStream_t side[kSide] = {};
    hipEvent_t ev_fork = nullptr;
    hipEvent_t ev_join[kSide] = {};
    bool overlap = true;
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
        pmv[p].first_tile = k.first_tile; pmv[p].n_tiles = k.n_tiles; pmv[p].pad = 0;
    }
    const size_t b_f = (F * sizeof(FieldMeta) + 255) / 256 * 256;
    const size_t b_p = (P * sizeof(PackMeta) + 255) / 256 * 256;
    const size_t b_s = (F * 4 + 255) / 256 * 256;
    const size_t b_i = (plan->mark_items.size() * sizeof(MarkItem) + 255) / 256 * 256;
    const size_t b_m = (plan->mark_fields.size() * 4 + 255) / 256 * 256;
    const size_t b_t = (plan->table_meta.size() * sizeof(TableMeta) + 255) / 256 * 256;
    const size_t b_tf = (plan->table_fields.size() * 4 + 255) / 256 * 256;
    const size_t b_ci = (plan->count_item_table.size() * 4 + 255) / 256 * 256;
    e = hipMalloc(&ds->blob, b_f + b_p + b_s + b_i + b_m + b_t + b_tf + 2 * b_ci);
    if (e != hipSuccess) { delete ds; return fail(PK_EHIP, hip_msg("hipMalloc(plan metadata)", e)); }
    ds->fmeta = reinterpret_cast<FieldMeta*>(ds->blob);
    ds->pmeta = reinterpret_cast<PackMeta*>(static_cast<char*>(ds->blob) + b_f);
    ds->slot_field = reinterpret_cast<int32_t*>(static_cast<char*>(ds->blob) + b_f + b_p);
    ds->mark_items = reinterpret_cast<MarkItem*>(static_cast<char*>(ds->blob) + b_f + b_p + b_s);
    ds->mark_fields = reinterpret_cast<int32_t*>(static_cast<char*>(ds->blob) + b_f + b_p + b_s + b_i);
    {
        char* at = static_cast<char*>(ds->blob) + b_f + b_p + b_s + b_i + b_m;
        ds->table_meta = reinterpret_cast<TableMeta*>(at); at += b_t;
        ds->table_fields = reinterpret_cast<int32_t*>(at); at += b_tf;
        ds->count_item_table = reinterpret_cast<int32_t*>(at); at += b_ci;
        ds->count_item_chunk = reinterpret_cast<int32_t*>(at);
    }
    e = hipMemcpy(ds->fmeta, fm.data(), F * sizeof(FieldMeta), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(ds->table_meta, plan->table_meta.data(), plan->table_meta.size() * sizeof(TableMeta), hipMemcpyHostToDevice);
    if (e == hipSuccess && !plan->table_fields.empty()) e = hipMemcpy(ds->table_fields, plan->table_fields.data(), plan->table_fields.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess && !plan->count_item_table.empty()) {
        e = hipMemcpy(ds->count_item_table, plan->count_item_table.data(), plan->count_item_table.size() * 4, hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(ds->count_item_chunk, plan->count_item_chunk.data(), plan->count_item_chunk.size() * 4, hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = hipMemcpy(ds->mark_items, plan->mark_items.data(), plan->mark_items.size() * sizeof(MarkItem), hipMemcpyHostToDevice);
    if (e == hipSuccess && !plan->mark_fields.empty()) e = hipMemcpy(ds->mark_fields, plan->mark_fields.data(), plan->mark_fields.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(ds->pmeta, pmv.data(), P * sizeof(PackMeta), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(ds->slot_field, plan->slot_field.data(), F * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(ds->blob); delete ds; return fail(PK_EHIP, hip_msg("hipMemcpy(plan metadata)", e)); }
    for (int i = 0; i < DeviceState::kSide && e == hipSuccess; ++i) {
        e = hipStreamCreateWithFlags(&ds->side[i], hipStreamNonBlocking);     // default priority
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ds->ev_join[i], hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ds->ev_fork, hipEventDisableTiming);
    if (e != hipSuccess) { (void)hipFree(ds->blob); delete ds; return fail(PK_EHIP, hip_msg("side stream setup", e)); }
    if (getenv("PK_TUNE_NO_OVERLAP")) ds->overlap = false;       // tuning aid
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
    bool aligned;
};
struct AdaArgs {
    void* W; float* A; const PackState* st; int p; const uint32_t* unique; const int32_t* cnt; const int32_t* hot;
    double* ghot; int dmax;
    const int32_t* hot_of; const int32_t* tile_first; int tp; int hot_chunk; const uint32_t* seg_ent; int ent_mult;
    int has_mean; const float* grad; int64_t gstride; int64_t out_dim; int D;
    float lr; float eps; int64_t nnz_bound; bool aligned;
};

template <typename WT, int VEC, int LPR, int NCH>
pk_status launch_pool(DeviceState* ds, hipStream_t stream, const PoolArgs& a)
{
    constexpr int GPB = NT / LPR;
    const unsigned grid = blocks_for(a.n_bags, GPB, a.grid_cap);
    PK_LAUNCH("pk_pool", (pk_pool_kernel<WT, VEC, LPR, NCH>), dim3(grid), dim3(NT), 0,
              static_cast<const WT*>(a.W), a.keys, a.po, a.st, a.fmeta, a.slot_field, a.B, a.D, a.n_bags, a.out,
              a.out_stride);
    return PK_OK;
}

template <typename WT, int VEC, int LPR, int NCH>
pk_status launch_adagrad(DeviceState* ds, hipStream_t stream, const AdaArgs& a)
{
    constexpr int GPB = NT / LPR;
    const unsigned grid = (blocks_for(a.nnz_bound, a.tp, 256 * 16) + 7u) & ~7u;
    PK_LAUNCH("pk_adagrad", (pk_adagrad_kernel<WT, VEC, LPR, NCH>), dim3(grid), dim3(NT), 0,
              static_cast<WT*>(a.W), a.A, a.st, a.p, a.unique, a.cnt, a.hot, a.ghot, a.dmax, a.hot_of, a.tile_first,
              a.tp, a.hot_chunk, a.seg_ent, a.ent_mult, a.has_mean, a.grad, a.gstride, a.out_dim, a.D, a.lr, a.eps);
    const unsigned hgrid = blocks_for(a.nnz_bound / (kWarmMax + 1) + 1, GPB, 1024);
    PK_LAUNCH("pk_adagrad_hot", (pk_adagrad_hot_kernel<WT, VEC, LPR, NCH>), dim3(hgrid), dim3(NT), 0,
              static_cast<WT*>(a.W), a.A, a.st, a.p, a.unique, a.hot, a.ghot, a.dmax, a.D, a.lr, a.eps);
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

pk_status pk_forward(const pk_plan* plan, void* const* W, const int64_t* ids, const int32_t* offsets, int32_t B,
                     int64_t nnz, float* out, int64_t out_row_stride, void* workspace, size_t ws_bytes,
                     void* hip_stream)
{
    pk_status rc = check_common(plan, B, nnz, workspace, ws_bytes, "pk_forward");
    if (rc != PK_OK) return rc;
    if (!W || !offsets || !out || (!ids && nnz > 0)) return fail(PK_EINVAL, "pk_forward: NULL argument");
    const int P = (int)plan->packs.size(), F = (int)plan->fields.size();
    for (int p = 0; p < P; ++p)
        if (!W[p]) return fail(PK_EINVAL, "pk_forward: W[" + std::to_string(p) + "] is NULL");
    if (out_row_stride < plan->out_dim) return fail(PK_ESHAPE, "pk_forward: out_row_stride is smaller than out_dim");
    DeviceState* ds = nullptr;
    rc = ensure_device_state(plan, &ds);
    if (rc != PK_OK) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    Ws ws{static_cast<char*>(workspace), make_layout(plan, B, nnz)};
    const Layout& L = ws.L;

    PackState* st = ws.at<PackState>(L.state);
    int32_t* fb = ws.at<int32_t>(L.fb);
    int32_t* delta = ws.at<int32_t>(L.delta);
    int32_t* slot_start = ws.at<int32_t>(L.slot_start);
    int32_t* packed_offsets = ws.at<int32_t>(L.packed_offsets);
    uint32_t* keys = ws.at<uint32_t>(L.keys);
    int32_t* inverse = ws.at<int32_t>(L.inverse);
    int32_t* occ_slot = ws.at<int32_t>(L.occ_slot);
    uint32_t* seg_ent = ws.at<uint32_t>(L.seg_ent);
    int32_t* tile_first = ws.at<int32_t>(L.tile_first);
    uint32_t* unique = ws.at<uint32_t>(L.unique);
    int32_t* cnt = ws.at<int32_t>(L.cnt);
    int32_t* hot = ws.at<int32_t>(L.hot);
    double* ghot = ws.at<double>(L.ghot);
    uint32_t* bitmap = ws.at<uint32_t>(L.bitmap);
    uint64_t* tile_desc = ws.at<uint64_t>(L.tile_desc);
    uint64_t* seg_desc = ws.at<uint64_t>(L.seg_desc);
    int32_t* rank = ws.at<int32_t>(L.rank);
    const int64_t n_tiles = L.n_tiles_total;
    const int64_t n_clear4 = (int64_t)(L.clear_bytes / 16);

    const unsigned clear_blocks = blocks_for(n_clear4, 1024 * 4, 1024);
    PK_LAUNCH("pk_setup", pk_setup_kernel, dim3(1 + clear_blocks), dim3(1024), 0, offsets, B, F, P, nnz, ds->pmeta,
              ds->slot_field, st, fb, delta, slot_start, packed_offsets, reinterpret_cast<uint4*>(tile_desc), n_clear4);

    const int kt = nnz < (1 << 20) ? 256 : 1024;      // occurrences per tile of the keys / inverse kernels
    const int use_lds = (F + 1) * 4 <= 32 * 1024;
    const int64_t key_blocks = std::max<int64_t>((nnz + kt - 1) / kt, ((int64_t)F * B + NT * 4 - 1) / (NT * 4));
    const dim3 key_grid((blocks_for(key_blocks, 1, 256 * 32) + 7u) & ~7u);
    const size_t key_lds = use_lds ? (size_t)(F + 1) * 4 : 0;
    if (kt == 256)
        PK_LAUNCH("pk_keys", pk_keys_kernel<256>, key_grid, dim3(NT), key_lds, ids, offsets, B, F, nnz, ds->fmeta,
                  ds->pmeta, st, fb, delta, slot_start, keys, packed_offsets, use_lds);
    else
        PK_LAUNCH("pk_keys", pk_keys_kernel<1024>, key_grid, dim3(NT), key_lds, ids, offsets, B, F, nnz, ds->fmeta,
                  ds->pmeta, st, fb, delta, slot_start, keys, packed_offsets, use_lds);

    // pooling needs the keys only: it runs beside the rest of the dedup chain
    const bool overlap = ds->overlap && !ds->prof_on && (P > 1 || nnz >= (1 << 20));   // fork+join cost a few us
    const int n_side = overlap ? std::min<int>(P, DeviceState::kSide) : 0;
    if (n_side) { rc = fork_streams(ds, stream, n_side); if (rc != PK_OK) return rc; }
    for (int p = 0; p < P; ++p) {
        const Pack& k = plan->packs[p];
        PoolArgs a{W[p], keys, packed_offsets + po_off(plan, p, B), st + p, ds->fmeta, ds->slot_field + k.first_slot,
                   B, k.dim, (int64_t)k.fields.size() * B, out, out_row_stride, 256 * 32,
                   cols_aligned(plan, p) && aligned16(out) && out_row_stride % 4 == 0 && aligned16(W[p])};
        hipStream_t ps = n_side ? ds->side[p % n_side] : stream;
        rc = k.dtype == PK_F32 ? dispatch_pool<float, 4>(ds, ps, k.dim, a)
                               : dispatch_pool<uint16_t, 8>(ds, ps, k.dim, a);
        if (rc != PK_OK) return rc;
    }

    PK_LAUNCH("pk_mark", pk_mark_kernel, dim3((unsigned)plan->mark_items.size()), dim3(kMarkThreads), 0, ds->mark_items,
              ds->mark_fields, ds->pmeta, st, fb, delta, keys, bitmap, nnz);
    PK_LAUNCH("pk_tiles", pk_tiles_kernel, dim3(blocks_for(n_tiles, 1, 1024)), dim3(NT), 0,
              reinterpret_cast<const uint4*>(bitmap), tile_desc, (int)n_tiles, ds->pmeta, st, P, rank, unique, cnt);
    const unsigned xq = (blocks_for(nnz, kt, 256 * 16) + 7u) & ~7u;
    if (kt == 256)
        PK_LAUNCH("pk_inverse", pk_inverse_kernel<256>, dim3(xq, P), dim3(NT), 0, ds->pmeta, st, keys,
                  reinterpret_cast<const uint4*>(bitmap), rank, inverse);
    else
        PK_LAUNCH("pk_inverse", pk_inverse_kernel<1024>, dim3(xq, P), dim3(NT), 0, ds->pmeta, st, keys,
                  reinterpret_cast<const uint4*>(bitmap), rank, inverse);
    if (!plan->count_item_table.empty())
        PK_LAUNCH("pk_count", pk_count_kernel, dim3((unsigned)plan->count_item_table.size()), dim3(kMarkThreads), 0,
                  ds->count_item_table, ds->count_item_chunk, ds->table_meta, ds->table_fields, ds->pmeta, st, fb, delta,
                  reinterpret_cast<const uint4*>(bitmap), rank, inverse, occ_slot, cnt, nnz);
    PK_LAUNCH("pk_segs", pk_segs_kernel, dim3(blocks_for(nnz, kSegTile, std::max(1, 1024 / P)), P), dim3(NT), 0,
              ds->pmeta, st, cnt, seg_desc, hot, ws.at<int32_t>(L.hot_of), ghot, L.dmax, tile_first, L.pos_tile);
    int64_t max_bags = 0;
    for (int p = 0; p < P; ++p) max_bags = std::max<int64_t>(max_bags, (int64_t)plan->packs[p].fields.size() * B);
    if (nnz / ((int64_t)F * B) >= 16)      // long bags: fewer bags per block
        PK_LAUNCH("pk_scatter", pk_scatter_kernel<32>, dim3((blocks_for(max_bags, 32, 256 * 16) + 7u) & ~7u, P), dim3(NT),
                  0, B, plan->out_dim, ds->fmeta, ds->pmeta, st, ds->slot_field, packed_offsets, inverse, occ_slot, cnt,
                  seg_ent, plan->any_mean ? 2 : 1);
    else
        PK_LAUNCH("pk_scatter", pk_scatter_kernel<256>, dim3((blocks_for(max_bags, 256, 256 * 16) + 7u) & ~7u, P),
                  dim3(NT), 0, B, plan->out_dim, ds->fmeta, ds->pmeta, st, ds->slot_field, packed_offsets, inverse,
                  occ_slot, cnt, seg_ent, plan->any_mean ? 2 : 1);
    if (n_side) { rc = join_streams(ds, stream, n_side); if (rc != PK_OK) return rc; }
    return PK_OK;
}

pk_status pk_backward_update(const pk_plan* plan, void* const* W, float* const* A, const float* grad_out,
                             int64_t grad_row_stride, int32_t B, int64_t nnz, float lr, float eps, void* workspace,
                             size_t ws_bytes, void* hip_stream)
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
    const bool overlap = ds->overlap && !ds->prof_on && P > 1;
    const int n_side = overlap ? std::min<int>(P, DeviceState::kSide) : 0;
    if (n_side) { rc = fork_streams(ds, stream, n_side); if (rc != PK_OK) return rc; }
    for (int p = 0; p < P; ++p) {
        const Pack& k = plan->packs[p];
        hipStream_t ps = n_side ? ds->side[p % n_side] : stream;
        AdaArgs a{W[p], A[p], st + p, p, ws.at<uint32_t>(L.unique), ws.at<int32_t>(L.cnt), ws.at<int32_t>(L.hot),
                  ws.at<double>(L.ghot), L.dmax, ws.at<int32_t>(L.hot_of), ws.at<int32_t>(L.tile_first), L.pos_tile,
                  nnz < (2 << 20) ? 64 : 256, ws.at<uint32_t>(L.seg_ent), plan->any_mean ? 2 : 1,
                  k.has_mean ? 1 : 0, grad_out, grad_row_stride, plan->out_dim, k.dim, lr, eps, nnz,
                  cols_aligned(plan, p) && aligned16(grad_out) && grad_row_stride % 4 == 0 && aligned16(W[p]) &&
                      aligned16(A[p])};
        rc = k.dtype == PK_F32 ? dispatch_adagrad<float, 4>(ds, ps, k.dim, a)
                               : dispatch_adagrad<uint16_t, 8>(ds, ps, k.dim, a);
        if (rc != PK_OK) return rc;
    }
    if (n_side) { rc = join_streams(ds, stream, n_side); if (rc != PK_OK) return rc; }
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
    if (seg_offsets) *seg_offsets = reinterpret_cast<const int32_t*>(base + L.cnt) + s.start + p;
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
