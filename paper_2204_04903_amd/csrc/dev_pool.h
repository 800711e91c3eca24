// H3-H5: gather + pool + concatenate, and the kernel in which small batches share the sort's launch.
// Part of pk_device.hip: included there, in this order, inside its anonymous namespace.

// ---------------------------------------------------------------------------
// H3+H4+H5: Gather and SegmentReduction (Sec. II-D) fused (K-Packing, Sec.
// III-B: both are memory-bound), one launch per pack.  A group of LPR lanes owns
// one bag; each lane covers VEC (x NCH) columns, so a row is read with one
// coalesced access.  The concatenation of the fields of a sample is the write
// address.
// ---------------------------------------------------------------------------
// What the pooling of a pack reads its rows' keys from: the packed keys and packed bag offsets the
// dedup stage left in the workspace, or (small batches, where the pooling runs beside the dedup in
// one launch) the caller's IDs and offsets, hashed here the same way.
struct PoolSrc {
    const uint32_t* keys_all; const int32_t* po; const PackState* st;      // from the workspace
    const int64_t* ids; const int32_t* offsets; int64_t nnz;               // from the caller's inputs
    uint32_t rows;                                                         // rows of the pack's table
};

// `block` of `nblocks` blocks of `nthreads` threads; HYB: rows may live in a Hot-storage;
// DEEP: eight rows of a bag in flight instead of four (the kernel that shares the dedup's
// launch has no registers for that); IDS: keys are formed from the caller's IDs
template <typename WT, int VEC, int LPR, int NCH, bool HYB, bool DEEP, bool IDS>
__device__ __forceinline__ void pool_body(const WT* __restrict__ W, const PoolSrc& src,
                                          const FieldMeta* __restrict__ fmeta, const int32_t* __restrict__ slot_field,
                                          int B, int D, int64_t n_bags, float* __restrict__ out, int64_t out_stride,
                                          int block, int nblocks, int nthreads, const HotView hv)
{
    const int GPB = nthreads / LPR;
    const int li = threadIdx.x % LPR, gi = threadIdx.x / LPR;
    const int n = IDS ? (int)src.nnz : src.st->nnz;
    const uint32_t* __restrict__ keys = IDS ? nullptr : src.keys_all + src.st->start;
    const int64_t* __restrict__ ids = src.ids;
    const uint32_t last_row = src.rows - 1;
    for (int64_t bag = (int64_t)block * GPB + gi; bag < n_bags; bag += (int64_t)nblocks * GPB) {
        const int j = (int)(bag / B);
        const int b = (int)(bag - (int64_t)j * B);
        const int f = slot_field[j];
        const FieldMeta m = fmeta[f];
        int q0, q1;
        if (IDS) {
            const int32_t* offs = src.offsets + (int64_t)f * B;
            q0 = min(max(offs[b], 0), n);                  // whatever the offsets hold, no read leaves ids
            q1 = min(max(offs[b + 1], q0), n);
        } else {
            q0 = min(max(src.po[bag], 0), n);
            q1 = min(max(src.po[bag + 1], q0), n);
        }
        // the key of position q; a key that is no row of the pack (only possible after rejected
        // offsets, which raise the error word) is bent to the last row so that no read leaves the table
        auto key_at = [&](int q) -> uint32_t {
            if (IDS) return m.base_row + fold_id(ids[q], m.rows, m.magic);
            return min(keys[q], last_row);
        };
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
                for (int k = 0; k < 8; ++k) r[k] = row_of<const WT, HYB>(W, hv, key_at(q + k), D);
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
            const WT* r0 = row_of<const WT, HYB>(W, hv, key_at(q), D);
            const WT* r1 = row_of<const WT, HYB>(W, hv, key_at(q + 1), D);
            const WT* r2 = row_of<const WT, HYB>(W, hv, key_at(q + 2), D);
            const WT* r3 = row_of<const WT, HYB>(W, hv, key_at(q + 3), D);
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
        // What is left of the bag (up to three rows) in one round: the rows that are there are asked for
        // together, the others count as zeros.  (One row after the other is a wait per row.)
        if (q < q1) {
            const int rem = q1 - q;
            const WT* r[3];
#pragma unroll
            for (int k = 0; k < 3; ++k) r[k] = row_of<const WT, HYB>(W, hv, k < rem ? key_at(q + k) : key_at(q), D);
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int d0 = (c * LPR + li) * VEC;
                if (d0 < D) {
                    float x[3][VEC];
#pragma unroll
                    for (int k = 0; k < 3; ++k) {
#pragma unroll
                        for (int v = 0; v < VEC; ++v) x[k][v] = 0.f;
                        if (k < rem) Row<WT, VEC>::load(r[k] + d0, x[k]);
                    }
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[c][v] += (x[0][v] + x[1][v]) + x[2][v];
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
               const PackState* __restrict__ st, uint32_t rows, const FieldMeta* __restrict__ fmeta,
               const int32_t* __restrict__ slot_field, int B, int D, int64_t n_bags,
               float* __restrict__ out, int64_t out_stride, const HotView hv)
{
    const PoolSrc src{keys_all, po, st, nullptr, nullptr, 0, rows};
    pool_body<WT, VEC, LPR, NCH, HYB, true, false>(W, src, fmeta, slot_field, B, D, n_bags, out, out_stride,
                                                   blockIdx.x, gridDim.x, NT, hv);
}

// Small batches: the whole forward pass is ONE launch.  The first blocks are the slices of the
// dedup (they find their occurrences in the caller's IDs), the next ones write what is per bag and
// per pack, and the rest pool: the pooling needs the rows' keys only, which it forms from the IDs
// itself, so it depends on nothing the other blocks write.  (With few occurrences a launch is
// mostly latency, and a second launch would wait for the first.)
constexpr int kFusedPacks = 16;
struct PoolPack {
    const void* W; const int32_t* slot_field;
    int64_t n_bags; int32_t D; int32_t variant; int32_t block_begin; uint32_t rows;
};
struct PoolJob {
    PoolPack pack[kFusedPacks];
    int32_t n_packs; int32_t B; int32_t n_blocks; int32_t pad;
    float* out; int64_t out_stride;
};

// variant = 12 * dtype + shape; the shapes in the order of the host's dispatch
#define PK_POOL_SHAPES(WT, VECW, base)                                                          \
    case base + 0:  pool_body<WT, VECW, 1, 1, false, false, true>(PK_POOL_ARGS); break;                 \
    case base + 1:  pool_body<WT, VECW, 2, 1, false, false, true>(PK_POOL_ARGS); break;                 \
    case base + 2:  pool_body<WT, VECW, 4, 1, false, false, true>(PK_POOL_ARGS); break;                 \
    case base + 3:  pool_body<WT, VECW, 8, 1, false, false, true>(PK_POOL_ARGS); break;                 \
    case base + 4:  pool_body<WT, VECW, 16, 1, false, false, true>(PK_POOL_ARGS); break;                \
    case base + 5:  pool_body<WT, VECW, 32, 1, false, false, true>(PK_POOL_ARGS); break;                \
    case base + 6:  pool_body<WT, VECW, 64, 1, false, false, true>(PK_POOL_ARGS); break;                \
    case base + 7:  pool_body<WT, 1, 4, 1, false, false, true>(PK_POOL_ARGS); break;                    \
    case base + 8:  pool_body<WT, 1, 16, 1, false, false, true>(PK_POOL_ARGS); break;                   \
    case base + 9:  pool_body<WT, 1, 64, 1, false, false, true>(PK_POOL_ARGS); break;                   \
    case base + 10: pool_body<WT, 1, 64, 2, false, false, true>(PK_POOL_ARGS); break;                   \
    case base + 11: pool_body<WT, 1, 64, 4, false, false, true>(PK_POOL_ARGS); break;
#define PK_POOL_ARGS                                                                            \
    static_cast<const WT_*>(k.W), src, a.fmeta, k.slot_field, pj.B, k.D, k.n_bags, pj.out, pj.out_stride, local,  \
        n_local, kSliceThreads, HotView{nullptr, nullptr, nullptr}

// WAVES: wavefronts per SIMD the kernel is compiled for.  8 lets two blocks share a compute unit, which a
// launch with more blocks than compute units needs; 4 gives a block twice the registers (nothing is then
// kept in scratch memory), which is faster when every block has a compute unit to itself.
template <int WAVES>
__global__ void __launch_bounds__(kSliceThreads, WAVES)
pk_fused_kernel(SliceArgs a, PoolJob pj, int slice_blocks, int meta_blocks)
{
    extern __shared__ int32_t s_dyn[];                     // kSliceTfWords words per field of a table
    __shared__ int32_t s_main[slice_lds_words(kSliceLogMax, kSliceRanks)];
    if ((int)blockIdx.x < slice_blocks) {
        slice_body<kSliceFused, kSliceThreads, kSliceLogMax, kSliceRanks>(a, blockIdx.x, s_main, s_dyn);
        return;
    }
    PK_PT(a, blockIdx.x, 0);
    if ((int)blockIdx.x < slice_blocks + meta_blocks) {
        meta_body(a, (int)blockIdx.x - slice_blocks, meta_blocks, s_main);
        PK_PT(a, blockIdx.x, 8);
        return;
    }
    const int pb = (int)blockIdx.x - slice_blocks - meta_blocks;
    int p = 0;
    while (p + 1 < pj.n_packs && pb >= pj.pack[p + 1].block_begin) ++p;
    const PoolPack k = pj.pack[p];
    const int local = pb - k.block_begin;
    const int n_local = (p + 1 < pj.n_packs ? pj.pack[p + 1].block_begin : pj.n_blocks) - k.block_begin;
    const PoolSrc src{nullptr, nullptr, nullptr, a.ids, a.offsets, a.nnz, k.rows};
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
    __syncthreads();
    PK_PT(a, blockIdx.x, 8);
}
