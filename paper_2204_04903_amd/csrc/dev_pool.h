// H3-H5: gather + pool + concatenate, and the kernel in which small batches share the sort's launch.
// Part of pk_device.hip: included there, in this order, inside its anonymous namespace.

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
