// H6 + H7: gradient reduction per distinct key fused with the sparse Adagrad update.
// Part of pk_device.hip: included there, in this order, inside its anonymous namespace.

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
                // square root and reciprocal as the hardware gives them (1 ulp each): the step is within
                // 3 ulp of lr*g/(sqrt(a)+eps), and it is at most lr in size
                w[c][v] = w[c][v] - lr * g * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(a[c][v]) + eps);
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
    const bool state_ok = (n_host < 0 || st->nnz == n_host) && st->error == 0;
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
    if (st[p].error) return;                               // as in pk_adagrad_kernel
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
                wrow[d] = wrow[d] - lr * g * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(a) + eps);
            }
        } else {
            uint16_t* wrow;
            float* arow;
            rows_of<uint16_t>(static_cast<uint16_t*>(ptrs.W[blockIdx.y]), ptrs.A[blockIdx.y], ptrs.hv[blockIdx.y], row, D, &wrow, &arow);
            for (int d = lane; d < D; d += 64) {
                const float g = (float)gh[(size_t)t * D + d];
                const float a = arow[d] + g * g;
                arow[d] = a;
                wrow[d] = (uint16_t)f32_to_bf16(bf16_to_f32(wrow[d]) - lr * g * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(a) + eps));
            }
        }
    }
}
