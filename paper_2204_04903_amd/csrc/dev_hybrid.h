// HybridHash (Sec. III-D, Alg. 1): the bookkeeping kernels of the Hot-storage.
// Part of pk_device.hip: included there, in this order, inside its anonymous namespace.

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
