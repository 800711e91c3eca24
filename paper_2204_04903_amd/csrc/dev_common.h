// Device helpers shared by the kernels: block scans, the folding hash, single-pass multi-block prefix
// sums (descriptors and look-back), the XCD-aware tile order.
// Part of pk_device.hip: included there, in this order, inside its anonymous namespace.

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

// The row of an ID: the ID, taken as an unsigned 64-bit number, modulo the table's rows (exact).
// magic = floor((2^64 - 1) / rows): the upper half of ID * magic is the quotient or up to two below
// it, so the remainder formed from it is put right by two conditional subtractions (rows <= 2^30:
// nothing overflows).  A dozen integer operations instead of a 64-bit division.
__device__ __forceinline__ uint64_t fold_magic(uint32_t rows) { return ~(uint64_t)0 / (uint64_t)rows; }

__device__ __forceinline__ uint32_t fold_id(int64_t id, uint32_t rows, uint64_t magic)
{
    const uint64_t u = (uint64_t)id;
    if (u < rows) return (uint32_t)u;
    const uint64_t q = __umul64hi(u, magic);
    uint64_t r = u - q * (uint64_t)rows;
    if (r >= rows) r -= rows;
    if (r >= rows) r -= rows;
    return (uint32_t)r;
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
// single-pass multi-block prefix sums: every work item publishes a 64-bit
// descriptor (state | flag | value b | value a) and sums the descriptors of the
// items before it.  Block i takes item i and nothing else, and an item waits
// only for lower items: the hardware starts the blocks of a launch in index
// order, so whatever a block waits for belongs to a block that has started (or
// finished), however many blocks the chip holds at once and whatever else runs
// beside the launch.  The wait is bounded all the same: running out of patience
// raises a flag, which travels with the sums to every later item; the kernels
// turn it into bit 1 of the pack's error word, the kernels after them skip
// their work and the tables stay as they are.
// ---------------------------------------------------------------------------
constexpr uint64_t kDescAgg = 1, kDescPfx = 2;
constexpr int kSpinLimit = 1 << 22;

// a: 31 bits, b: 29 bits, flags: 2 bits (the bits of the error word)
__device__ __forceinline__ uint64_t make_desc(uint64_t state, uint32_t a, uint32_t b, uint32_t flags)
{
    return (state << 62) | ((uint64_t)(flags & 3u) << 60) | ((uint64_t)(b & 0x1FFFFFFFu) << 31) | (uint64_t)(a & 0x7FFFFFFFu);
}

__device__ __forceinline__ void publish_desc(uint64_t* d, uint64_t v)
{
    __hip_atomic_store(d, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One round of a look-back: lane i reads d[-i] if it is `valid`; the wave waits until every valid lane's
// descriptor is there (bounded), then adds, into acc_*, the descriptors from lane 0 up to the nearest one
// that carries a prefix.  Returns whether a prefix was met.
__device__ __forceinline__ bool lookback_round(const uint64_t* d_lane0, bool valid, uint32_t* acc_a, uint32_t* acc_b,
                                               uint32_t* acc_f)
{
    const int lane = threadIdx.x & 63;
    uint64_t d = make_desc(kDescAgg, 0, 0, 0);
    int spins = 0;
    while (true) {
        if (valid) d = __hip_atomic_load(d_lane0 - lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool ready = (d >> 62) != 0;
        if (__ballot(ready) == ~0ull) break;
        if (++spins > kSpinLimit) {
            d = make_desc(kDescPfx, 0, 0, 2);          // flag bit 1: waited too long
            break;
        }
        __builtin_amdgcn_s_sleep(2);
    }
    const uint64_t pfx_mask = __ballot(valid && (d >> 62) == kDescPfx);
    int last = 64;                                       // lanes [0, last] contribute
    if (pfx_mask) last = __ffsll((unsigned long long)pfx_mask) - 1;
    if (valid && lane <= last) {
        *acc_a += (uint32_t)(d & 0x7FFFFFFFull);
        *acc_b += (uint32_t)((d >> 31) & 0x1FFFFFFFull);
        *acc_f |= (uint32_t)((d >> 60) & 3ull);
    }
    return pfx_mask != 0;
}

// Sums of a and b, and the OR of the flags, over the items [first, me) of one chain (the slices of a pack).
// Two levels keep the walk short however many blocks run side by side: items are taken in groups of 64,
// and the last item of a group also publishes the group's sum (and, once it knows it, the prefix up to
// the group's end) in gdesc[g0 + group], so an item reads its own group's earlier items and then whole
// groups.  own_*: what this item itself adds.  Called by all 64 lanes of one wave.
__device__ __forceinline__ void lookback_grouped(uint64_t* desc, uint64_t* gdesc, int first, int g0, int me,
                                                 uint32_t own_a, uint32_t own_b, uint32_t own_f,
                                                 uint32_t* out_a, uint32_t* out_b, uint32_t* out_f)
{
    const int lane = threadIdx.x & 63;
    const int l = me - first, g = l >> 6, r = l & 63;
    uint32_t a = 0, b = 0, f = 0;
    bool done = lookback_round(desc + me - 1, lane < r, &a, &b, &f);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        a += __shfl_xor(a, o, 64);
        b += __shfl_xor(b, o, 64);
        f |= __shfl_xor(f, o, 64);
    }
    if (r == 63 && lane == 0)
        publish_desc(gdesc + g0 + g, make_desc(done ? kDescPfx : kDescAgg, a + own_a, b + own_b, f | own_f));
    uint32_t ga = 0, gb = 0, gf = 0;
    for (int hi = g; hi > 0 && !done; hi -= 64)
        done = lookback_round(gdesc + g0 + hi - 1, hi - 1 - lane >= 0, &ga, &gb, &gf);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        ga += __shfl_xor(ga, o, 64);
        gb += __shfl_xor(gb, o, 64);
        gf |= __shfl_xor(gf, o, 64);
    }
    *out_a = a + ga;
    *out_b = b + gb;
    *out_f = f | gf;
}

// cnt[idx] += 1 for every lane with `active`, and the value before the lane's own increment is
// returned.  IDs are heavily skewed (Sec. II-B), so many lanes of a wavefront often hit one counter,
// and LDS atomics on one address run one after the other: the lanes that share the first active
// lane's counter are combined into one add (up to two such groups are peeled off); a wavefront whose
// first group is a single lane is taken to have few repeats and goes on with plain atomics.
// Must be called by all 64 lanes of a wavefront together.
__device__ __forceinline__ int lds_inc_grouped(int32_t* cnt, uint32_t idx, bool active)
{
    const int lane = threadIdx.x & 63;
    int pos = 0;
    bool todo = active;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const uint64_t m = __ballot(todo);
        if (!m) return pos;
        const int leader = __ffsll((unsigned long long)m) - 1;
        const uint32_t v = (uint32_t)__shfl((int)idx, leader, 64);
        const bool mine = todo && idx == v;
        const uint64_t same = __ballot(mine);
        const int n = __popcll(same);
        int base = 0;
        if (lane == leader) base = atomicAdd(&cnt[v], n);
        base = __shfl(base, leader, 64);
        if (mine) {
            pos = base + __popcll(same & ((1ull << lane) - 1ull));
            todo = false;
        }
        if (n == 1) break;
    }
    if (todo) pos = atomicAdd(&cnt[idx], 1);
    return pos;
}

// The same for counters that are few (idx < n, n small and the same for the whole wavefront): with a
// handful of counters nearly every lane shares its counter with others, and LDS atomics on one address
// run one after the other, so the wavefront goes through the counters and makes one add for each that
// some lane wants.  POS: the value before the lane's own increment is returned.
constexpr int kFewCounters = 2;
template <bool POS>
__device__ __forceinline__ int lds_inc_few(int32_t* cnt, uint32_t idx, bool active, int n)
{
    const int lane = threadIdx.x & 63;
    int pos = 0;
    for (int s = 0; s < n; ++s) {
        const bool mine = active && idx == (uint32_t)s;
        const uint64_t m = __ballot(mine);
        if (!m) continue;
        const int leader = __ffsll((unsigned long long)m) - 1;
        int base = 0;
        if (lane == leader) base = atomicAdd(&cnt[s], __popcll(m));
        if (POS) {
            base = __shfl(base, leader, 64);
            if (mine) pos = base + __popcll(m & ((1ull << lane) - 1ull));
        }
    }
    return pos;
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
