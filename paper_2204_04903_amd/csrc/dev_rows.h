// Row access (fp32 / bf16, 16 bytes per lane) and where a row lives (plain table or HybridHash).
// Part of pk_device.hip: included there, in this order, inside its anonymous namespace.

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

// (rows and dimensions are unsigned 32-bit numbers: the products below are one 32 x 32 -> 64 bit multiply each)
template <typename WT, bool HYB>
__device__ __forceinline__ WT* row_of(WT* cold, const HotView& hv, uint32_t row, int D)
{
    if constexpr (HYB) {
        const int s = hv.slot_of[row];
        if (s >= 0) return static_cast<WT*>(hv.W_hot) + (size_t)((uint64_t)(uint32_t)s * (uint32_t)D);
    }
    return cold + (size_t)((uint64_t)row * (uint32_t)D);
}

// the row's weights and its accumulator
template <typename WT>
__device__ __forceinline__ void rows_of(WT* W, float* A, const HotView& hv, uint32_t row, int D, WT** wrow, float** arow)
{
    if (hv.slot_of) {
        const int s = hv.slot_of[row];
        if (s >= 0) {
            *wrow = static_cast<WT*>(hv.W_hot) + (size_t)((uint64_t)(uint32_t)s * (uint32_t)D);
            *arow = hv.A_hot + (size_t)((uint64_t)(uint32_t)s * (uint32_t)D);
            return;
        }
    }
    *wrow = W + (size_t)((uint64_t)row * (uint32_t)D);
    *arow = A + (size_t)((uint64_t)row * (uint32_t)D);
}
