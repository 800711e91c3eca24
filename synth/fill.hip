// Seeded synthetic embedding-table values, device side (gfx950).
//
// Input generation only.  Writes, straight into HBM, the same bits that
// fill.c produces on the host for the same (seed, table, row, col): tables of
// tens of GB are initialised in place instead of being uploaded.  See fill.c
// for the definition of the value function.
#include <hip/hip_runtime.h>
#include <stdint.h>

#define SYNTH_GOLD   0x9E3779B97F4A7C15ull
#define SYNTH_ROWMUL 0xD1342543DE82EF95ull
#define SYNTH_SCALE  2.6429e-7f

__device__ __forceinline__ uint64_t synth_mix(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ float synth_value(uint64_t tkey, uint64_t row, uint64_t col)
{
    uint64_t h = synth_mix(tkey ^ (row * SYNTH_ROWMUL + col));
    int32_t s = (int32_t)(h & 0xFFFF) + (int32_t)((h >> 16) & 0xFFFF) +
                (int32_t)((h >> 32) & 0xFFFF) + (int32_t)(h >> 48) - 131070;
    return __fmul_rn((float)s, SYNTH_SCALE);
}

__device__ __forceinline__ uint16_t synth_bf16_rne(float v)
{
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <typename T>
__global__ void __launch_bounds__(256)
synth_fill_kernel(T* __restrict__ out, int64_t rows, int32_t dim, uint64_t tkey)
{
    const int64_t n = rows * (int64_t)dim;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride) {
        const int64_t r = e / dim;
        const int32_t c = (int32_t)(e - r * dim);
        const float v = synth_value(tkey, (uint64_t)r, (uint64_t)c);
        if constexpr (sizeof(T) == 4) out[e] = v;
        else out[e] = synth_bf16_rne(v);
    }
}

static uint64_t host_mix(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// W: device pointer to rows*dim elements (fp32 when dtype==0, bf16 bit
// patterns when dtype==1).  Enqueues on `stream` and returns the HIP error
// code of the launch (0 = success); negative for bad arguments.
extern "C" int synth_fill_device(void* W, int64_t rows, int32_t dim, int32_t dtype,
                                 uint64_t seed, int32_t table, void* stream)
{
    if (!W || rows <= 0 || dim <= 0 || (dtype != 0 && dtype != 1)) return -1;
    const uint64_t tkey = host_mix(seed + SYNTH_GOLD * (uint64_t)(table + 1));
    const int64_t n = rows * (int64_t)dim;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipStream_t s = (hipStream_t)stream;
    if (dtype == 0)
        hipLaunchKernelGGL(synth_fill_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, s,
                           (float*)W, rows, dim, tkey);
    else
        hipLaunchKernelGGL(synth_fill_kernel<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, s,
                           (uint16_t*)W, rows, dim, tkey);
    return (int)hipGetLastError();
}
