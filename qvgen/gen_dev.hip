// Device-side twin of the host feature generator: fills an n x dim feature table directly in
// HBM so that tables of tens of GB never pass through host memory.  Pure data generation; the
// integer part is exact and the single fp32 multiply and the fp16 conversion (round to nearest
// even, done with integer operations) round identically on host and device, so both produce the same bits.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <cstdint>

namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t x) {
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27; x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}
__device__ __forceinline__ uint64_t hash4(uint64_t seed, uint64_t dom, uint64_t a, uint64_t b) {
    uint64_t x = mix64(seed ^ (dom * 0xD6E8FEB86659FD93ull + 0x9E3779B97F4A7C15ull));
    x = mix64(x + a * 0x9E3779B97F4A7C15ull + 1);
    x = mix64(x ^ (b * 0xC2B2AE3D27D4EB4Full + 2));
    return x;
}
__device__ __forceinline__ float feature_value(uint64_t seed, uint64_t i, uint64_t j) {
    uint64_t h = hash4(seed, 3, i, j);
    int32_t s = (int32_t)(h & 0xFFFF) + (int32_t)((h >> 16) & 0xFFFF) +
                (int32_t)((h >> 32) & 0xFFFF) + (int32_t)(h >> 48) - 131070;
    return __fmul_rn((float)s, 2.6428998e-5f);
}

// fp32 -> fp16, round to nearest even, written out with integer operations (the same steps as
// the host generator) so that the compiler cannot merge the multiply and the conversion into
// one mixed-precision instruction with a single rounding.
__device__ __forceinline__ uint16_t f32_to_f16_rne(float f) {
    uint32_t x = __float_as_uint(f);
    uint32_t sign = (x >> 16) & 0x8000u;
    int32_t e = (int32_t)((x >> 23) & 0xFF) - 127 + 15;
    uint32_t m = x & 0x7FFFFFu;
    if (e >= 31) return (uint16_t)(sign | 0x7C00u);
    if (e <= 0) {
        if (e < -10) return (uint16_t)sign;
        m |= 0x800000u;
        int shift = 14 - e;
        uint32_t half = m >> shift, rem = m & ((1u << shift) - 1), mid = 1u << (shift - 1);
        if (rem > mid || (rem == mid && (half & 1))) ++half;
        return (uint16_t)(sign | half);
    }
    uint32_t half = ((uint32_t)e << 10) | (m >> 13), rem = m & 0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (half & 1))) ++half;
    return (uint16_t)(sign | half);
}

template <typename T>
__global__ void fill_features(uint64_t seed, int64_t row_begin, int64_t n_rows, int64_t dim, T* out) {
    int64_t total = n_rows * dim;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x) {
        int64_t r = idx / dim, j = idx - r * dim;
        float v = feature_value(seed, (uint64_t)(row_begin + r), (uint64_t)j);
        if constexpr (sizeof(T) == 4) out[idx] = v;
        else out[idx] = f32_to_f16_rne(v);
    }
}

// Plain 16-byte-per-lane copy of a known size: the yardstick that hardware byte counters
// (FETCH_SIZE / WRITE_SIZE) are scaled by when the library's kernels are profiled.
__global__ void copy_bytes(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n_vec) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += (int64_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

}  // namespace

extern "C" int qg_copy_device(const void* src, void* dst, int64_t n_bytes, void* stream) {
    int64_t n_vec = n_bytes / 16;
    if (n_vec <= 0) return 0;
    int64_t blocks = (n_vec + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(copy_bytes, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst, n_vec);
    return (int)hipGetLastError();
}

extern "C" int qg_features_device(uint64_t seed, int64_t row_begin, int64_t n_rows, int64_t dim,
                                  int elem_bytes, void* out, void* stream) {
    if (n_rows <= 0 || dim <= 0) return 0;
    int64_t total = n_rows * dim;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipStream_t s = (hipStream_t)stream;
    if (elem_bytes == 4)
        hipLaunchKernelGGL(fill_features<float>, dim3((unsigned)blocks), dim3(256), 0, s, seed, row_begin, n_rows, dim, (float*)out);
    else if (elem_bytes == 2)
        hipLaunchKernelGGL(fill_features<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, s, seed, row_begin, n_rows, dim, (uint16_t*)out);
    else
        return -1;
    return (int)hipGetLastError();
}
