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

// Random single-word operations over a table: the yardstick for the dedup kernels, whose cost is
// the number of random device-scope atomics / loads / stores rather than bytes.
// mode 0: atomicMin u64 (result unused), 1: atomicMin u32, 2: store 8 B, 3: load 8 B,
//      4: atomicMin u64 at workgroup scope, 5: atomicMin u64 (device scope) with every XCD confined
//      to its own eighth of the table, 6: as 5 at workgroup scope, 7: load 8 B, confined likewise.
// The confined modes ask whether keeping a table inside one XCD's L2 raises the rate.
__device__ __forceinline__ uint32_t xcc_id() {       // hardware register XCC_ID, bits 3:0
    return __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7u;
}

template <int MODE>
__global__ void random_ops(uint64_t* t64, uint32_t* t32, uint64_t n_slots, int64_t n_ops, uint64_t salt, uint64_t* sink) {
    uint64_t acc = 0;
    const bool confined = MODE >= 5;
    const uint64_t span = confined ? n_slots / 8 : n_slots;
    const uint64_t base = confined ? (uint64_t)xcc_id() * span : 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_ops; i += (int64_t)gridDim.x * blockDim.x) {
        const uint64_t s = base + mix64((uint64_t)i + salt) % span;
        if (MODE == 0 || MODE == 5) atomicMin((unsigned long long*)&t64[s], (unsigned long long)i);
        if (MODE == 1) atomicMin(&t32[s], (uint32_t)i);
        if (MODE == 2) t64[s] = (uint64_t)i;
        if (MODE == 3 || MODE == 7) acc += t64[s];
        if (MODE == 4 || MODE == 6) __hip_atomic_fetch_min(&t64[s], (uint64_t)i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    if (acc == 0x123456789ull) *sink = acc;
}

// xcd_of[b] = XCD that ran workgroup b
__global__ void xcd_map(uint32_t* xcd_of) {
    if (threadIdx.x == 0) xcd_of[blockIdx.x] = xcc_id();
}

}  // namespace

extern "C" int qg_random_ops_device(int mode, void* table, int64_t n_slots, int64_t n_ops, uint64_t salt, void* stream) {
    if (n_slots < 16 || n_ops <= 0) return 0;
    int64_t blocks = (n_ops + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipStream_t s = (hipStream_t)stream;
    uint64_t* t64 = (uint64_t*)table;
    uint32_t* t32 = (uint32_t*)table;
    uint64_t* sink = t64 + (n_slots - 1);
    dim3 g((unsigned)blocks), b(256);
#define QG_MODE(M) case M: hipLaunchKernelGGL(random_ops<M>, g, b, 0, s, t64, t32, (uint64_t)n_slots - 1, n_ops, salt, sink); break;
    switch (mode) {
        QG_MODE(0) QG_MODE(1) QG_MODE(2) QG_MODE(3) QG_MODE(4) QG_MODE(5) QG_MODE(6) QG_MODE(7)
        default: return -1;
    }
#undef QG_MODE
    return (int)hipGetLastError();
}

// out[b] = XCD of workgroup b for a launch of n_blocks workgroups
extern "C" int qg_xcd_map_device(void* out, int64_t n_blocks, void* stream) {
    if (n_blocks <= 0) return 0;
    hipLaunchKernelGGL(xcd_map, dim3((unsigned)n_blocks), dim3(64), 0, (hipStream_t)stream, (uint32_t*)out);
    return (int)hipGetLastError();
}

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
