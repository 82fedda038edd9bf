// Hardware yardsticks for bench.py --hardware-rates: random single-word operations over a table and
// the XCD a workgroup runs on.  Nothing here generates inputs or belongs to the library: the kernels
// only measure what the GPU does with access patterns like those of the dedup kernels.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t x) {     // splitmix64 finaliser
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
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

extern "C" int bp_random_ops(int mode, void* table, int64_t n_slots, int64_t n_ops, uint64_t salt, void* stream) {
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
extern "C" int bp_xcd_map(void* out, int64_t n_blocks, void* stream) {
    if (n_blocks <= 0) return 0;
    hipLaunchKernelGGL(xcd_map, dim3((unsigned)n_blocks), dim3(64), 0, (hipStream_t)stream, (uint32_t*)out);
    return (int)hipGetLastError();
}

