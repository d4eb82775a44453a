// Small device-side helpers for gfx950 kernels (wave64).
#pragma once
#include <type_traits>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace seedv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// float -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ uint32_t pack2bf(float lo, float hi) {
    return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16);
}

// Activations that feed a projection are kept as TWO bf16 values per element, hi = bf16(x) and
// lo = bf16(x - hi): the MFMA then sees x to ~16 significant bits while the weights stay plain bf16, so
// rounding of activations does not accumulate over the layers (a single bf16 costs ~0.2 % per projection).
// Offset (in elements) of the hi part of element (row r, column c) in the MFMA-fragment-packed layout
// [m-tile][k-tile][hi|lo][lane][8]: 16 rows x 32 columns per 1 KiB tile, lane = (r % 16) + 16 * ((c % 32) / 8);
// the lo part sits kActLoOffset elements further.
constexpr int kActLoOffset = 512;
__device__ __host__ __forceinline__ size_t packed_offset(int r, int c, int KT) {
    return (((((size_t)(r >> 4) * KT + (c >> 5)) * 2) * 64) + (r & 15) + 16 * ((c & 31) >> 3)) * 8 + (c & 7);
}
__device__ __forceinline__ void split_bf16(float x, uint16_t &hi, uint16_t &lo) {
    hi = f2bf(x);
    lo = f2bf(x - bf2f(hi));
}

// The same split for two values with the hardware conversion (v_cvt_pk_bf16_f32, round to nearest even):
// half the instructions of the integer form.  hi2 / lo2 hold x0's part in the low half.
__device__ __forceinline__ void split_bf16_x2(float x0, float x1, uint32_t &hi2, uint32_t &lo2) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const bf16x2_t h = __builtin_convertvector((f32x2_t){x0, x1}, bf16x2_t);
    hi2 = *reinterpret_cast<const uint32_t *>(&h);
    const bf16x2_t l = __builtin_convertvector(
        (f32x2_t){x0 - __uint_as_float(hi2 << 16), x1 - __uint_as_float(hi2 & 0xFFFF0000u)}, bf16x2_t);
    lo2 = *reinterpret_cast<const uint32_t *>(&l);
}

// bf16 V cache of one head, "chunk-tiled transposed": [cap/32][dh][32 keys].  The attention kernel reads V^T
// fragments (16 dims x 32 keys, 16 bytes per lane); with this order the 32-key chunk it works on is one
// contiguous dh*64-byte block, like the matching K chunk ([cap][dh] row-major), instead of dh pieces of 64
// bytes that lie 2*cap bytes apart.  cap is a multiple of 32.
__device__ __host__ __forceinline__ size_t vt_offset(int d, int key, int dh) {
    return ((size_t)(key >> 5) * dh + d) * 32 + (key & 31);
}

__device__ __forceinline__ float wave_reduce_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// The same sum without the LDS crossbar for the first four steps: lanes are combined inside their row of 16 by
// DPP moves (xor 1, xor 2, mirror of 8, mirror of 16: plain vector-ALU operands), and the four row sums are
// read as scalars.  A __shfl_xor step is a ds_bpermute with its own round trip; six of them per value, for a
// dozen values one after the other, is microseconds.  (Different association than wave_reduce_sum.)
__device__ __forceinline__ float wave_reduce_sum_dpp(float v) {
    auto step = [](float x, auto ctrl) {
        const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, 0xf, 0xf, true);
        return x + __builtin_bit_cast(float, moved);
    };
    v = step(v, std::integral_constant<int, 0xB1>{});    // quad_perm [1,0,3,2]
    v = step(v, std::integral_constant<int, 0x4E>{});    // quad_perm [2,3,0,1]
    v = step(v, std::integral_constant<int, 0x141>{});   // row_half_mirror
    v = step(v, std::integral_constant<int, 0x140>{});   // row_mirror
    const int bits = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(bits, 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(bits, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(bits, 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(bits, 48));
    return (r0 + r1) + (r2 + r3);
}

// Data handed from one workgroup to another INSIDE a launch (split-K partials, per-tile sums of squares)
// moves with agent-scope relaxed atomic stores / loads: they write through, resp. read around, the per-XCD
// L2, so the hand-over needs no full-L2 write-back / invalidate fence (which costs ~100 us per launch when
// every workgroup issues one); ordering is "wait for my stores, workgroup barrier, bump the counter".
__device__ __forceinline__ void store_agent(float *p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_agent(const float *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// two adjacent floats (8-byte aligned) as one 64-bit access
__device__ __forceinline__ void store2_agent(float *p, float x, float y) {
    const unsigned long long w = (unsigned long long)__float_as_uint(x) | ((unsigned long long)__float_as_uint(y) << 32);
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void load2_agent(const float *p, float &x, float &y) {
    const unsigned long long w = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
    x = __uint_as_float((uint32_t)w);
    y = __uint_as_float((uint32_t)(w >> 32));
}
// four adjacent floats (16-byte aligned) as two 64-bit accesses
__device__ __forceinline__ void store4_agent(float *p, const f32x4 &v) {
    store2_agent(p, v[0], v[1]);
    store2_agent(p + 2, v[2], v[3]);
}
__device__ __forceinline__ f32x4 load4_agent(const float *p) {
    f32x4 v;
    float a, b, c, e;
    load2_agent(p, a, b);
    load2_agent(p + 2, c, e);
    v[0] = a; v[1] = b; v[2] = c; v[3] = e;
    return v;
}
// all of this workgroup's earlier stores have completed; returns true in the workgroup that arrives last
__device__ __forceinline__ bool arrive_last(int *counter, int expected, int *s_flag) {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) {
        const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = (old == expected - 1);
        if (*s_flag) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // re-arm
    }
    __syncthreads();
    return *s_flag != 0;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding global
// load of the wavefront (vmcnt(0)), which would drain a prefetch queue at each chunk; here only the LDS counter
// is drained, global loads stay in flight across the barrier.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

}  // namespace seedv
