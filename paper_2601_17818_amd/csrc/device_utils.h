// Small device helpers: bf16 bit conversions and wavefront reductions (wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vitcop {

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// 16-byte streaming (non-temporal) load / store: data touched exactly once.
__device__ __forceinline__ uint4 ld_nt16(const void* p) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_nt16(void* p, const uint4& u) {
    u32x4 v = {u.x, u.y, u.z, u.w};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Two floats -> packed bf16 pair (round to nearest even), `a` in the low half.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    f32x2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Sum of squares of the 8 bf16 values packed in a uint4.
__device__ __forceinline__ float sumsq8(const uint4& u, float acc) {
    float a;
    a = bf16_lo(u.x); acc = fmaf(a, a, acc);
    a = bf16_hi(u.x); acc = fmaf(a, a, acc);
    a = bf16_lo(u.y); acc = fmaf(a, a, acc);
    a = bf16_hi(u.y); acc = fmaf(a, a, acc);
    a = bf16_lo(u.z); acc = fmaf(a, a, acc);
    a = bf16_hi(u.z); acc = fmaf(a, a, acc);
    a = bf16_lo(u.w); acc = fmaf(a, a, acc);
    a = bf16_hi(u.w); acc = fmaf(a, a, acc);
    return acc;
}

// Workgroup-wide exclusive scan of per-index counts over [first, end), in chunks of THREADS
// indices: store(i, count_i, exclusive_prefix_i) runs for every index, the total is returned.
// wave_tot: THREADS/64 ints of LDS.  Must be called by all THREADS threads; the last
// __syncthreads of the final chunk orders everything `store` wrote to LDS.
template <int THREADS, typename CountOf, typename Store>
__device__ inline int block_exclusive_scan(int first, int end, int* wave_tot, CountOf count_of, Store store) {
    const int tid = threadIdx.x;
    int running = 0;
    for (int i0 = first; i0 < end; i0 += THREADS) {
        const int i = i0 + tid;
        const int f = i < end ? count_of(i) : 0;
        int incl = f;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o, 64);
            if ((tid & 63) >= o) incl += t;
        }
        if ((tid & 63) == 63) wave_tot[tid >> 6] = incl;
        __syncthreads();
        int before = running, chunk = 0;
#pragma unroll
        for (int w = 0; w < THREADS / 64; ++w) {
            if (w < (tid >> 6)) before += wave_tot[w];
            chunk += wave_tot[w];
        }
        if (i < end) store(i, f, before + incl - f);
        running += chunk;
        __syncthreads();
    }
    return running;
}

}  // namespace vitcop
