// Small device helpers shared by the kernel files.
#ifndef SB_DEVICE_UTILS_H
#define SB_DEVICE_UTILS_H

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

namespace sb {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

#define SB_INF __builtin_inff()

__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// float -> bf16, round to nearest even (finite inputs)
__device__ __forceinline__ uint16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
typedef float f32x2v __attribute__((ext_vector_type(2)));
// two floats -> a packed bf16 pair, round to nearest even (the hardware's conversion)
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2v{a, b}, bf16x2v));
}
__device__ __forceinline__ float ldf(const float* p) { return *p; }
__device__ __forceinline__ float ldf(const uint16_t* p) { return bf2f(*p); }

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

// value v of row m, column i -> the two bf16 parts used by the MFMA path:
// rows 0..7 hold the high parts, rows 8..15 the low parts (v ~= hi + lo).
__device__ __forceinline__ void split_store(uint16_t* xs, int ld, int m, int i, float v) {
    uint16_t hi = f2bf(v);
    uint16_t lo = f2bf(v - bf2f(hi));
    xs[(size_t)m * ld + i] = hi;
    xs[(size_t)(8 + m) * ld + i] = lo;
}
// the same with the low parts `lo_rows` rows after the high parts (prompt passes keep more rows)
__device__ __forceinline__ void split_store_rows(uint16_t* xs, int ld, int lo_rows, int m, int i, float v) {
    uint16_t hi = f2bf(v);
    uint16_t lo = f2bf(v - bf2f(hi));
    xs[(size_t)m * ld + i] = hi;
    xs[(size_t)(lo_rows + m) * ld + i] = lo;
}

// four values of row m, columns n..n+3 -> the two bf16 planes (8-byte stores)
__device__ __forceinline__ void split_store4(uint16_t* xs, int ld, int lo_rows, int m, int n, float4 v) {
    const uint16_t h0 = f2bf(v.x), h1 = f2bf(v.y), h2 = f2bf(v.z), h3 = f2bf(v.w);
    const uint16_t l0 = f2bf(v.x - bf2f(h0)), l1 = f2bf(v.y - bf2f(h1)), l2 = f2bf(v.z - bf2f(h2)), l3 = f2bf(v.w - bf2f(h3));
    *reinterpret_cast<uint2*>(xs + (size_t)m * ld + n) = make_uint2((uint32_t)h0 | ((uint32_t)h1 << 16), (uint32_t)h2 | ((uint32_t)h3 << 16));
    *reinterpret_cast<uint2*>(xs + (size_t)(lo_rows + m) * ld + n) =
        make_uint2((uint32_t)l0 | ((uint32_t)l1 << 16), (uint32_t)l2 | ((uint32_t)l3 << 16));
}

__device__ __forceinline__ void unpack8(uint4 v, float (&w)[8]) {
    w[0] = __uint_as_float(v.x << 16); w[1] = __uint_as_float(v.x & 0xffff0000u);
    w[2] = __uint_as_float(v.y << 16); w[3] = __uint_as_float(v.y & 0xffff0000u);
    w[4] = __uint_as_float(v.z << 16); w[5] = __uint_as_float(v.z & 0xffff0000u);
    w[6] = __uint_as_float(v.w << 16); w[7] = __uint_as_float(v.w & 0xffff0000u);
}
__device__ __forceinline__ void load8(const uint16_t* p, float (&w)[8]) {
    uint4 v = *reinterpret_cast<const uint4*>(p);
    w[0] = __uint_as_float(v.x << 16); w[1] = __uint_as_float(v.x & 0xffff0000u);
    w[2] = __uint_as_float(v.y << 16); w[3] = __uint_as_float(v.y & 0xffff0000u);
    w[4] = __uint_as_float(v.z << 16); w[5] = __uint_as_float(v.z & 0xffff0000u);
    w[6] = __uint_as_float(v.w << 16); w[7] = __uint_as_float(v.w & 0xffff0000u);
}
__device__ __forceinline__ void load8(const float* p, float (&w)[8]) {
    float4 a = *reinterpret_cast<const float4*>(p);
    float4 b = *reinterpret_cast<const float4*>(p + 4);
    w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w;
    w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
}

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + expf(-g)) * u; }

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
// streaming (non-temporal) 128-bit load: weights are read once per launch
__device__ __forceinline__ uint4 ld_weights_packed(const uint16_t* p) {
    u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

}  // namespace sb
#endif
