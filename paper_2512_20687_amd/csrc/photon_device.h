// Device-side helpers shared by the gfx950 kernels: 128-bit vector access,
// bf16 <-> fp32 conversion, DPP lane-group reductions for 64-wide wavefronts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace photon {

typedef uint16_t bf16_t;          // raw bfloat16 bits
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// fp32 -> bf16, round to nearest even: gfx950 converts a pair in one instruction (v_cvt_pk_bf16_f32).
typedef __bf16 bf16x2_native __attribute__((ext_vector_type(2)));
typedef float float2_native __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const float2_native v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_native));
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return pack_bf16x2(f, 0.f) & 0xffffu; }
// Split a pair of fp32 values into packed bf16 heads and packed bf16 remainders (x = head + remainder + O(2^-17 x)).
__device__ __forceinline__ void split_bf16x2(float a, float b, uint32_t& hi, uint32_t& lo) {
  hi = pack_bf16x2(a, b);
  lo = pack_bf16x2(a - bf16_lo(hi), b - bf16_hi(hi));
}

// One 16-byte chunk of a row as VEC fp32 values (VEC = 4 for fp32 storage, 8 for bf16).
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int VEC = 4;
  __device__ static __forceinline__ void load(const float* p, float (&v)[4]) {
    float4_t r = *reinterpret_cast<const float4_t*>(p);
    v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
  }
  __device__ static __forceinline__ void zero(float (&v)[4]) { v[0] = v[1] = v[2] = v[3] = 0.f; }
  __device__ static __forceinline__ void store(float* p, const float (&v)[4]) {
    float4_t r; r.x = v[0]; r.y = v[1]; r.z = v[2]; r.w = v[3];
    *reinterpret_cast<float4_t*>(p) = r;
  }
};
template <> struct Vec16<bf16_t> {
  static constexpr int VEC = 8;
  __device__ static __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
    uint4_t r = *reinterpret_cast<const uint4_t*>(p);
    v[0] = bf16_lo(r.x); v[1] = bf16_hi(r.x); v[2] = bf16_lo(r.y); v[3] = bf16_hi(r.y);
    v[4] = bf16_lo(r.z); v[5] = bf16_hi(r.z); v[6] = bf16_lo(r.w); v[7] = bf16_hi(r.w);
  }
  __device__ static __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
    uint4_t r;
    r.x = pack_bf16x2(v[0], v[1]); r.y = pack_bf16x2(v[2], v[3]);
    r.z = pack_bf16x2(v[4], v[5]); r.w = pack_bf16x2(v[6], v[7]);
    *reinterpret_cast<uint4_t*>(p) = r;
  }
};

// Raw 16-byte load kept as bits (conversion deferred so many loads stay in flight).
__device__ __forceinline__ uint4_t load16(const void* p) { return *reinterpret_cast<const uint4_t*>(p); }
// Same, marked non-temporal: data that is used exactly once should not displace anything in the caches.
__device__ __forceinline__ uint4_t load16_stream(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const uint4_t*>(p));
}
template <typename T> __device__ __forceinline__ void unpack16(const uint4_t& r, float* v);
template <> __device__ __forceinline__ void unpack16<float>(const uint4_t& r, float* v) {
  v[0] = __uint_as_float(r.x); v[1] = __uint_as_float(r.y); v[2] = __uint_as_float(r.z); v[3] = __uint_as_float(r.w);
}
template <> __device__ __forceinline__ void unpack16<bf16_t>(const uint4_t& r, float* v) {
  v[0] = bf16_lo(r.x); v[1] = bf16_hi(r.x); v[2] = bf16_lo(r.y); v[3] = bf16_hi(r.y);
  v[4] = bf16_lo(r.z); v[5] = bf16_hi(r.z); v[6] = bf16_lo(r.w); v[7] = bf16_hi(r.w);
}

// ---- 8-bit floating point (OCP E4M3: bias 7, no infinities, largest finite value 448) for K/V cache storage ----
struct fp8_t { uint8_t bits; };
typedef float f32x2_native __attribute__((ext_vector_type(2)));
// Two fp32 values -> two E4M3 bytes (lo in bits 0..7), nearest even.  The conversion instruction turns magnitudes
// beyond the format's range into NaN; storage saturates instead, so the values are clamped first (NaN stays NaN).
__device__ __forceinline__ uint32_t pack_fp8x2(float lo, float hi) {
  lo = fminf(fmaxf(lo, -448.f), 448.f);
  hi = fminf(fmaxf(hi, -448.f), 448.f);
  return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(lo, hi, 0, false) & 0xffffu;
}
template <> __device__ __forceinline__ void unpack16<fp8_t>(const uint4_t& r, float* v) {
  const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const f32x2_native a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);
    const f32x2_native b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);
    v[4 * i] = a.x; v[4 * i + 1] = a.y; v[4 * i + 2] = b.x; v[4 * i + 3] = b.y;
  }
}

template <typename T> __device__ __forceinline__ float to_f32(T x);
template <> __device__ __forceinline__ float to_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t x) { return __uint_as_float(uint32_t(x) << 16); }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return bf16_t(f32_to_bf16_bits(x)); }
template <> __device__ __forceinline__ fp8_t from_f32<fp8_t>(float x) { return fp8_t{(uint8_t)(pack_fp8x2(x, 0.f) & 0xffu)}; }

// ---- cross-lane moves on the data-parallel-primitive path (no LDS traffic) ----
template <int CTRL> __device__ __forceinline__ float dpp(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
constexpr int DPP_XOR1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141;  // lane i <-> 7-i inside each 8 lanes
constexpr int DPP_MIRROR = 0x140;       // lane i <-> 15-i inside each 16 lanes

// Sum over aligned groups of G consecutive lanes (G = 1, 2, 4, 8, 16, 32); every lane gets the total.
template <int G> __device__ __forceinline__ float group_sum(float x) {
  if (G >= 2) x += dpp<DPP_XOR1>(x);
  if (G >= 4) x += dpp<DPP_XOR2>(x);
  if (G >= 8) x += dpp<DPP_HALF_MIRROR>(x);
  if (G >= 16) x += dpp<DPP_MIRROR>(x);
  if (G >= 32) x += __shfl_xor(x, 16);
  return x;
}

// rotate a 128-bit register by 8 lanes inside every row of 16 lanes
__device__ __forceinline__ uint4_t rotate8(const uint4_t& v) {
  constexpr int ROW_ROR8 = 0x128;
  uint4_t r;
  r.x = __builtin_amdgcn_update_dpp(0, v.x, ROW_ROR8, 0xf, 0xf, false);
  r.y = __builtin_amdgcn_update_dpp(0, v.y, ROW_ROR8, 0xf, 0xf, false);
  r.z = __builtin_amdgcn_update_dpp(0, v.z, ROW_ROR8, 0xf, 0xf, false);
  r.w = __builtin_amdgcn_update_dpp(0, v.w, ROW_ROR8, 0xf, 0xf, false);
  return r;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float silu(float g) { return g / (1.0f + __expf(-g)); }

// operand of the bf16 matrix-core instructions: 8 consecutive k of one row
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2_native __attribute__((ext_vector_type(2)));
// Two fp32 values rounded to nearest-even fp16, saturated to the largest finite fp16, packed (lo in bits 0..15).
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
  const float2_native v = {fminf(fmaxf(lo, -65504.f), 65504.f), fminf(fmaxf(hi, -65504.f), 65504.f)};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_native));
}
// Same without the saturation, for values known to lie in [0, 1].
__device__ __forceinline__ uint32_t pack_f16x2_unit(float lo, float hi) {
  const float2_native v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_native));
}
__device__ __forceinline__ bf16x8_t as_bf16x8(const uint4_t& v) { return __builtin_bit_cast(bf16x8_t, v); }

// cos and sin of the rotary angle pos * theta^(-2i/d_h); the angle is formed in double because positions reach 10^5
__device__ __forceinline__ void rope_angle(int pos, int i, int d_h, float theta, float& c, float& s) {
  if (theta == 0.f) { c = 1.f; s = 0.f; return; }
  const double inv_freq = exp2(-2.0 * (double)i / (double)d_h * log2((double)theta));
  double sd, cd;
  sincos((double)pos * inv_freq, &sd, &cd);
  c = (float)cd; s = (float)sd;
}

constexpr float LOG2E = 1.4426950408889634f;
constexpr float NEG_BIG = -1.0e30f;     // finite stand-in for -inf as running maximum

}  // namespace photon
