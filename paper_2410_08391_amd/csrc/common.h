// Device-side helpers shared by the HIP kernels of libkvp (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvp {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
__device__ __forceinline__ void from_f32(float& d, float v) { d = v; }
__device__ __forceinline__ void from_f32(bf16& d, float v) { d = (bf16)v; }  // round-to-nearest-even

// Value of another lane of the same row of 16 lanes, chosen by a DPP control word (quad
// permutations and row mirrors: every lane has a source, so no lane reads the fill value).
template <int CTRL>
__device__ __forceinline__ float row_dpp(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
// Sum / max over the 64 lanes of a wavefront; every lane gets the result.  The four steps inside
// a row of 16 lanes are DPP operands of the add itself (neighbour, pair, half-row mirror, row
// mirror: after them every lane of a row holds the row's total); only the two steps across
// rows go through the cross-lane network.
__device__ __forceinline__ float wave_sum(float v) {
  v += row_dpp<0xB1>(v);      // quad_perm [1,0,3,2]
  v += row_dpp<0x4E>(v);      // quad_perm [2,3,0,1]
  v += row_dpp<0x141>(v);     // row_half_mirror
  v += row_dpp<0x140>(v);     // row_mirror
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, row_dpp<0xB1>(v));
  v = fmaxf(v, row_dpp<0x4E>(v));
  v = fmaxf(v, row_dpp<0x141>(v));
  v = fmaxf(v, row_dpp<0x140>(v));
  v = fmaxf(v, __shfl_xor(v, 16, 64));
  v = fmaxf(v, __shfl_xor(v, 32, 64));
  return v;
}

// 16-byte load of data that is read once per call (weights of a one-token step, the predicted cache): the
// non-temporal hint keeps the line from displacing reused data in L2 and the memory-side cache, and the chip
// streams such reads measurably faster than plain loads.
__device__ __forceinline__ bf16x8 load_stream8(const bf16* p) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  return __builtin_bit_cast(bf16x8, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)));
}

// Loads 8 consecutive elements as floats (16-byte load for bf16, two for float).
__device__ __forceinline__ void load8(const bf16* p, float (&out)[8]) {
  bf16x8 v = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
  for (int i = 0; i < 8; ++i) out[i] = (float)v[i];
}
__device__ __forceinline__ void load8(const float* p, float (&out)[8]) {
  f32x4 a = *reinterpret_cast<const f32x4*>(p);
  f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
  for (int i = 0; i < 4; ++i) { out[i] = a[i]; out[4 + i] = b[i]; }
}

// Rotary angle for pair index d of a head: pos * theta^(-2d/head_dim).
// log2(theta) is passed in so the kernel evaluates exp2f(-(2d/hd) * log2_theta).
__device__ __forceinline__ void rope_sincos(int pos, int d, int head_dim, float log2_theta, float& s, float& c) {
  float inv_freq = exp2f(-(2.0f * (float)d / (float)head_dim) * log2_theta);
  float ang = (float)pos * inv_freq;
  // sincosf with full range reduction: positions reach 8191 rad at the first frequency.
  sincosf(ang, &s, &c);
}

}  // namespace kvp
