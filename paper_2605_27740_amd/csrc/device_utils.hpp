// Device-side helpers shared by the gfx950 kernels: 16-byte vector loads of fp32 / bf16 rows,
// bf16 <-> fp32 conversion, and cross-lane reductions over groups of 8..64 lanes (wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace unique {

using bf16_t = uint16_t;  // raw bf16 bit pattern

constexpr int kWave = 64;

template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int kVec = 4; };   // elements per 16-byte load
template <> struct Elem<bf16_t> { static constexpr int kVec = 8; };

__device__ __forceinline__ float bits_to_float(uint32_t u) { return __uint_as_float(u); }

// fp32 -> bf16, round to nearest even; NaN stays NaN.
__device__ __forceinline__ bf16_t float_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

__device__ __forceinline__ void store_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(bf16_t* p, float v) { *p = float_to_bf16(v); }
__device__ __forceinline__ float load_elem(const float* p) { return *p; }
__device__ __forceinline__ float load_elem(const bf16_t* p) { return bits_to_float((uint32_t)(*p) << 16); }

// One 16-byte load expanded to fp32 lanes. p must be 16-byte aligned.
__device__ __forceinline__ void load_vec(const float* p, float (&out)[4]) {
  const float4 v = *reinterpret_cast<const float4*>(p);
  out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
__device__ __forceinline__ void unpack_bf16x8(const uint4& v, float (&out)[8]) {
  out[0] = bits_to_float(v.x << 16); out[1] = bits_to_float(v.x & 0xffff0000u);
  out[2] = bits_to_float(v.y << 16); out[3] = bits_to_float(v.y & 0xffff0000u);
  out[4] = bits_to_float(v.z << 16); out[5] = bits_to_float(v.z & 0xffff0000u);
  out[6] = bits_to_float(v.w << 16); out[7] = bits_to_float(v.w & 0xffff0000u);
}
__device__ __forceinline__ void load_vec(const bf16_t* p, float (&out)[8]) {
  const uint4 v = *reinterpret_cast<const uint4*>(p);
  unpack_bf16x8(v, out);
}

// Raw 16-byte register image of a row chunk, so that loads can be issued early and unpacked late.
struct Raw16 { uint4 v; };
__device__ __forceinline__ Raw16 load_raw(const void* p) {
  Raw16 r; r.v = *reinterpret_cast<const uint4*>(p); return r;
}
// The same load marked non-temporal: for data that is read once per launch (K/V pages, statistic
// records). A plain streaming read measures about 6.3 TB/s on MI355X, a non-temporal one about 7.1 TB/s.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
// `nt` is uniform per launch: small working sets are better left to the caches (they are re-read by the next step).
__device__ __forceinline__ Raw16 load_raw_stream(const void* p, bool nt) {
  if (nt) {
    const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    Raw16 r; r.v = make_uint4(t.x, t.y, t.z, t.w); return r;
  }
  return load_raw(p);
}
__device__ __forceinline__ Raw16 zero_raw() { Raw16 r; r.v = make_uint4(0u, 0u, 0u, 0u); return r; }
__device__ __forceinline__ void unpack_raw(const Raw16& r, float (&out)[4], const float*) {
  out[0] = bits_to_float(r.v.x); out[1] = bits_to_float(r.v.y);
  out[2] = bits_to_float(r.v.z); out[3] = bits_to_float(r.v.w);
}
__device__ __forceinline__ void unpack_raw(const Raw16& r, float (&out)[8], const bf16_t*) {
  unpack_bf16x8(r.v, out);
}

// ---- DPP lane exchange inside a row of 16 lanes (no LDS traffic) ----
template <int kCtrl>
__device__ __forceinline__ float dpp_mov(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, 0xf, 0xf, true));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each 8
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each 16

// Minimum / maximum of an unsigned value over the 64 lanes of a wave (every lane gets the result): four DPP
// exchanges inside the rows of 16 lanes, then two cross-row shuffles.
template <bool kMax>
__device__ __forceinline__ uint32_t wave_allreduce_minmax(uint32_t x) {
  auto op = [](uint32_t a, uint32_t b) { return kMax ? (a > b ? a : b) : (a < b ? a : b); };
  x = op(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kDppXor1, 0xf, 0xf, true));
  x = op(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kDppXor2, 0xf, 0xf, true));
  x = op(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kDppHalfMirror, 0xf, 0xf, true));
  x = op(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kDppMirror, 0xf, 0xf, true));
  x = op(x, (uint32_t)__shfl_xor((int)x, 16, kWave));
  x = op(x, (uint32_t)__shfl_xor((int)x, 32, kWave));
  return x;
}

// Inclusive prefix sum over the 64 lanes of a wave: four row shifts inside each row of 16 lanes (a lane whose
// source lies outside its row adds 0), then lane 15 of rows 0 and 2 is added to rows 1 and 3, then lane 31 to
// rows 2 and 3. No LDS traffic.
__device__ __forceinline__ int wave_inclusive_scan(int x) {
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, true);   // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, true);   // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, true);   // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, true);   // row_shr:8
  x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
  x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
  return x;
}

struct OpSum { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };
struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); } };

// All-reduce over aligned groups of kWidth consecutive lanes (kWidth in 1,2,4,8,16,32,64): every lane
// of a group ends with the group's result.
template <int kWidth, typename Op>
__device__ __forceinline__ float group_allreduce(float x, Op op) {
  static_assert(kWidth == 1 || kWidth == 2 || kWidth == 4 || kWidth == 8 || kWidth == 16 || kWidth == 32 ||
                kWidth == 64, "group width");
  if constexpr (kWidth >= 2) x = op(x, dpp_mov<kDppXor1>(x));
  if constexpr (kWidth >= 4) x = op(x, dpp_mov<kDppXor2>(x));
  if constexpr (kWidth >= 8) x = op(x, dpp_mov<kDppHalfMirror>(x));
  if constexpr (kWidth >= 16) x = op(x, dpp_mov<kDppMirror>(x));
  if constexpr (kWidth >= 32) x = op(x, __shfl_xor(x, 16, kWave));
  if constexpr (kWidth >= 64) x = op(x, __shfl_xor(x, 32, kWave));
  return x;
}

// All-reduce across the kGroups = 64 / kStride lane groups of a wave: combines lanes that share
// lane % kStride. kStride in {8, 16, 32, 64}.
template <int kStride, typename Op>
__device__ __forceinline__ float cross_group_allreduce(float x, Op op) {
  if constexpr (kStride <= 8) x = op(x, __shfl_xor(x, 8, kWave));
  if constexpr (kStride <= 16) x = op(x, __shfl_xor(x, 16, kWave));
  if constexpr (kStride <= 32) x = op(x, __shfl_xor(x, 32, kWave));
  return x;
}

// Order-preserving map of fp32 to uint32 (larger float -> larger key); NaN maps to 0, below everything.
__device__ __forceinline__ uint32_t float_to_ordered(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;
  if (u == 0x80000000u) u = 0u;  // -0 and +0 compare equal
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

}  // namespace unique
