// Device-side helpers shared by the kernels of the eOptShrinkQ library (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "eoq.h"

namespace eoqdev {

typedef _Float16 half_t;

// ---- cross-lane moves (DPP) -------------------------------------------------------------------
// ctrl: 0xB1 = lane^1 and 0x4E = lane^2 inside groups of 4; 0x120+n = rotate by n inside rows of 16;
// 0x140 = mirror of a row of 16 (lane -> 15 - lane), 0x141 = mirror of each half row (lane -> 7 - lane).
template <int CTRL>
__device__ __forceinline__ double dpp_mov(double v) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __builtin_amdgcn_mov_dpp(lo, CTRL, 0xF, 0xF, true);
  hi = __builtin_amdgcn_mov_dpp(hi, CTRL, 0xF, 0xF, true);
  return __hiloint2double(hi, lo);
}
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp_mov(int v) {
  return __builtin_amdgcn_mov_dpp(v, CTRL, 0xF, 0xF, true);
}

// sum over the 2 / 4 lanes of an aligned group; every lane of the group gets the total
template <typename T>
__device__ __forceinline__ T pair_sum(T v) { return v + dpp_mov<0xB1>(v); }
template <typename T>
__device__ __forceinline__ T quad_sum(T v) {
  v += dpp_mov<0xB1>(v);
  v += dpp_mov<0x4E>(v);
  return v;
}
// sum over a row of 16 lanes; every lane of the row gets a total (association may differ by lane)
__device__ __forceinline__ double row16_sum(double v) {
  v += dpp_mov<0xB1>(v);
  v += dpp_mov<0x4E>(v);
  v += dpp_mov<0x124>(v);
  v += dpp_mov<0x128>(v);
  return v;
}
// the same with a butterfly of commutative pair sums (lane^1, lane^2, 7-lane, 15-lane): bit-identical in all
// 16 lanes
__device__ __forceinline__ double row16_sum_uniform(double v) {
  v += dpp_mov<0xB1>(v);
  v += dpp_mov<0x4E>(v);
  v += dpp_mov<0x141>(v);
  v += dpp_mov<0x140>(v);
  return v;
}
__device__ __forceinline__ double readlane_f64(double v, int lane) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
  return __hiloint2double(hi, lo);
}
// sum over the 64 lanes of the wave; bit-identical in every lane
__device__ __forceinline__ double wave_sum_uniform(double v) {
  v = row16_sum(v);
  return (readlane_f64(v, 0) + readlane_f64(v, 16)) + (readlane_f64(v, 32) + readlane_f64(v, 48));
}
__device__ __forceinline__ double wave_sum_shfl(double v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

// ---- number formats ---------------------------------------------------------------------------
// double -> binary16 with a single rounding (round-to-odd into binary32 first)
__device__ __forceinline__ uint16_t double_to_half_bits(double x) {
  float f = __double2float_rz(x);
  if ((double)f != x) f = __int_as_float(__float_as_int(f) | 1);
  half_t h = (half_t)f;
  return *reinterpret_cast<uint16_t*>(&h);
}
// float -> binary16, round to nearest even, saturating at the largest finite value (one median-of-three, then the
// conversion)
__device__ __forceinline__ uint16_t float_to_half_bits(float f) {
  f = __builtin_amdgcn_fmed3f(f, -65504.0f, 65504.0f);
  half_t h = (half_t)f;
  return *reinterpret_cast<uint16_t*>(&h);
}
// Kernels that set the mode bit FP16_OVFL (binary16 results that overflow become the largest finite value instead of
// infinity) get the same saturation from the conversion alone.
__device__ __forceinline__ void set_fp16_overflow_clamp() { __builtin_amdgcn_s_setreg(1 | (23 << 6) | (0 << 11), 1); }
__device__ __forceinline__ uint16_t float_to_half_bits_clamped_by_mode(float f) {
  half_t h = (half_t)f;
  return *reinterpret_cast<uint16_t*>(&h);
}
// two floats -> two binary16 in one word (low half first), round to nearest even: one v_cvt_pk_f16_f32
__device__ __forceinline__ uint32_t pack_half2(float a, float b) {
  typedef _Float16 half2v __attribute__((ext_vector_type(2)));
  typedef float float2v __attribute__((ext_vector_type(2)));
  const float2v v = {a, b};
  const half2v h = __builtin_convertvector(v, half2v);
  return *reinterpret_cast<const uint32_t*>(&h);
}
__device__ __forceinline__ float half_bits_to_float(uint16_t b) {
  half_t h = *reinterpret_cast<half_t*>(&b);
  return (float)h;
}

// Load 8 consecutive elements of a block (binary16 or float32) as floats.
__device__ __forceinline__ void load8(const void* base, int dtype, size_t elem, float (&v)[8]) {
  if (dtype == EOQ_F16) {
    const uint4 raw = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + elem);
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = half_bits_to_float((uint16_t)(w[i] & 0xFFFFu));
      v[2 * i + 1] = half_bits_to_float((uint16_t)(w[i] >> 16));
    }
  } else {
    const float4 a = *reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem);
    const float4 b = *reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
}

// The four bytes of each of x0 .. x3, transposed: out[k] = bytes k of x0, x1, x2, x3 (x0 lowest).  Eight byte
// permutes: pairs first (bytes 0/1 and 2/3 of two words interleaved), then the halves of the pairs.
__device__ __forceinline__ void transpose_bytes(uint32_t x0, uint32_t x1, uint32_t x2, uint32_t x3, uint32_t (&out)[4]) {
  const uint32_t a01 = __builtin_amdgcn_perm(x1, x0, 0x05010400u), b01 = __builtin_amdgcn_perm(x1, x0, 0x07030602u);
  const uint32_t a23 = __builtin_amdgcn_perm(x3, x2, 0x05010400u), b23 = __builtin_amdgcn_perm(x3, x2, 0x07030602u);
  out[0] = __builtin_amdgcn_perm(a23, a01, 0x05040100u);
  out[1] = __builtin_amdgcn_perm(a23, a01, 0x07060302u);
  out[2] = __builtin_amdgcn_perm(b23, b01, 0x05040100u);
  out[3] = __builtin_amdgcn_perm(b23, b01, 0x07060302u);
}

// Compile-time loop: every index into a per-lane register array must be a constant before the optimiser
// first looks at the array, otherwise the array is kept in (scratch) memory.
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}
#define EOQ_SFOR(var, n, ...) eoqdev::static_for<0, n>([&](auto var##_ic) __attribute__((always_inline)) { \
  constexpr int var = decltype(var##_ic)::value; __VA_ARGS__ })

// old with lane LANE (a constant) replaced by the wave-uniform value val: one instruction (v_writelane_b32) where a
// compare and a select per lane would be two.  Reached through the compiler's own intrinsic, not inline assembly:
// a vector compare that has just written the scalar operand must be two instructions away, and only the compiler
// sees both.
extern "C" __device__ uint32_t eoq_llvm_writelane(uint32_t val, uint32_t lane, uint32_t old) __asm("llvm.amdgcn.writelane.i32");
template <int LANE>
__device__ __forceinline__ uint32_t write_lane(uint32_t old, uint32_t val) {
  return eoq_llvm_writelane(val, LANE, old);
}

}  // namespace eoqdev
