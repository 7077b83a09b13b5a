// 16-bit helpers, MFMA wrappers and the "fragment-tiled" memory layouts of the bf16 path.
//
// Number formats: the caller's weights are bf16.  Every bf16 value of magnitude in
// [2^-17, 65504] is exactly an fp16 value, so the re-tiled weights are stored as fp16 and the
// matrix cores run in fp16 (same rate and bytes as bf16): activations and the KV cache then
// keep 11 significant bits instead of 8, which is what the log-probability tolerance needs.
//
// v_mfma_f32_16x16x32_f16 computes D[16x16] += A[16x32] B[32x16] per wavefront.  Lane l
// supplies 8 consecutive k values of one row of A (row l % 16, k = 8 (l / 16) + 0..7) and,
// symmetrically, of one column of B (column l % 16).  It receives D[4 (l / 16) + r][l % 16],
// r = 0..3.  A 16 x 32 operand block is therefore 64 lanes x 16 bytes = 1 KiB; storing blocks
// lane-major makes every operand load one fully coalesced 1 KiB wavefront access.
//
// Tiled matrix X[R rows, K cols] ("R-major operand", R padded to 16, K padded to 32):
//   element (r, k) lives at  ((k / 32) * (Rpad / 16) + r / 16) * 512 + (((k % 32) / 8) * 16 + r % 16) * 8 + k % 8
// Weights use the same block but row-tile-major, so that one row tile streams contiguously along K:
//   element (n, k) lives at  ((n / 16) * (Kpad / 32) + k / 32) * 512 + (((k % 32) / 8) * 16 + n % 16) * 8 + k % 8
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mtmc {

typedef uint16_t bf16_t;  // bf16 bit pattern (the caller's weights)
typedef uint16_t h16_t;   // IEEE fp16 bit pattern (MFMA operands: re-tiled weights, activations, KV cache)
typedef __attribute__((ext_vector_type(8))) _Float16 v8h;  // one lane's share of a 16x32 MFMA operand (fp16)
typedef __attribute__((ext_vector_type(2))) _Float16 v2h;
typedef __attribute__((ext_vector_type(4))) float v4f;
typedef __attribute__((ext_vector_type(4))) uint32_t v4u;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }
// fp32 -> fp16, round to nearest even, saturating at the largest finite fp16
__device__ __forceinline__ _Float16 f32_to_h(float f) {
  return (_Float16)fminf(fmaxf(f, -65504.f), 65504.f);
}
__device__ __forceinline__ h16_t f32_to_h16(float f) { return __builtin_bit_cast(h16_t, f32_to_h(f)); }
__device__ __forceinline__ uint32_t pack_h16x2(float lo, float hi) {
  const v2h v = {f32_to_h(lo), f32_to_h(hi)};
  return __builtin_bit_cast(uint32_t, v);
}

// Bit of the library's device error flag that an activation producer raises when a value it stores as fp16 is
// not finite or exceeds the fp16 range (the stored value is then the clamped one, -65504 for a NaN): the results
// of the call are unreliable and the next poll of the flag reports it.
constexpr int kErrFp16Range = 8;
__device__ __forceinline__ bool fits_h16(float f) { return fabsf(f) <= 65504.f; }  // false for NaN
// The converters every activation / KV-cache producer uses: same values as above, and the flag on a clamp.
__device__ __forceinline__ h16_t f32_to_h16_flag(float f, int* err_flag) {
  if (!fits_h16(f)) atomicOr(err_flag, kErrFp16Range);
  return f32_to_h16(f);
}
__device__ __forceinline__ uint32_t pack_h16x2_flag(float lo, float hi, int* err_flag) {
  if (!fits_h16(lo) || !fits_h16(hi)) atomicOr(err_flag, kErrFp16Range);
  return pack_h16x2(lo, hi);
}

// The same for an epilogue that converts many values: the out-of-range test is collected in a per-lane flag that the
// caller raises once at its end (one atomic per kernel part instead of a branch per pair).
__device__ __forceinline__ uint32_t pack_h16x2_track(float lo, float hi, bool& out_of_range) {
  out_of_range |= !fits_h16(lo) | !fits_h16(hi);
  return pack_h16x2(lo, hi);
}

// For values known to lie inside the fp16 range (probabilities in [0, 1]): no clamp.
__device__ __forceinline__ uint32_t pack_h16x2_inrange(float lo, float hi) {
  const v2h v = {(_Float16)lo, (_Float16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

__host__ __device__ __forceinline__ size_t act_off(int r, int k, int Rpad) {
  return ((size_t)(k >> 5) * (Rpad >> 4) + (r >> 4)) * 512 + ((((k & 31) >> 3) << 4) + (r & 15)) * 8 + (k & 7);
}
__host__ __device__ __forceinline__ size_t wgt_off(int n, int k, int Kpad) {
  return ((size_t)(n >> 4) * (Kpad >> 5) + (k >> 5)) * 512 + ((((k & 31) >> 3) << 4) + (n & 15)) * 8 + (k & 7);
}

__device__ __forceinline__ v8h load_frag(const h16_t* tile_base, int lane) {
  const v4u raw = *reinterpret_cast<const v4u*>(tile_base + lane * 8);
  return __builtin_bit_cast(v8h, raw);
}

__device__ __forceinline__ v4f mfma16(v8h a, v8h b, v4f c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

}  // namespace mtmc
