// Shared device-side helpers for the rlgen kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16_t;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define WAVE 64

// GEMM operands (weights and fp16 activations) are stored "K-block major": a matrix X[rows, K] is laid out
// as [ceil(K / 64)][rows][64], so the 64 K-values of a row are 128 contiguous bytes and the tile a GEMM block
// stages (BM rows x 64) is one contiguous run.  A wave-wide 16-byte-per-lane load then reads one contiguous
// kilobyte, which the texture path of gfx950 serves about twice as fast as eight separate 128-byte row
// pieces (measured: 34 vs 16 bytes/clk/CU from L2 at 4 waves per CU).
__host__ __device__ __forceinline__ size_t kblk_off(int row, int col, int rows) {
  return ((size_t)(col >> 6) * rows + row) * 64 + (col & 63);
}
__host__ __device__ __forceinline__ size_t kblk_elems(size_t rows, size_t K) { return ((K + 63) / 64) * rows * 64; }

// fp32 -> bf16, round to nearest even (finite inputs; NaN stays NaN).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
}

// Sticky device-detected input faults (bit flags in ctx->status word).
#define RLGEN_FAULT_TOKEN   1u
#define RLGEN_FAULT_UNIFORM 2u
#define RLGEN_FAULT_GROUP   4u      // sequences declared to share a prefix (rlgen_set_score_groups) do not
#define RLGEN_FAULT_RANGE   8u      // an activation exceeded the largest finite fp16 value and was clamped

// A value held as the sum of two bf16 numbers, hi = bf16(f) and lo = bf16(f - hi): 16 significant bits with bf16's
// exponent range (the operand format of the library's precise mode).  f - hi is exact in fp32.
__device__ __forceinline__ void split_bf16(float f, uint16_t& hi, uint16_t& lo) {
  hi = f32_to_bf16_bits(f);
  lo = f32_to_bf16_bits(f - bf16_bits_to_f32(hi));
}
// the same for two values, packed for 32-bit stores: returns (hi, lo) with hi = (bf16 a, bf16 b) and lo likewise
__device__ __forceinline__ u32x2 split_bf16x2(float a, float b) {
  uint16_t ah, al, bh, bl;
  split_bf16(a, ah, al);
  split_bf16(b, bh, bl);
  u32x2 r;
  r[0] = (uint32_t)ah | ((uint32_t)bh << 16);
  r[1] = (uint32_t)al | ((uint32_t)bl << 16);
  return r;
}
#define SPLIT_BF16X2(a, b, hi, lo) do { const u32x2 t_ = split_bf16x2(a, b); (hi) = t_[0]; (lo) = t_[1]; } while (0)

// fp32 -> fp16, round to nearest even, saturating at the largest finite fp16.
__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) {
  const f16_t h = (f16_t)fminf(fmaxf(f, -65504.f), 65504.f);
  return __builtin_bit_cast(uint16_t, h);
}
// Would f32_to_f16_bits clamp this value?  (65520 is the first value that rounds beyond 65504; NaN counts.)
__device__ __forceinline__ bool f16_out_of_range(float f) { return !(fabsf(f) < 65520.f); }
// Raises the sticky fp16-range flag if this lane saw a value the fp16 conversion clamped (rare: one atomic per such lane).
__device__ __forceinline__ void flag_f16_range(bool sat, unsigned* status) {
  if (sat && status != nullptr) atomicOr(status, RLGEN_FAULT_RANGE);
}
__device__ __forceinline__ float f16_bits_to_f32(uint16_t b) { return (float)__builtin_bit_cast(f16_t, b); }
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
  return (uint32_t)f32_to_f16_bits(lo) | ((uint32_t)f32_to_f16_bits(hi) << 16);
}
// Eight bf16 values (as loaded from the KV cache) to fp16.  Every bf16 value whose magnitude lies in
// fp16's normal range converts exactly (8 significant bits fit in 11); larger finite values saturate.
__device__ __forceinline__ f16x8 bf16x8_to_f16x8(u32x4 v) {
  typedef __fp16 h2 __attribute__((ext_vector_type(2)));
  f16x8 r;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const h2 h = __builtin_amdgcn_cvt_pkrtz(__uint_as_float(v[e] << 16), __uint_as_float(v[e] & 0xffff0000u));
    r[2 * e] = (f16_t)h[0];
    r[2 * e + 1] = (f16_t)h[1];
  }
  return r;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}
