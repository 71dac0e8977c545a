// Operand layouts and number formats of the 16-bit path (config dtype DED_BF16).
//
// Number formats.  Weights arrive as bf16 and the K/V cache holds 2-byte elements, as the configuration
// says; but every matrix-core operand is IEEE half (f16, 11-bit significand), not bf16 (8-bit):
//   * bf16 weights and injected bf16 K/V are widened to f16 once (exact for |x| >= 2^-14; smaller
//     magnitudes land on the f16 subnormal grid, absolute error <= 2^-25);
//   * K/V computed by the model are stored as f16;
//   * GEMM inputs (normalised activations, attention output, SwiGLU product) and the attention queries
//     are kept as a pair hi + lo of f16 values (hi = f16(x), lo = f16(x - hi)), i.e. ~22 significant
//     bits, and the products W.hi + W.lo / K.q_hi + K.q_lo are both accumulated in fp32.
// With bf16 activations the logits of a 7B-shape model are off by up to 6e-2 after 2 layers and
// 2e-1 after 16 (fp64 emulation of the rounding points); this scheme stays below 2e-2 at 32 layers
// at the cost of extra matrix-core work only - the path is bound by weight / cache bytes, which do not change.
//
// A fragment is what one v_mfma_f32_16x16x32_f16 operand holds: 64 lanes x 8 consecutive elements of
// the contraction index; lane = (contraction_group << 4) | row_in_tile.  Units below: 2-byte elements.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ded {

typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// Weights: 64-feature group -> k step -> 4 feature tiles -> lane: the order a GEMM wavefront reads them,
// so that every wavefront walks one contiguous stream.  Feature counts are padded to a multiple of 64.
constexpr int PACKW_TILES = 4;
__host__ __device__ inline int64_t packw_index(int n, int k, int K) {
  int lane = (((k & 31) >> 3) << 4) | (n & 15);
  int64_t frag = ((int64_t)(n >> 6) * (K >> 5) + (k >> 5)) * PACKW_TILES + ((n >> 4) & 3);
  return ((frag << 6) + lane) * 8 + (k & 7);
}
// GEMM inputs X[R][K]: k step -> 16-row block -> plane (0 = hi, 1 = lo) -> lane
__host__ __device__ inline int64_t packx_index(int r, int k, int RB, int plane) {
  int lane = (((k & 31) >> 3) << 4) | (r & 15);
  int64_t frag = (((int64_t)(k >> 5) * RB + (r >> 4)) << 1) + plane;
  return ((frag << 6) + lane) * 8 + (k & 7);
}
// inside one (sequence, kv head) block of PackQ: virtual row vr, head dim 128, plane hi / lo
__host__ __device__ inline int64_t packq_index(int vr, int hdim, int plane) {
  int lane = (((hdim & 31) >> 3) << 4) | (vr & 15);
  int64_t frag = ((((int64_t)(vr >> 4) << 2) + (hdim >> 5)) << 1) + plane;
  return ((frag << 6) + lane) * 8 + (hdim & 7);
}
// inside one (sequence, kv head) block of the key cache
__host__ __device__ inline int64_t packk_index(int key, int hdim) {
  int kl = key & 31;
  int m = ((kl >> 3) << 2) | (kl & 3);  // tile row: the two 16-row tiles of a 32-key group interleave
  int c = (kl >> 2) & 1;                // so that one lane ends up with 8 consecutive keys
  int lane = (((hdim & 31) >> 3) << 4) | m;
  int64_t frag = ((int64_t)(key >> 5) * 2 + c) * 4 + (hdim >> 5);
  return ((frag << 6) + lane) * 8 + (hdim & 7);
}
// inside one (sequence, kv head) block of the transposed value cache
__host__ __device__ inline int64_t packvt_index(int key, int hdim) {
  int kl = key & 31;
  int lane = ((kl >> 3) << 4) | (hdim & 15);
  int64_t frag = (int64_t)(key >> 5) * 8 + (hdim >> 4);
  return ((frag << 6) + lane) * 8 + (kl & 7);
}

__device__ inline uint16_t f32_to_bf16(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ inline uint16_t f32_to_f16(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }  // RNE
__device__ inline float f16_to_f32(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
__device__ inline uint16_t bf16_to_f16(uint16_t b) { return f32_to_f16(bf16_to_f32(b)); }
// x ~= hi + lo with hi = f16(x), lo = f16(x - hi)
__device__ inline void split_f16(float x, uint16_t& hi, uint16_t& lo) {
  _Float16 h = (_Float16)x;
  hi = __builtin_bit_cast(uint16_t, h);
  lo = __builtin_bit_cast(uint16_t, (_Float16)(x - (float)h));
}

}  // namespace ded
