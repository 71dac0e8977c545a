// Index functions of the matrix-core operand layouts used by the bf16 path (units: bf16 elements).
// A fragment is what one v_mfma_f32_16x16x32_bf16 operand holds: 64 lanes x 8 consecutive elements
// of the contraction index; lane = (contraction_group << 4) | row_in_tile.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ded {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// Weights: 64-feature group -> k step -> 4 feature tiles -> lane: the order a GEMM wavefront reads them,
// so that every wavefront walks one contiguous stream.  Feature counts are padded to a multiple of 64.
constexpr int PACKW_TILES = 4;
__host__ __device__ inline int64_t packw_index(int n, int k, int K) {
  int lane = (((k & 31) >> 3) << 4) | (n & 15);
  int64_t frag = ((int64_t)(n >> 6) * (K >> 5) + (k >> 5)) * PACKW_TILES + ((n >> 4) & 3);
  return ((frag << 6) + lane) * 8 + (k & 7);
}
__host__ __device__ inline int64_t packx_index(int r, int k, int RB) {
  int lane = (((k & 31) >> 3) << 4) | (r & 15);
  return ((((int64_t)(k >> 5) * RB + (r >> 4)) << 6) + lane) * 8 + (k & 7);
}
// inside one (sequence, kv head) block of PackQ: virtual row vr, head dim 128
__host__ __device__ inline int64_t packq_index(int vr, int hdim) {
  int lane = (((hdim & 31) >> 3) << 4) | (vr & 15);
  return ((((int64_t)(vr >> 4) * 4 + (hdim >> 5)) << 6) + lane) * 8 + (hdim & 7);
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
__device__ inline uint32_t pack2_bf16(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

}  // namespace ded
