// Skinny bf16 GEMM on the CDNA matrix cores: Y[r][n] = sum_k X[r][k] W[n][k] for a few tens of rows.
//
// At tree sizes (R <= 64 rows) the projection is bound by streaming the weights from HBM once, so
// the kernel is organised around that stream:
//   * weights are pre-laid-out as MFMA A-operand fragments (PackW): a wavefront fetches one
//     16-feature x 32-k fragment with a single fully coalesced 1 KiB load, straight into registers;
//   * the activations (PackX, the B operand) are small and shared by every workgroup: each
//     workgroup stages a 64-row x 128-k chunk through LDS, double buffered;
//   * a workgroup = 4 wavefronts x TN feature tiles; the k range can be split over blockIdx.y
//     (split-K) to fill 256 CUs; slices are written separately and summed in a fixed order by the
//     consumer kernel (no atomics -> deterministic).
// v_mfma_f32_16x16x32_bf16: A = weights (M = 16 features), B = activations (N = 16 rows),
// C[m][n] lands in lane (n + 16*(m/4)), element m%4: four consecutive features of one row.
#include <algorithm>

#include "bf16_layout.h"
#include "ded_kernels.h"

namespace ded {

namespace {

constexpr int KCH = 4;  // k fragments (of 32) per chunk -> 128 k per chunk

template <int TN>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(float* __restrict__ part, int64_t part_stride,
                                                          const uint4* __restrict__ xp, const uint4* __restrict__ wp,
                                                          int RB, int NT, int KT, int n_chunks, int splits,
                                                          int64_t out_row_stride) {
  __shared__ uint4 lds[2][KCH * 4 * 64];  // [buffer][k fragment][row block][lane], 2 x 16 KiB
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nt0 = (blockIdx.x * 4 + wave) * TN;
  const int split = blockIdx.y;
  const int rb0 = blockIdx.z * 4;
  const int c_begin = (int)((int64_t)split * n_chunks / splits);
  const int c_end = (int)((int64_t)(split + 1) * n_chunks / splits);

  f32x4_t acc[TN][4];
#pragma unroll
  for (int t = 0; t < TN; ++t)
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) acc[t][rb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  uint4 a0[TN][KCH], a1[TN][KCH];  // weight fragments of the current / next chunk
  uint4 xr[KCH];                   // activation chunk in flight to LDS

  auto load_a = [&](uint4(&a)[TN][KCH], int c) {
#pragma unroll
    for (int t = 0; t < TN; ++t) {
      const bool ok = nt0 + t < NT;
      const uint4* src = wp + (((int64_t)(nt0 + t) * KT + (int64_t)c * KCH) << 6) + lane;
#pragma unroll
      for (int k = 0; k < KCH; ++k) a[t][k] = ok ? src[k << 6] : make_uint4(0, 0, 0, 0);
    }
  };
  auto load_x = [&](int c) {
#pragma unroll
    for (int k = 0; k < KCH; ++k) xr[k] = xp[((((int64_t)c * KCH + k) * RB + rb0) << 6) + tid];
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int k = 0; k < KCH; ++k) lds[buf][k * 256 + tid] = xr[k];
  };
  auto compute = [&](const uint4(&a)[TN][KCH], int buf) {
#pragma unroll
    for (int k = 0; k < KCH; ++k) {
      bf16x8_t b[4];
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) b[rb] = __builtin_bit_cast(bf16x8_t, lds[buf][k * 256 + rb * 64 + lane]);
#pragma unroll
      for (int t = 0; t < TN; ++t) {
        bf16x8_t av = __builtin_bit_cast(bf16x8_t, a[t][k]);
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
          acc[t][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, b[rb], acc[t][rb], 0, 0, 0);
      }
    }
  };

  if (c_begin < c_end) {
    load_a(a0, c_begin);
    load_x(c_begin);
    store_x(0);
    __syncthreads();
    int c = c_begin;
    while (true) {
      // even step: current = a0 / lds[0], next = a1 / lds[1]
      bool more = c + 1 < c_end;
      if (more) {
        load_a(a1, c + 1);
        load_x(c + 1);
      }
      compute(a0, 0);
      if (!more) break;
      store_x(1);
      __syncthreads();
      ++c;
      // odd step: current = a1 / lds[1], next = a0 / lds[0]
      more = c + 1 < c_end;
      if (more) {
        load_a(a0, c + 1);
        load_x(c + 1);
      }
      compute(a1, 1);
      if (!more) break;
      store_x(0);
      __syncthreads();
      ++c;
    }
  }

  float* out = part + (int64_t)split * part_stride;
  const int row_in = lane & 15, quad = lane >> 4;
#pragma unroll
  for (int t = 0; t < TN; ++t) {
    if (nt0 + t >= NT) continue;
    const int n = (nt0 + t) * 16 + quad * 4;
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) {
      const int64_t r = (int64_t)(rb0 + rb) * 16 + row_in;
      f32x4_t v = acc[t][rb];
      *reinterpret_cast<float4*>(out + r * out_row_stride + n) = make_float4(v[0], v[1], v[2], v[3]);
    }
  }
}

inline int feature_tiles_per_wave(int rows_pad, int N) {
  // two feature tiles per wavefront halve the activation re-reads; use them once the grid is wide enough
  int NT = N / 16;
  int gx2 = (NT + 7) / 8;
  return gx2 * (rows_pad / 64) >= 256 ? 2 : 1;
}

}  // namespace

int bf16_gemm_pick_splits(int rows_pad, int N, int K) {
  int TN = feature_tiles_per_wave(rows_pad, N);
  int NT = N / 16;
  int base = ((NT + 4 * TN - 1) / (4 * TN)) * (rows_pad / 64);
  int chunks = K / (32 * KCH);
  int s = std::max(1, 512 / std::max(base, 1));
  s = std::min(s, 8);
  s = std::min(s, std::max(1, chunks / 2));
  return s;
}

void bf16_gemm(float* part, int64_t part_stride, const bf16_t* x_packed, const bf16_t* w_packed, int rows_pad,
               int N, int K, int splits, int64_t out_row_stride, hipStream_t s) {
  if (rows_pad <= 0 || rows_pad % 64 || N % 16 || K % (32 * KCH) || splits < 1) return;
  const int RB = rows_pad / 16, NT = N / 16, KT = K / 32, chunks = KT / KCH;
  if (splits > chunks) splits = chunks;
  const int TN = feature_tiles_per_wave(rows_pad, N);
  dim3 grid((NT + 4 * TN - 1) / (4 * TN), splits, RB / 4);
  const uint4* xp = reinterpret_cast<const uint4*>(x_packed);
  const uint4* wp = reinterpret_cast<const uint4*>(w_packed);
  if (TN == 2)
    hipLaunchKernelGGL(gemm_skinny_kernel<2>, grid, dim3(256), 0, s, part, part_stride, xp, wp, RB, NT, KT, chunks,
                       splits, out_row_stride);
  else
    hipLaunchKernelGGL(gemm_skinny_kernel<1>, grid, dim3(256), 0, s, part, part_stride, xp, wp, RB, NT, KT, chunks,
                       splits, out_row_stride);
}

}  // namespace ded
