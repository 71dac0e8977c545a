// Skinny bf16 GEMM on the CDNA matrix cores: Y[r][n] = sum_k X[r][k] W[n][k] for a few tens of rows.
//
// At tree sizes (R <= 64 rows) the projection is bound by streaming the weights from HBM once, so
// the kernel is a set of independent, perfectly sequential weight streams:
//   * weights are pre-laid-out (PackW) as MFMA A-operand fragments in the order a wavefront consumes
//     them: 64-feature group -> k step -> 4 feature tiles -> lane.  One k step of a group is 4 KiB
//     of contiguous memory fetched by four fully coalesced 1 KiB loads straight into registers, and
//     consecutive k steps continue the same stream (DRAM-page friendly; measured ~15 % faster than
//     four interleaved 1 KiB streams);
//   * the activations (PackX, B operand) are small (64 rows x K) and live in L2; every wavefront
//     fetches the four 1 KiB row-block fragments of its k step directly, next to the weight loads;
//   * a wavefront owns one feature group (64 features) x 64 rows and walks its own k range with a
//     register ring of RING k steps (no barriers, no LDS in the main loop);
//   * the NW wavefronts of a workgroup split the k range between them and combine their
//     accumulators through LDS in a fixed tree order; blockIdx.y adds a global split-K on top
//     whose slices are written separately and summed in slice order by the consumer kernel
//     (no atomics -> bit-reproducible).
// v_mfma_f32_16x16x32_bf16: A = weights (M = 16 features), B = activations (N = 16 rows),
// C[m][n] lands in lane (n + 16*(m/4)), element m%4: four consecutive features of one row.
#include <algorithm>
#include <cstdio>
#include <cstdlib>

#include "bf16_layout.h"
#include "ded_kernels.h"

namespace ded {

namespace {

constexpr int TN = PACKW_TILES;  // feature tiles per group (fixed by the weight layout)
constexpr int PD = 4;            // k steps (of 32) per group of the k-range split
#ifndef DED_GEMM_RING
#define DED_GEMM_RING 2
#endif
constexpr int RING = DED_GEMM_RING;  // k steps in flight per wavefront (1, 2 or 4)
#ifndef DED_GEMM_MINW
#define DED_GEMM_MINW 2
#endif

#ifdef DED_GEMM_TRACE
__device__ unsigned long long* g_trace = nullptr;  // [wave][4] wall-clock stamps (debug builds only)
#define DED_STAMP(i)                                                                              \
  if (g_trace && lane == 0)                                                                       \
    g_trace[(((size_t)(blockIdx.y * gridDim.x + blockIdx.x)) * NW + wave) * 4 + (i)] = wall_clock64();
#else
#define DED_STAMP(i)
#endif

template <int NW>
__global__ __launch_bounds__(NW * 64, DED_GEMM_MINW) void gemm_stream_kernel(
    float* __restrict__ part, int64_t part_stride, const uint4* __restrict__ xp, const uint4* __restrict__ wp,
    int RB, int N, int KT, int splits, int64_t out_row_stride) {
  __shared__ float4 red[(NW > 1 ? NW / 2 : 1) * TN * 4 * 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ng = blockIdx.x;
  const int split = blockIdx.y;
  const int rb0 = blockIdx.z * 4;
  // this wavefront's k range, in groups of PD steps
  const int groups = KT / PD;
  const int parts = splits * NW;
  const int gi = split * NW + wave;
  const int g_begin = (int)((int64_t)gi * groups / parts);
  const int g_end = (int)((int64_t)(gi + 1) * groups / parts);

  f32x4_t acc[TN][4];
#pragma unroll
  for (int t = 0; t < TN; ++t)
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) acc[t][rb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  DED_STAMP(0)

  if (g_begin < g_end) {
    const uint4* wsrc = wp + (((int64_t)ng * KT * TN) << 6) + lane;
    // per k step the activations of the 4 row blocks x 2 planes (hi, lo) are 8 KiB of contiguous memory
    const uint4* xsrc = xp + ((int64_t)rb0 << 7) + lane;
    const int64_t xstep = (int64_t)RB << 7;

    uint4 wr[RING][TN], xr[RING][8];
    auto issue = [&](int slot, int kt) {
#pragma unroll
      for (int t = 0; t < TN; ++t) wr[slot][t] = wsrc[((int64_t)kt * TN + t) << 6];
#pragma unroll
      for (int i = 0; i < 8; ++i) xr[slot][i] = xsrc[kt * xstep + (i << 6)];
    };
    auto compute = [&](int slot) {
      f16x8_t b[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) b[i] = __builtin_bit_cast(f16x8_t, xr[slot][i]);
#pragma unroll
      for (int plane = 0; plane < 2; ++plane)  // 16 independent accumulators between dependent products
#pragma unroll
        for (int t = 0; t < TN; ++t) {
          f16x8_t a = __builtin_bit_cast(f16x8_t, wr[slot][t]);
#pragma unroll
          for (int rb = 0; rb < 4; ++rb)
            acc[t][rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b[2 * rb + plane], acc[t][rb], 0, 0, 0);
        }
    };

    int kt = g_begin * PD;
    const int kt_last = g_end * PD - RING;  // first step of the last ring-full (range length % RING == 0)
#pragma unroll
    for (int j = 0; j < RING; ++j) issue(j, kt + j);
    for (; kt < kt_last; kt += RING) {
#pragma unroll
      for (int j = 0; j < RING; ++j) {
        compute(j);
        issue(j, kt + RING + j);
      }
    }
#pragma unroll
    for (int j = 0; j < RING; ++j) compute(j);
  }
  DED_STAMP(1)

  // combine the NW k ranges: wave w += wave w + stride, stride = NW/2 .. 1
  if (NW > 1) {
#pragma unroll
    for (int stride = NW / 2; stride >= 1; stride >>= 1) {
      if (wave >= stride && wave < 2 * stride) {
        float4* dst = red + (int64_t)(wave - stride) * TN * 4 * 64 + lane;
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
          for (int rb = 0; rb < 4; ++rb) {
            f32x4_t v = acc[t][rb];
            dst[(t * 4 + rb) * 64] = make_float4(v[0], v[1], v[2], v[3]);
          }
      }
      __syncthreads();
      if (wave < stride) {
        const float4* src = red + (int64_t)wave * TN * 4 * 64 + lane;
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
          for (int rb = 0; rb < 4; ++rb) {
            float4 v = src[(t * 4 + rb) * 64];
            acc[t][rb] += f32x4_t{v.x, v.y, v.z, v.w};
          }
      }
      __syncthreads();
    }
  }

  DED_STAMP(2)
  if (wave == 0) {
    float* out = part + (int64_t)split * part_stride;
    const int row_in = lane & 15, quad = lane >> 4;
#pragma unroll
    for (int t = 0; t < TN; ++t) {
      const int n = (ng * TN + t) * 16 + quad * 4;
      if (n >= N) continue;  // ragged last group (N % 64 != 0): padded features are dropped
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        const int64_t r = (int64_t)(rb0 + rb) * 16 + row_in;
        f32x4_t v = acc[t][rb];
        *reinterpret_cast<float4*>(out + r * out_row_stride + n) = make_float4(v[0], v[1], v[2], v[3]);
      }
    }
  }
  DED_STAMP(3)
}

struct GemmPlan {
  int nw, splits;
};

// Debug knob: DED_GEMM_TUNE="nw,target_wgs" overrides the heuristic (nw in {1,2,4,8}).
struct Tune {
  int nw = 4, target = 384;
  Tune() {
    if (const char* e = getenv("DED_GEMM_TUNE")) {
      int b = 0, c = 0;
      if (sscanf(e, "%d,%d", &b, &c) == 2 && (b == 1 || b == 2 || b == 4 || b == 8) && c > 0) {
        nw = b;
        target = c;
      }
    }
  }
};

GemmPlan make_plan(int rows_pad, int N, int K) {
  static const Tune tune;
  GemmPlan p;
  p.nw = tune.nw;
  const int NG = (N + 16 * TN - 1) / (16 * TN), groups = K / (32 * PD);
  while (p.nw > 1 && p.nw > groups) p.nw /= 2;
  const int base = NG * (rows_pad / 64);
  int s = (tune.target + base - 1) / base;
  s = std::min(s, 8);
  s = std::min(s, std::max(1, groups / p.nw));
  p.splits = std::max(s, 1);
  return p;
}

template <int NW>
void launch(float* part, int64_t part_stride, const uint4* xp, const uint4* wp, int RB, int N, int KT, int splits,
            int64_t out_row_stride, hipStream_t s) {
  dim3 grid((N + 16 * TN - 1) / (16 * TN), splits, RB / 4);
  hipLaunchKernelGGL((gemm_stream_kernel<NW>), grid, dim3(NW * 64), 0, s, part, part_stride, xp, wp, RB, N, KT,
                     splits, out_row_stride);
}

}  // namespace

int bf16_gemm_pick_splits(int rows_pad, int N, int K) { return make_plan(rows_pad, N, K).splits; }

bool bf16_gemm(float* part, int64_t part_stride, const bf16_t* x_packed, const bf16_t* w_packed, int rows_pad,
               int N, int K, int splits, int64_t out_row_stride, hipStream_t s) {
  if (rows_pad <= 0 || rows_pad % 64 || N % 16 || K % (32 * PD) || splits < 1) return false;
  const int RB = rows_pad / 16, KT = K / 32, groups = KT / PD;
  if (splits > groups) return false;
  int nw = make_plan(rows_pad, N, K).nw;
  while (nw > 1 && splits * nw > groups) nw /= 2;  // every wavefront needs at least one group
  const uint4* xp = reinterpret_cast<const uint4*>(x_packed);
  const uint4* wp = reinterpret_cast<const uint4*>(w_packed);
  switch (nw) {
    case 8: launch<8>(part, part_stride, xp, wp, RB, N, KT, splits, out_row_stride, s); break;
    case 4: launch<4>(part, part_stride, xp, wp, RB, N, KT, splits, out_row_stride, s); break;
    case 2: launch<2>(part, part_stride, xp, wp, RB, N, KT, splits, out_row_stride, s); break;
    default: launch<1>(part, part_stride, xp, wp, RB, N, KT, splits, out_row_stride, s); break;
  }
  return true;
}

}  // namespace ded
