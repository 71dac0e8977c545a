// Skinny 16-bit GEMM on the CDNA matrix cores: Y[r][n] = sum_k X[r][k] W[n][k] for a few tens of rows.
//
// At tree sizes (R <= 64 rows) the projection is bound by streaming the weights from HBM once.  What
// was measured on MI355X and shaped these kernels:
//   * plain 16-byte-per-lane streaming tops out near 6.2 TB/s for the chip and near 52 GB/s per CU,
//     so every CU has to stream its equal share (~24 GB/s) for the whole kernel, and whatever else a
//     CU loads (the activations) comes out of the same per-CU budget, even when it hits in L2;
//   * a wavefront that reads one contiguous stream is ~15 % faster than one that interleaves four.
// Hence:
//   * weights are pre-laid-out (PackW, f16) as MFMA A-operand fragments in the order a wavefront
//     consumes them: 64-feature group -> k step -> 4 feature tiles -> lane; one k step of a group is
//     4 KiB of contiguous memory fetched by four coalesced 1 KiB loads straight into registers;
//   * activations (PackX, B operand, hi/lo f16 planes) are shared: in the "wide" kernel the NWN
//     wavefronts of a workgroup own NWN neighbouring feature groups over the same k range and the
//     activation chunks go through LDS once per workgroup (double buffered, one barrier per chunk);
//   * narrow outputs (few feature groups) use the "stream" kernel instead: one feature group per
//     workgroup, the NW wavefronts split the k range and combine through LDS in a fixed tree order;
//   * blockIdx.y is a global split-K whose slices are written separately and summed in slice order
//     by the consumer kernel (no atomics -> bit-reproducible); the planner picks the shape whose
//     workgroup count fills the 256 CUs most evenly with the least extra traffic.
// v_mfma_f32_16x16x32_f16: A = weights (M = 16 features), B = activations (N = 16 rows),
// C[m][n] lands in lane (n + 16*(m/4)), element m%4: four consecutive features of one row.
// X = hi + lo (two planes): both products accumulate into the same fp32 registers.
#include <algorithm>
#include <cstdio>
#include <cstdlib>

#include "bf16_layout.h"
#include "ded_kernels.h"

namespace ded {

namespace {

constexpr int TN = PACKW_TILES;  // feature tiles per group (fixed by the weight layout)
constexpr int PD = 4;            // k steps (of 32) per group of the k-range split
constexpr int RING = 2;          // k steps in flight per wavefront (stream kernel)

#ifdef DED_GEMM_TRACE
__device__ unsigned long long* g_trace = nullptr;  // [workgroup][wave][4] wall-clock stamps (debug builds only)
#define DED_STAMP(i)                                                                                       \
  if (g_trace && (threadIdx.x & 63) == 0)                                                                  \
    g_trace[((((size_t)blockIdx.y * gridDim.x + blockIdx.x) * (blockDim.x >> 6)) + (threadIdx.x >> 6)) * 4 + (i)] = \
        wall_clock64();
#else
#define DED_STAMP(i)
#endif

__device__ inline void store_tile(float* out, int64_t out_row_stride, int ng, int N, int rb0, int lane,
                                  const f32x4_t (&acc)[TN][4]) {
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

// ------------------------------------------------------------------------------------------
// Stream kernel: one feature group per workgroup, NW wavefronts split the k range.
// ------------------------------------------------------------------------------------------
template <int NW, int PLANES>
__global__ __launch_bounds__(NW * 64, 2) void gemm_stream_kernel(float* __restrict__ part, int64_t part_stride,
                                                                 const uint4* __restrict__ xp,
                                                                 const uint4* __restrict__ wp, int RB, int N, int KT,
                                                                 int splits, int64_t out_row_stride) {
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

  if (g_begin < g_end) {
    const uint4* wsrc = wp + (((int64_t)ng * KT * TN) << 6) + lane;
    // per k step the activations of the 4 row blocks x 2 planes (hi, lo) are 8 KiB of contiguous memory
    const uint4* xsrc = xp + ((int64_t)rb0 << 7) + lane;
    const int64_t xstep = (int64_t)RB << 7;

    uint4 wr[RING][TN], xr[RING][4 * PLANES];
    auto issue = [&](int slot, int kt) {
#pragma unroll
      for (int t = 0; t < TN; ++t) wr[slot][t] = wsrc[((int64_t)kt * TN + t) << 6];
#pragma unroll
      for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int p = 0; p < PLANES; ++p) xr[slot][rb * PLANES + p] = xsrc[kt * xstep + ((rb * 2 + p) << 6)];
    };
    auto compute = [&](int slot) {
#pragma unroll
      for (int p = 0; p < PLANES; ++p)  // 16 independent accumulators between dependent products
#pragma unroll
        for (int t = 0; t < TN; ++t) {
          f16x8_t a = __builtin_bit_cast(f16x8_t, wr[slot][t]);
#pragma unroll
          for (int rb = 0; rb < 4; ++rb)
            acc[t][rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                a, __builtin_bit_cast(f16x8_t, xr[slot][rb * PLANES + p]), acc[t][rb], 0, 0, 0);
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
  if (wave == 0) store_tile(part + (int64_t)split * part_stride, out_row_stride, ng, N, rb0, lane, acc);
}

// ------------------------------------------------------------------------------------------
// Wide kernel: a workgroup owns NWN neighbouring feature groups over one k range.  Its 2 x NWN
// wavefronts form two halves: half h walks the h-th half of the k range, wavefront wn of a half owns
// feature group wn.  The activation chunks (CH k steps x 4 row blocks x PLANES) of each half are
// staged through LDS once per half (double buffered, one barrier per chunk), so the activations cost
// 1/NWN of what they would if every wavefront fetched its own.  Two wavefronts per SIMD overlap each
// other's LDS waits and barriers; the halves are added through LDS at the end (fixed order).
// ------------------------------------------------------------------------------------------
template <int NWN, int PLANES>
__global__ __launch_bounds__(NWN * 128, 2) void gemm_wide_kernel(float* __restrict__ part, int64_t part_stride,
                                                                 const uint4* __restrict__ xp,
                                                                 const uint4* __restrict__ wp, int RB, int N, int KT,
                                                                 int splits, int64_t out_row_stride) {
  constexpr int TH = NWN * 64;                    // threads per half
  constexpr int CH = (NWN == 4 || PLANES == 1) ? 2 : 1;  // k steps per activation chunk (<= 4 staged units / thread)
  constexpr int STEP_U4 = 4 * PLANES * 64;        // uint4 units of activations per k step
  constexpr int CHUNK_U4 = CH * STEP_U4;
  constexpr int PER_THREAD = (CHUNK_U4 + TH - 1) / TH;
  constexpr int ACC_U4 = TN * 4 * 64;             // float4 units of one wavefront's accumulators
  constexpr int LDS_U4 = (2 * 2 * CHUNK_U4 > NWN * ACC_U4) ? 2 * 2 * CHUNK_U4 : NWN * ACC_U4;
  __shared__ uint4 lds[LDS_U4];                   // [half][buffer][chunk]; reused for the final reduction
  const int half = threadIdx.x / TH;
  const int tid = threadIdx.x - half * TH, lane = tid & 63, wn = tid >> 6;
  uint4* xs = lds + half * 2 * CHUNK_U4;
  const int NG = (N + 16 * TN - 1) / (16 * TN);
  const int ng_raw = blockIdx.x * NWN + wn;
  const int ng = ng_raw < NG ? ng_raw : NG - 1;  // surplus wavefront of the last tile: valid reads, no store
  const int split = blockIdx.y;
  const int rb0 = blockIdx.z * 4;
  const int groups = KT / PD;
  const int g_begin = (int)((int64_t)split * groups / splits);
  const int g_end = (int)((int64_t)(split + 1) * groups / splits);
  const int n_chunks = (g_end - g_begin) * (PD / CH) / 2;  // per half; the range holds an even number of chunks
  const int kt0 = g_begin * PD + half * n_chunks * CH;

  f32x4_t acc[TN][4];
#pragma unroll
  for (int t = 0; t < TN; ++t)
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) acc[t][rb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const uint4* wsrc = wp + (((int64_t)ng * KT * TN) << 6) + lane;
  const uint4* xsrc = xp + ((int64_t)rb0 << 7);
  const int64_t xstep = (int64_t)RB << 7;

  struct WChunk {
    uint4 f[CH][TN];
  };
  struct XStage {
    uint4 u[PER_THREAD];
  };
  auto load_w = [&](int c) {
    WChunk w;
#pragma unroll
    for (int s = 0; s < CH; ++s)
#pragma unroll
      for (int t = 0; t < TN; ++t) w.f[s][t] = wsrc[((int64_t)(kt0 + c * CH + s) * TN + t) << 6];
    return w;
  };
  // unit u of a chunk: step s = u / STEP_U4, inside the step (rb, plane, lane) in memory order
  auto load_x = [&](int c) {
    XStage x;
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      int u = tid + i * TH;
      if (CHUNK_U4 % TH == 0 || u < CHUNK_U4) {
        int s = u / STEP_U4, v = u - s * STEP_U4;
        int src = PLANES == 2 ? v : ((v >> 6) * 128 + (v & 63));  // one plane: skip the lo fragments
        x.u[i] = xsrc[(int64_t)(kt0 + c * CH + s) * xstep + src];
      }
    }
    return x;
  };
  auto store_x = [&](int buf, const XStage& x) {
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      int u = tid + i * TH;
      if (CHUNK_U4 % TH == 0 || u < CHUNK_U4) xs[buf * CHUNK_U4 + u] = x.u[i];
    }
  };
  auto compute = [&](const WChunk& w, int buf) {
#pragma unroll
    for (int s = 0; s < CH; ++s) {
      f16x8_t b[4 * PLANES];
#pragma unroll
      for (int i = 0; i < 4 * PLANES; ++i)
        b[i] = __builtin_bit_cast(f16x8_t, xs[buf * CHUNK_U4 + s * STEP_U4 + (i << 6) + lane]);
#pragma unroll
      for (int p = 0; p < PLANES; ++p)
#pragma unroll
        for (int t = 0; t < TN; ++t) {
          f16x8_t a = __builtin_bit_cast(f16x8_t, w.f[s][t]);
#pragma unroll
          for (int rb = 0; rb < 4; ++rb)
            acc[t][rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b[rb * PLANES + p], acc[t][rb], 0, 0, 0);
        }
    }
  };

  DED_STAMP(0)
  // Weight chunks are fetched two chunks ahead (three register buffers, rotated), activation chunks one
  // ahead (LDS double buffer).  In every iteration the activation loads are issued BEFORE the weight loads
  // of the farther chunk, so that waiting for them (loads retire in order) leaves the weight loads in flight.
  // Both halves run the same number of iterations, hence the same number of barriers (n_chunks >= 2).
  WChunk w0 = load_w(0);
  store_x(0, load_x(0));
  WChunk w1 = load_w(1);
  __syncthreads();
  DED_STAMP(1)
  int buf = 0;
  for (int c = 0; c + 2 < n_chunks; ++c) {
    XStage xn = load_x(c + 1);
    WChunk w2 = load_w(c + 2);
    compute(w0, buf);
    store_x(buf ^ 1, xn);
    __syncthreads();
    w0 = w1;
    w1 = w2;
    buf ^= 1;
  }
  {  // last two chunks: nothing left to prefetch
    XStage xn = load_x(n_chunks - 1);
    compute(w0, buf);
    store_x(buf ^ 1, xn);
    __syncthreads();
    compute(w1, buf ^ 1);
  }
  DED_STAMP(2)
  // second half -> LDS -> first half adds and stores
  __syncthreads();
  float4* red = reinterpret_cast<float4*>(lds) + wn * ACC_U4 + lane;
  if (half == 1) {
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        f32x4_t v = acc[t][rb];
        red[(t * 4 + rb) * 64] = make_float4(v[0], v[1], v[2], v[3]);
      }
  }
  __syncthreads();
  if (half == 0) {
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        float4 v = red[(t * 4 + rb) * 64];
        acc[t][rb] += f32x4_t{v.x, v.y, v.z, v.w};
      }
    if (ng_raw < NG) store_tile(part + (int64_t)split * part_stride, out_row_stride, ng, N, rb0, lane, acc);
  }
  DED_STAMP(3)
}

// Debug knob: DED_GEMM_TUNE="nwn,splits" forces the kernel shape (nwn 0 = stream kernel).
struct Tune {
  int nwn = -1, splits = 0;
  Tune() {
    if (const char* e = getenv("DED_GEMM_TUNE")) {
      int a = -1, b = 0;
      if (sscanf(e, "%d,%d", &a, &b) == 2 && a >= 0 && a <= 4 && b >= 1) {
        nwn = a;
        splits = b;
      }
    }
  }
};

constexpr int kCUs = 256;

// relative cost of a shape: weight stream slowed down by activation reloads and uneven CU filling,
// plus the split-K slices that are written here and read back by the consumer
double shape_cost(int64_t w_bytes, int64_t slice_bytes, int wgs, double x_per_w, int splits) {
  int rounds = (wgs + kCUs - 1) / kCUs;
  double eff = (double)wgs / (double)(rounds * kCUs);
  double stream = (double)w_bytes * (1.0 + 0.35 * x_per_w) / eff;
  return stream + 2.0 * (double)slice_bytes * (splits > 1 ? splits : 0);
}

}  // namespace

GemmPlan bf16_gemm_plan(int rows_pad, int N, int K, int planes, int max_splits) {
  static const Tune tune;
  const int NG = (N + 16 * TN - 1) / (16 * TN), groups = K / (32 * PD), rg = rows_pad / 64;
  const int64_t w_bytes = (int64_t)NG * 64 * K * 2, slice = (int64_t)rows_pad * N * 4;
  GemmPlan best{0, 4, 1};
  double best_cost = 1e300;
  for (int nwn = 0; nwn <= 4; ++nwn) {
    if (tune.nwn >= 0 && nwn != tune.nwn) continue;
    if (nwn == 1) continue;  // a 1-wide tile is the stream kernel
    for (int s = 1; s <= 8 && s <= groups && s <= max_splits; ++s) {
      if (tune.nwn >= 0 && max_splits > 1 && s != std::min(tune.splits, groups)) continue;
      GemmPlan p{nwn, 1, s};
      double x_per_w;
      int wgs;
      if (nwn == 0) {
        p.nw = 4;
        while (p.nw > 1 && s * p.nw > groups) p.nw /= 2;
        wgs = NG * s * rg;
        x_per_w = planes;  // every wavefront reloads its own activations: 64 rows per 64 features
      } else {
        if (groups / s < 2) continue;  // each half needs at least two chunks
        wgs = ((NG + nwn - 1) / nwn) * s * rg;
        x_per_w = (double)planes / nwn;
      }
      double c = shape_cost(w_bytes, slice, wgs, x_per_w, s);
      if (c < best_cost) {
        best_cost = c;
        best = p;
      }
    }
  }
  return best;
}

bool bf16_gemm(float* part, int64_t part_stride, const bf16_t* x_packed, const bf16_t* w_packed, int rows_pad,
               int N, int K, int planes, const GemmPlan& plan, int64_t out_row_stride, hipStream_t s) {
  if (rows_pad <= 0 || rows_pad % 64 || N % 16 || K % (32 * PD) || (planes != 1 && planes != 2)) return false;
  const int RB = rows_pad / 16, KT = K / 32, groups = KT / PD;
  const int NG = (N + 16 * TN - 1) / (16 * TN);
  const int splits = plan.splits;
  if (splits < 1 || splits > groups) return false;
  const uint4* xp = reinterpret_cast<const uint4*>(x_packed);
  const uint4* wp = reinterpret_cast<const uint4*>(w_packed);
#define DED_LAUNCH_T(KERNEL, A, B, GX, THREADS)                                                            \
  hipLaunchKernelGGL((KERNEL<A, B>), dim3(GX, splits, RB / 4), dim3(THREADS), 0, s, part, part_stride, xp, \
                     wp, RB, N, KT, splits, out_row_stride)
#define DED_LAUNCH(KERNEL, A, B, GX) DED_LAUNCH_T(KERNEL, A, B, GX, A * 64)
#define DED_LAUNCH_W(A, B, GX) DED_LAUNCH_T(gemm_wide_kernel, A, B, GX, A * 128)
  if (plan.nwn == 0) {
    int nw = plan.nw >= 4 ? 4 : plan.nw >= 2 ? 2 : 1;
    while (nw > 1 && splits * nw > groups) nw /= 2;  // every wavefront needs at least one k group
    if (planes == 2) {
      if (nw == 4) DED_LAUNCH(gemm_stream_kernel, 4, 2, NG);
      else if (nw == 2) DED_LAUNCH(gemm_stream_kernel, 2, 2, NG);
      else DED_LAUNCH(gemm_stream_kernel, 1, 2, NG);
    } else {
      if (nw == 4) DED_LAUNCH(gemm_stream_kernel, 4, 1, NG);
      else if (nw == 2) DED_LAUNCH(gemm_stream_kernel, 2, 1, NG);
      else DED_LAUNCH(gemm_stream_kernel, 1, 1, NG);
    }
    return true;
  }
  if (groups / splits < 2) return false;
  const int gx = (NG + plan.nwn - 1) / plan.nwn;
  if (planes == 2) {
    if (plan.nwn == 4) DED_LAUNCH_W(4, 2, gx);
    else if (plan.nwn == 3) DED_LAUNCH_W(3, 2, gx);
    else if (plan.nwn == 2) DED_LAUNCH_W(2, 2, gx);
    else return false;
  } else {
    if (plan.nwn == 4) DED_LAUNCH_W(4, 1, gx);
    else if (plan.nwn == 3) DED_LAUNCH_W(3, 1, gx);
    else if (plan.nwn == 2) DED_LAUNCH_W(2, 1, gx);
    else return false;
  }
#undef DED_LAUNCH
#undef DED_LAUNCH_W
#undef DED_LAUNCH_T
  return true;
}

}  // namespace ded
