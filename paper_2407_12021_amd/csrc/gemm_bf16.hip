// Skinny 16-bit GEMM on the CDNA matrix cores with fused epilogues:
//   Y[r][n] = sum_k X[r][k] W[n][k] for a few tens of rows, followed in the same kernel by what the
//   decoder does with Y (rotary embedding + cache append, SiLU*up, residual add + next input, logits).
//
// At tree sizes (R <= 64 rows) the projection is bound by streaming the weights from HBM once.  What
// was measured on MI355X and shaped these kernels:
//   * plain 16-byte-per-lane streaming tops out near 6.2 TB/s for the chip and near 52 GB/s per CU,
//     so every CU has to stream its equal share (~24 GB/s) for the whole kernel, and whatever else a
//     CU loads (the activations) comes out of the same per-CU budget, even when it hits in L2;
//   * a wavefront that reads one contiguous stream is ~15 % faster than one that interleaves four;
//   * every launch costs ~3.5 us even back-to-back, and a small dependent kernel 6-10 us, which is
//     why the split-K reduction and the element-wise stages live in the GEMM's epilogue.
// Hence:
//   * weights are pre-laid-out (PackW, f16) as MFMA A-operand fragments in the order a wavefront
//     consumes them: 64-feature group -> k step -> 4 feature tiles -> lane; one k step of a group is
//     4 KiB of contiguous memory fetched by four coalesced 1 KiB loads straight into registers;
//   * activations (PackX, B operand, hi/lo f16 planes) are shared: in the "wide" kernel the NWN
//     wavefronts of a half-workgroup own NWN neighbouring feature groups over the same k range and
//     the activation chunks go through LDS once (double buffered, one barrier per chunk);
//   * narrow outputs use the "stream" kernel: one feature group per workgroup, the NW wavefronts
//     split the k range and combine through LDS in a fixed tree order;
//   * blockIdx.y is a global split-K.  Every slice is written to its own buffer; the workgroup that
//     finishes LAST for an output tile (atomic ticket, device-coherent slice accesses, no waiting) re-reads all
//     slices IN SLICE ORDER and runs the epilogue, so the result does not depend on arrival order.
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
constexpr int RING = 2;          // k steps in flight per wavefront (stream kernel); divides PD

#ifdef DED_GEMM_TRACE
__device__ unsigned long long* g_trace = nullptr;  // [workgroup][wave][8] wall-clock stamps (debug builds only)
#define DED_STAMP(i)                                                                                       \
  if (g_trace && (threadIdx.x & 63) == 0)                                                                  \
    g_trace[((((size_t)blockIdx.y * gridDim.x + blockIdx.x) * (blockDim.x >> 6)) + (threadIdx.x >> 6)) * 8 + (i)] = \
        wall_clock64();
#else
#define DED_STAMP(i)
#endif

typedef f32x4_t Acc[TN][4];  // one wavefront's tile: 4 feature tiles x 4 row blocks

// With a single 64-row group the weights of a skinny GEMM are read exactly once per launch (ONCE): loaded with the
// non-temporal hint they stream through the caches without displacing anything, which measured ~12 % more read
// bandwidth on a plain streaming kernel (6.8 against 6.0 TB/s).  With two or three row groups the later rounds of
// the launch find the weights in the last-level cache, and the hint would cost that.  The volatile flavour is for
// prefetches that must stay where they are written.
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
template <bool ONCE>
__device__ inline uint4 load_weights(const uint4* q) {
  if constexpr (ONCE) {
    const u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(q));
    return make_uint4(r.x, r.y, r.z, r.w);
  } else {
    return *q;
  }
}
template <bool ONCE>
__device__ inline uint4 load_weights_pinned(const uint4* q) {
  if constexpr (ONCE) {
    const u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const volatile u32x4_t*>(q));
    return make_uint4(r.x, r.y, r.z, r.w);
  } else {
    // (component-wise: a volatile load of the whole vector is compiled to an uncached system-scope access)
    const volatile uint4* c = q;
    uint4 r;
    r.x = c->x, r.y = c->y, r.z = c->z, r.w = c->w;
    return r;
  }
}

// Split-K slices travel between workgroups of one launch, which may sit on different XCDs with separate
// L2 caches.  Instead of device-scope fences (a whole-L2 write-back and invalidate per workgroup, measured
// at 3-4x the kernel time; even an acquire fence in the last workgroup alone, followed by plain 16-byte
// loads, was 10-20 % slower) the slices are written and read with device-scope relaxed atomic accesses, which
// go through to the memory side on their own; ordering comes from waiting for the stores to complete
// before the ticket is taken, and from the ticket's return value before the loads are issued.
// A slice is private to the kernel, so it is kept in accumulator order: tile (row group, feature group) ->
// (t, rb) -> half -> lane, 8 bytes each: every store / load instruction covers 512 contiguous bytes.
// -DDED_SPLITK_FENCES builds the memory-model-only variant instead (plain slice accesses, a release fence before
// the ticket and an acquire fence after it): the fallback should a future part or driver not give the
// write-through / read-through behaviour of device-scope atomics that the default relies on.
#ifdef DED_SPLITK_FENCES
__device__ inline void slice_store(unsigned long long* p, unsigned long long v) { *p = v; }
__device__ inline unsigned long long slice_load(const unsigned long long* p) { return *p; }
#else
__device__ inline void slice_store(unsigned long long* p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline unsigned long long slice_load(unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
#endif

__device__ inline unsigned long long pack2(float a, float b) {
  return ((unsigned long long)__float_as_uint(b) << 32) | __float_as_uint(a);
}
__device__ inline int64_t slice_tile_offset(int rb0, int NG, int ng) { return ((int64_t)(rb0 >> 2) * NG + ng) * (TN * 4 * 256); }

__device__ inline void store_slice(float* slice, int NG, int ng, int rb0, int lane, const Acc& acc) {
  unsigned long long* q = reinterpret_cast<unsigned long long*>(slice + slice_tile_offset(rb0, NG, ng)) + lane;
#pragma unroll
  for (int t = 0; t < TN; ++t)
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) {
      const f32x4_t v = acc[t][rb];
      slice_store(q + (t * 4 + rb) * 128, pack2(v[0], v[1]));
      slice_store(q + (t * 4 + rb) * 128 + 64, pack2(v[2], v[3]));
    }
}

// acc[t][j] = sum over slices 0..splits-1 (in slice order) of row block rb_lo + j of the tile, j < RBN
template <int RBN>
__device__ inline void load_slices(const float* part, int64_t part_stride, int splits, int NG, int ng, int rb0,
                                   int rb_lo, int lane, Acc& acc) {
#pragma unroll
  for (int t = 0; t < TN; ++t)
#pragma unroll
    for (int j = 0; j < RBN; ++j) acc[t][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const float* base = part + slice_tile_offset(rb0, NG, ng) + rb_lo * 256;
#pragma unroll 4
  for (int s = 0; s < splits; ++s) {
    unsigned long long* q =
        reinterpret_cast<unsigned long long*>(const_cast<float*>(base) + (int64_t)s * part_stride) + lane;
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
      for (int j = 0; j < RBN; ++j) {
        unsigned long long a = slice_load(q + (t * 4 + j) * 128);
        unsigned long long b = slice_load(q + (t * 4 + j) * 128 + 64);
        acc[t][j] += f32x4_t{__uint_as_float((unsigned)a), __uint_as_float((unsigned)(a >> 32)),
                             __uint_as_float((unsigned)b), __uint_as_float((unsigned)(b >> 32))};
      }
  }
}

// The same for a wavefront that holds only RBN row blocks of its tile (first one: rb_lo) in acc[t][0 .. RBN-1].
template <int RBN>
__device__ inline void store_slice_rows(float* slice, int NG, int ng, int rb0, int rb_lo, int lane, const Acc& acc) {
  unsigned long long* q =
      reinterpret_cast<unsigned long long*>(slice + slice_tile_offset(rb0, NG, ng) + rb_lo * 256) + lane;
#pragma unroll
  for (int t = 0; t < TN; ++t)
#pragma unroll
    for (int j = 0; j < RBN; ++j) {
      const f32x4_t v = acc[t][j];
      slice_store(q + (t * 4 + j) * 128, pack2(v[0], v[1]));
      slice_store(q + (t * 4 + j) * 128 + 64, pack2(v[2], v[3]));
    }
}

// acc[t][j] (in: this workgroup's own slice values, which it still holds) = sum over slices 0..S-1 in slice order,
// the own values standing in for slice `split`: only the S - 1 other slices are fetched, all loads in flight
// together.  The result does not depend on which workgroup arrived last.
template <int RBN, int S>
__device__ inline void sum_other_slices(const float* part, int64_t part_stride, int split, int NG, int ng, int rb0,
                                        int rb_lo, int lane, Acc& acc) {
  const float* base = part + slice_tile_offset(rb0, NG, ng) + rb_lo * 256;
  unsigned long long a[S - 1][TN][RBN], b[S - 1][TN][RBN];
#pragma unroll
  for (int k = 0; k < S - 1; ++k) {
    const int sl = k + (k >= split ? 1 : 0);
    unsigned long long* q =
        reinterpret_cast<unsigned long long*>(const_cast<float*>(base) + (int64_t)sl * part_stride) + lane;
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
      for (int j = 0; j < RBN; ++j) {
        a[k][t][j] = slice_load(q + (t * 4 + j) * 128);
        b[k][t][j] = slice_load(q + (t * 4 + j) * 128 + 64);
      }
  }
  f32x4_t own[TN][RBN];
#pragma unroll
  for (int t = 0; t < TN; ++t)
#pragma unroll
    for (int j = 0; j < RBN; ++j) own[t][j] = acc[t][j];
  // position p of the sum takes slice p: the own values at p == split, else the fetched slice k = p - (p > split)
#pragma unroll
  for (int p = 0; p < S; ++p) {
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
      for (int j = 0; j < RBN; ++j) {
        const int lo = p > 0 ? p - 1 : 0, hi = p < S - 1 ? p : S - 2;  // the fetched slice is one of a[lo], a[hi]
        const bool use_lo = p > split;
        const unsigned long long ua = use_lo ? a[lo][t][j] : a[hi][t][j];
        const unsigned long long ub = use_lo ? b[lo][t][j] : b[hi][t][j];
        const f32x4_t other = f32x4_t{__uint_as_float((unsigned)ua), __uint_as_float((unsigned)(ua >> 32)),
                                      __uint_as_float((unsigned)ub), __uint_as_float((unsigned)(ub >> 32))};
        const f32x4_t v = p == split ? own[t][j] : other;
        acc[t][j] = p == 0 ? v : acc[t][j] + v;
      }
  }
}

template <int RBN>
__device__ inline void sum_slices_keep_own(const float* part, int64_t part_stride, int split, int splits, int NG,
                                           int ng, int rb0, int rb_lo, int lane, Acc& acc) {
  if (splits == 2) {
    sum_other_slices<RBN, 2>(part, part_stride, split, NG, ng, rb0, rb_lo, lane, acc);
  } else if (splits == 4) {
    sum_other_slices<RBN, 4>(part, part_stride, split, NG, ng, rb0, rb_lo, lane, acc);
  } else if (splits == 3) {
    sum_other_slices<RBN, 3>(part, part_stride, split, NG, ng, rb0, rb_lo, lane, acc);
  } else {
    load_slices<RBN>(part, part_stride, splits, NG, ng, rb0, rb_lo, lane, acc);  // all slices, the own one included
  }
}

__device__ inline uint2 pack4_f16(float a, float b, float c, float d) {
  return make_uint2((uint32_t)f32_to_f16(a) | ((uint32_t)f32_to_f16(b) << 16),
                    (uint32_t)f32_to_f16(c) | ((uint32_t)f32_to_f16(d) << 16));
}
__device__ inline void split4_f16(const float (&v)[4], uint2& hi, uint2& lo) {
  uint16_t h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) split_f16(v[i], h[i], l[i]);
  hi = make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16));
  lo = make_uint2((uint32_t)l[0] | ((uint32_t)l[1] << 16), (uint32_t)l[2] | ((uint32_t)l[3] << 16));
}

// ------------------------------------------------------------------------------------------
// Epilogues.  Run by one wavefront on RBN row blocks (first one: rbase) of a 64-feature group; acc[t][j]
// holds row block rbase + j.  A lane holds, for row (rbase + j) * 16 + (lane & 15), the 4 features
// t * 16 + (lane >> 4) * 4 + i.  Feature groups of the QKV and gate/up matrices are interleaved at pack
// time (packw_source_row) so that tiles t and t + 2 of a group hold partner features: rotary pairs
// (i, i + 64), or gate / up.
// ------------------------------------------------------------------------------------------
// RMSNorm scale of the GEMM input rows: 1 / sqrt(sum(x^2) / d + eps), from the per-(row, 64-feature group)
// sums that the producer stored.  The sums were written by another kernel, usually from another XCD, and a
// load issued when they are needed costs ~3 us; at kernel start it would delay the first weight chunk (loads
// return in order).  So the wavefronts of a workgroup share the job: each fetches a slice of the groups for
// row rb0 * 16 + lane a few iterations before its k loop ends (ssq_issue; <= 8 float2 registers), adds them
// up after the loop, and the partial sums meet in LDS at the barrier the kernel has there anyway.
constexpr int SSQ_REGS = 8;
struct SsqPart {
  float2 v[SSQ_REGS];
};
__device__ inline void ssq_clear(SsqPart& p) {
#pragma unroll
  for (int i = 0; i < SSQ_REGS; ++i) p.v[i] = make_float2(0.f, 0.f);
}
// wavefront `wv` of `nwv` takes float2 units [wv * per, wv * per + per) of the row's ssq_groups / 2
__device__ inline void ssq_issue(const GemmEpilogue& e, int rb0, int lane, int wv, int nwv, SsqPart& p) {
  if (!e.ssq_in) return;
  const int n2 = e.ssq_groups >> 1, per = (n2 + nwv - 1) / nwv, g0 = wv * per;
  const float2* src = reinterpret_cast<const float2*>(e.ssq_in + (int64_t)(rb0 * 16 + lane) * e.ssq_groups);
#pragma unroll
  for (int i = 0; i < SSQ_REGS; ++i)
    if (i < per && g0 + i < n2) p.v[i] = src[g0 + i];
}
// partial sum of this wavefront's slice -> LDS (call before a workgroup barrier)
__device__ inline void ssq_publish(const GemmEpilogue& e, int rb0, int lane, int wv, int nwv, const SsqPart& p,
                                   float* s_ssq) {
  if (!e.ssq_in) return;
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < SSQ_REGS; ++i) s += p.v[i].x + p.v[i].y;
  const int n2 = e.ssq_groups >> 1, per = (n2 + nwv - 1) / nwv, g0 = wv * per;
  const float2* src = reinterpret_cast<const float2*>(e.ssq_in + (int64_t)(rb0 * 16 + lane) * e.ssq_groups);
  for (int i = SSQ_REGS; i < per && g0 + i < n2; ++i) s += src[g0 + i].x + src[g0 + i].y;  // very wide rows only
  s_ssq[wv * 64 + lane] = s;
}
// after that barrier: scale of row rb0 * 16 + lane (partials added in wavefront order)
__device__ inline float ssq_scale(const GemmEpilogue& e, int lane, int nwv, const float* s_ssq) {
  if (!e.ssq_in) return 1.f;
  float s = 0.f;
  for (int w = 0; w < nwv; ++w) s += s_ssq[w * 64 + lane];
  return 1.0f / sqrtf(s * e.inv_k + e.eps);
}

template <int EPI, int RBN>
__device__ inline void run_epilogue(const GemmEpilogue& e, int ng, int N, int rb0, int rbase, float row_scale, int lane,
                                    Acc& acc) {
  const int row_in = lane & 15, quad = lane >> 4;
  float scale[RBN];
#pragma unroll
  for (int j = 0; j < RBN; ++j) scale[j] = __shfl(row_scale, (rbase - rb0 + j) * 16 + row_in);

  if (EPI == EPI_LOGITS) {
#pragma unroll
    for (int t = 0; t < TN; ++t) {
      const int n = (ng * TN + t) * 16 + quad * 4;
      if (n >= N) continue;
#pragma unroll
      for (int rb = 0; rb < RBN; ++rb) {
        const int64_t r = (int64_t)(rbase + rb) * 16 + row_in;
        f32x4_t v = acc[t][rb] * scale[rb];
        *reinterpret_cast<float4*>(e.out + r * e.out_stride + n) = make_float4(v[0], v[1], v[2], v[3]);
      }
    }
  } else if (EPI == EPI_TOP2) {
    // what the approval walk needs of a logits row, without the row: the best value of this 64-feature group, its
    // feature index (lowest on ties), the second best value, and whether any value is NaN or infinite
    uint4* dst = reinterpret_cast<uint4*>(e.top2_part);
#pragma unroll
    for (int rb = 0; rb < RBN; ++rb) {
      const int64_t r = (int64_t)(rbase + rb) * 16 + row_in;
      float v1 = -INFINITY, v2 = -INFINITY;
      int i1 = 0x7fffffff, bad = 0;
#pragma unroll
      for (int t = 0; t < TN; ++t) {
        const int n = (ng * TN + t) * 16 + quad * 4;
        if (n >= N) continue;
        const f32x4_t v = acc[t][rb] * scale[rb];
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // ascending feature index: a later equal value never replaces the first
          const float x = v[i];
          bad |= !(fabsf(x) <= 3.402823466e38f);
          if (x > v1) {
            v2 = v1;
            v1 = x;
            i1 = n + i;
          } else if (x > v2) {
            v2 = x;
          }
        }
      }
#pragma unroll
      for (int off = 16; off <= 32; off <<= 1) {  // the four lanes that share the row
        const float ov1 = __shfl_xor(v1, off), ov2 = __shfl_xor(v2, off);
        const int oi1 = __shfl_xor(i1, off);
        bad |= __shfl_xor(bad, off);
        if (ov1 > v1 || (ov1 == v1 && oi1 < i1)) {
          v2 = fmaxf(v1, ov2);
          v1 = ov1;
          i1 = oi1;
        } else {
          v2 = fmaxf(v2, ov1);
        }
      }
      if (quad == 0)
        dst[r * e.top2_groups + ng] = make_uint4(__float_as_uint(v1), (uint32_t)i1, __float_as_uint(v2), (uint32_t)bad);
    }
  } else if (EPI == EPI_RESIDUAL) {
    // x += Y;  next GEMM input = (x * gain) as hi/lo f16 (its 1/rms is applied by the consumer);  sum(x^2) per group
#pragma unroll
    for (int rb = 0; rb < RBN; ++rb) {
      const int r = (rbase + rb) * 16 + row_in;
      float ss = 0.f;
#pragma unroll
      for (int t = 0; t < TN; ++t) {
        const int n = (ng * TN + t) * 16 + quad * 4;
        float* xp = e.x + (int64_t)r * N + n;
        float4 xv = *reinterpret_cast<const float4*>(xp);
        float4 g = *reinterpret_cast<const float4*>(e.gain + n);
        float xn[4] = {xv.x + acc[t][rb][0], xv.y + acc[t][rb][1], xv.z + acc[t][rb][2], xv.w + acc[t][rb][3]};
        *reinterpret_cast<float4*>(xp) = make_float4(xn[0], xn[1], xn[2], xn[3]);
        ss += xn[0] * xn[0] + xn[1] * xn[1] + xn[2] * xn[2] + xn[3] * xn[3];
        float y[4] = {xn[0] * g.x, xn[1] * g.y, xn[2] * g.z, xn[3] * g.w};
        uint2 hi, lo;
        split4_f16(y, hi, lo);
        *reinterpret_cast<uint2*>(e.y_packed + packx_index(r, n, e.rb_total, 0)) = hi;
        *reinterpret_cast<uint2*>(e.y_packed + packx_index(r, n, e.rb_total, 1)) = lo;
      }
      ss += __shfl_xor(ss, 16);
      ss += __shfl_xor(ss, 32);
      if (quad == 0) e.ssq_out[(int64_t)r * (N / 64) + ng] = ss;
    }
  } else if (EPI == EPI_SILU) {
    // group ng = gate features [32 ng, 32 ng + 32) in tiles 0, 1 and the matching up features in tiles 2, 3
#pragma unroll
    for (int rb = 0; rb < RBN; ++rb) {
      const int r = (rbase + rb) * 16 + row_in;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int f = ng * 32 + t * 16 + quad * 4;
        if (2 * f >= N) continue;
        float h[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float gv = acc[t][rb][i] * scale[rb], uv = acc[t + 2][rb][i] * scale[rb];
          h[i] = gv / (1.0f + __expf(-gv)) * uv;
        }
        *reinterpret_cast<uint2*>(e.y_packed + packx_index(r, f, e.rb_total, 0)) = pack4_f16(h[0], h[1], h[2], h[3]);
      }
    }
  } else if (EPI == EPI_QKV) {
    // group ng = head slot ng / 2, dims [32 j, 32 j + 32) in tiles 0, 1 and their rotary partners (+64) in tiles 2, 3
    const int hs = ng >> 1, j = ng & 1;
    const int G = e.H / e.Hkv;
#pragma unroll
    for (int rb = 0; rb < RBN; ++rb) {
      const int r = (rbase + rb) * 16 + row_in;
      if (r >= e.rows) continue;
      const int b = r / e.n_step, node = r - b * e.n_step;
      const bool real = node < e.seq_n[b];
      const int slot = e.seq_p[b] + node;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int d0 = 32 * j + 16 * t + quad * 4;
        float a[4], c[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          a[i] = acc[t][rb][i] * scale[rb];
          c[i] = acc[t + 2][rb][i] * scale[rb];
        }
        if (hs < e.H + e.Hkv) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float2 cs = e.rope_tab[(int64_t)r * 64 + d0 + i];
            float ra = a[i] * cs.x - c[i] * cs.y;
            float rc = c[i] * cs.x + a[i] * cs.y;
            a[i] = ra;
            c[i] = rc;
          }
        }
        if (hs < e.H) {
          const int kvh = hs / G, g = hs - kvh * G;
          const int vr = g * e.n_step + node;
          uint16_t* base = e.q_packed + ((int64_t)b * e.Hkv + kvh) * ((int64_t)G * e.n_step * 128 * 2);
          uint2 hi, lo;
          split4_f16(a, hi, lo);
          *reinterpret_cast<uint2*>(base + packq_index(vr, d0, 0)) = hi;
          *reinterpret_cast<uint2*>(base + packq_index(vr, d0, 1)) = lo;
          split4_f16(c, hi, lo);
          *reinterpret_cast<uint2*>(base + packq_index(vr, d0 + 64, 0)) = hi;
          *reinterpret_cast<uint2*>(base + packq_index(vr, d0 + 64, 1)) = lo;
        } else if (real && hs < e.H + e.Hkv) {
          uint16_t* base = e.k_cache + ((int64_t)b * e.Hkv + (hs - e.H)) * ((int64_t)e.cap * 128);
          *reinterpret_cast<uint2*>(base + packk_index(slot, d0)) = pack4_f16(a[0], a[1], a[2], a[3]);
          *reinterpret_cast<uint2*>(base + packk_index(slot, d0 + 64)) = pack4_f16(c[0], c[1], c[2], c[3]);
        } else if (real) {
          uint16_t* base = e.v_cache + ((int64_t)b * e.Hkv + (hs - e.H - e.Hkv)) * ((int64_t)e.cap * 128);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            base[packvt_index(slot, d0 + i)] = f32_to_f16(a[i]);
            base[packvt_index(slot, d0 + 64 + i)] = f32_to_f16(c[i]);
          }
        }
      }
    }
  }
}

// Split-K hand-over (splits > 1), second part: called by the whole workgroup after its wavefronts have issued their
// slice stores.  Returns true in the workgroup that arrived last for its output tile.
__device__ inline bool take_ticket(int splits, int* counters, int* s_flag) {
#ifdef DED_SPLITK_FENCES
  __atomic_thread_fence(__ATOMIC_RELEASE);  // agent scope is the default of a thread fence in HIP device code
#else
  __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0): this wavefront's slice stores have completed
#endif
  DED_STAMP(4)
  __syncthreads();
  if (threadIdx.x == 0) {
    int* ticket = counters + (blockIdx.z * gridDim.x + blockIdx.x);
    int prev = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int last = prev == splits - 1;
    if (last) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next launch
    *s_flag = last;
  }
  __syncthreads();
#ifdef DED_SPLITK_FENCES
  if (*s_flag) __atomic_thread_fence(__ATOMIC_ACQUIRE);
#endif
  DED_STAMP(5)
  return *s_flag != 0;
}

// Hand-over of whole tiles: the wavefronts that hold a complete workgroup tile (`owner`) write it as this
// workgroup's slice; the last-arriving workgroup then re-reads all slices in slice order (load_slices, any of its
// wavefronts) and runs the epilogue.
__device__ inline bool finish_split(float* part, int64_t part_stride, int split, int splits, int* counters, int NG,
                                    int ng, int rb0, int lane, bool owner, const Acc& acc, int* s_flag) {
  if (owner) store_slice(part + (int64_t)split * part_stride, NG, ng, rb0, lane, acc);
  return take_ticket(splits, counters, s_flag);
}

// ------------------------------------------------------------------------------------------
// Stream kernel: one feature group per workgroup, NW wavefronts split the k range.
// ------------------------------------------------------------------------------------------
template <int NW, int PLANES, int EPI, bool ONCE>
__global__ __launch_bounds__(NW * 64, 2) void gemm_stream_kernel(float* __restrict__ part, int64_t part_stride,
                                                                 const uint4* __restrict__ xp,
                                                                 const uint4* __restrict__ wp, int RB, int N, int KT,
                                                                 int splits, int* __restrict__ counters,
                                                                 GemmEpilogue epi) {
  __shared__ float4 red[(NW > 1 ? NW / 2 : 1) * TN * 4 * 64];
  __shared__ float s_ssq[NW * 64];
  __shared__ int s_flag;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ng = blockIdx.x;
  const int split = blockIdx.y;
  const int rb0 = blockIdx.z * 4;
  // this wavefront's k range, in units of RING steps (the finest grain the loop allows: K = 11008 over 16
  // wavefronts is 21 or 22 steps each, where whole groups of PD steps would give 20 or 24)
  const int units = KT / RING;
  const int parts = splits * NW;
  const int gi = split * NW + wave;
  const int g_begin = (int)((int64_t)gi * units / parts);
  const int g_end = (int)((int64_t)(gi + 1) * units / parts);

  Acc acc;
#pragma unroll
  for (int t = 0; t < TN; ++t)
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) acc[t][rb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  DED_STAMP(0)
  SsqPart ssq;
  ssq_clear(ssq);
  if (g_begin < g_end) {
    const uint4* wsrc = wp + (((int64_t)ng * KT * TN) << 6) + lane;
    // per k step the activations of the 4 row blocks x 2 planes (hi, lo) are 8 KiB of contiguous memory
    const uint4* xsrc = xp + ((int64_t)rb0 << 7) + lane;
    const int64_t xstep = (int64_t)RB << 7;

    uint4 wr[RING][TN], xr[RING][4 * PLANES];
    auto issue = [&](int slot, int kt) {
#pragma unroll
      for (int t = 0; t < TN; ++t) wr[slot][t] = load_weights<ONCE>(wsrc + (((int64_t)kt * TN + t) << 6));
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

    int kt = g_begin * RING;
    const int kt_last = g_end * RING - RING;  // first step of the last ring-full
#pragma unroll
    for (int j = 0; j < RING; ++j) issue(j, kt + j);
    const int kt_ssq = kt_last - 8 * RING > kt ? kt_last - 8 * RING : kt;  // 8 ring turns before the end
    if (kt >= kt_last) ssq_issue(epi, rb0, lane, wave, NW, ssq);
    for (; kt < kt_last; kt += RING) {
#pragma unroll
      for (int j = 0; j < RING; ++j) {
        compute(j);
        issue(j, kt + RING + j);
      }
      if (kt == kt_ssq) ssq_issue(epi, rb0, lane, wave, NW, ssq);
    }
#pragma unroll
    for (int j = 0; j < RING; ++j) compute(j);
  } else {
    ssq_issue(epi, rb0, lane, wave, NW, ssq);
  }
  ssq_publish(epi, rb0, lane, wave, NW, ssq, s_ssq);
  if (NW == 1) __syncthreads();

  DED_STAMP(2)
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
  DED_STAMP(3)
  const float row_scale = ssq_scale(epi, lane, NW, s_ssq);  // the reduction above had at least one barrier
  if (splits == 1) {
    if (wave == 0) run_epilogue<EPI, 4>(epi, ng, N, rb0, rb0, row_scale, lane, acc);
  } else if (finish_split(part, part_stride, split, splits, counters, gridDim.x, ng, rb0, lane, wave == 0, acc, &s_flag)) {
    constexpr int RBN = 4 / NW;  // the wavefronts of the last workgroup share the tile's row blocks
    load_slices<RBN>(part, part_stride, splits, gridDim.x, ng, rb0, wave * RBN, lane, acc);
    DED_STAMP(6)
    run_epilogue<EPI, RBN>(epi, ng, N, rb0, rb0 + wave * RBN, row_scale, lane, acc);
  }
  DED_STAMP(7)
}

// ------------------------------------------------------------------------------------------
// Wide kernel: a workgroup owns NWN neighbouring feature groups over one k range.  Its 2 x NWN
// wavefronts form two halves: half h walks the h-th half of the k range, wavefront wn of a half owns
// feature group wn.  The activation chunks (CH k steps x 4 row blocks x PLANES) of each half are
// staged through LDS once per half (double buffered, one barrier per chunk), so the activations cost
// 1/NWN of what they would if every wavefront fetched its own.  Two wavefronts per SIMD overlap each
// other's LDS waits and barriers; the halves are added through LDS at the end (fixed order).
// ------------------------------------------------------------------------------------------
template <int NWN, int PLANES, int EPI, bool ONCE>
__global__ __launch_bounds__(NWN * 128, 2) void gemm_wide_kernel(float* __restrict__ part, int64_t part_stride,
                                                                 const uint4* __restrict__ xp,
                                                                 const uint4* __restrict__ wp, int RB, int N, int KT,
                                                                 int splits, int* __restrict__ counters,
                                                                 GemmEpilogue epi) {
  constexpr int TH = NWN * 64;                    // threads per half
  constexpr int CH = (NWN == 4 || PLANES == 1) ? 2 : 1;  // k steps per activation chunk (<= 4 staged units / thread)
  constexpr int STEP_U4 = 4 * PLANES * 64;        // uint4 units of activations per k step
  constexpr int CHUNK_U4 = CH * STEP_U4;
  constexpr int PER_THREAD = (CHUNK_U4 + TH - 1) / TH;
  constexpr int ACC_U4 = TN * 4 * 64;             // float4 units of one wavefront's accumulators
  constexpr int LDS_U4 = (2 * 2 * CHUNK_U4 > NWN * ACC_U4) ? 2 * 2 * CHUNK_U4 : NWN * ACC_U4;
  __shared__ uint4 lds[LDS_U4];                   // [half][buffer][chunk]; reused for the final reduction
  __shared__ float s_ssq[2 * NWN * 64];
  __shared__ int s_flag;
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

  Acc acc;
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
      for (int t = 0; t < TN; ++t) w.f[s][t] = load_weights<ONCE>(wsrc + (((int64_t)(kt0 + c * CH + s) * TN + t) << 6));
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
  // Software pipeline.  Loads return in order, so waiting for an activation chunk also waits for every
  // weight chunk issued before it: with activations one chunk ahead an iteration could not be shorter than
  // one HBM round trip (measured: 16 iterations of 1.4 us).  Hence activations are fetched TWO chunks ahead
  // (registers; the LDS copy stays double buffered) and weights THREE: the wait for activation chunk c + 1
  // then only needs loads that are two iterations old.  In every iteration the activation loads are issued
  // before the weight loads.  Both halves run the same number of iterations and barriers (n_chunks >= 2).
  // Kernel shapes whose chunks hold two k steps keep the shallower pipeline (activations one chunk ahead,
  // weights two): their iterations are twice as long, and the deeper one does not fit the register file.
  constexpr bool DEEP = CH == 1;
  SsqPart ssq;
  ssq_clear(ssq);
  const int wv = threadIdx.x >> 6;
  const int c_ssq = n_chunks - 14;  // fetch the row sums ~10 iterations before the loop ends
  if constexpr (DEEP) {
    // Weights three chunks ahead, activations two.  The ring slots are fixed registers (the loop is unrolled by the
    // ring length and leaves from the middle): a copy between slots would have to wait for the load that still
    // writes its source.  The loads go through volatile accesses: the compiler otherwise sinks a prefetch to the
    // block of its first use, i.e. issues it one iteration before it is needed whatever the source says.  Fetches
    // past the range re-read its last chunk (in bounds, never used).
    const int c_max = n_chunks - 1;
    auto cl = [&](int c) { return c < c_max ? c : c_max; };
    auto ldv = [](const volatile uint4* q) {
      uint4 r;
      r.x = q->x, r.y = q->y, r.z = q->z, r.w = q->w;
      return r;
    };
    auto load_w_pinned = [&](int c) {
      WChunk w;
#pragma unroll
      for (int t = 0; t < TN; ++t) w.f[0][t] = load_weights_pinned<ONCE>(wsrc + (((int64_t)(kt0 + c) * TN + t) << 6));
      return w;
    };
    auto load_x_pinned = [&](int c) {
      XStage x;
#pragma unroll
      for (int i = 0; i < PER_THREAD; ++i) {
        int u = tid + i * TH;
        if (CHUNK_U4 % TH != 0 && u >= CHUNK_U4) u = CHUNK_U4 - 1;  // surplus threads fetch the last unit again
        x.u[i] = ldv(xsrc + (int64_t)(kt0 + c) * xstep + u);        // CH == 1, two planes: unit u of the step
      }
      return x;
    };
    static_assert(!DEEP || (CH == 1 && PLANES == 2), "the pinned loads assume one two-plane k step per chunk");
    const int c_ssq4 = c_ssq > 0 ? c_ssq / 4 * 4 : 0;
    XStage xa = load_x_pinned(0), xb;  // xa: even chunks, xb: odd chunks
    WChunk w0 = load_w_pinned(0);
    xb = load_x_pinned(cl(1));
    WChunk w1 = load_w_pinned(cl(1));
    WChunk w2 = load_w_pinned(cl(2));
    WChunk w3;
    store_x(0, xa);
    __syncthreads();
    DED_STAMP(1)
    for (int c = 0;;) {
      if (c == c_ssq4) ssq_issue(epi, rb0, lane, wv, 2 * NWN, ssq);
      xa = load_x_pinned(cl(c + 2));
      w3 = load_w_pinned(cl(c + 3));
      compute(w0, 0);
      store_x(1, xb);
      __syncthreads();
      if (++c >= n_chunks) break;
      xb = load_x_pinned(cl(c + 2));
      w0 = load_w_pinned(cl(c + 3));
      compute(w1, 1);
      store_x(0, xa);
      __syncthreads();
      if (++c >= n_chunks) break;
      xa = load_x_pinned(cl(c + 2));
      w1 = load_w_pinned(cl(c + 3));
      compute(w2, 0);
      store_x(1, xb);
      __syncthreads();
      if (++c >= n_chunks) break;
      xb = load_x_pinned(cl(c + 2));
      w2 = load_w_pinned(cl(c + 3));
      compute(w3, 1);
      store_x(0, xa);
      __syncthreads();
      if (++c >= n_chunks) break;
    }
  } else {
    WChunk w0 = load_w(0);
    XStage x0 = load_x(0);
    WChunk w1 = load_w(1);
    int buf = 0;
    store_x(0, x0);
    __syncthreads();
    DED_STAMP(1)
    if (c_ssq < 0) ssq_issue(epi, rb0, lane, wv, 2 * NWN, ssq);
    for (int c = 0; c + 2 < n_chunks; ++c) {
      XStage xn = load_x(c + 1);
      WChunk w2 = load_w(c + 2);
      if (c == c_ssq) ssq_issue(epi, rb0, lane, wv, 2 * NWN, ssq);
      compute(w0, buf);
      store_x(buf ^ 1, xn);
      __syncthreads();
      w0 = w1;
      w1 = w2;
      buf ^= 1;
    }
    XStage xn = load_x(n_chunks - 1);  // last two chunks: nothing left to prefetch
    compute(w0, buf);
    store_x(buf ^ 1, xn);
    __syncthreads();
    compute(w1, buf ^ 1);
  }
  DED_STAMP(2)
  ssq_publish(epi, rb0, lane, threadIdx.x >> 6, 2 * NWN, ssq, s_ssq);
  // the halves are added through LDS: half h ends up with row blocks 2h, 2h + 1 of its feature group, in
  // acc[t][0..1]; each half hands the other the two row blocks it does not finish
  __syncthreads();
  {
    constexpr int HALF_U4 = TN * 2 * 64;  // two row blocks of one wavefront's accumulators
    float4* out = reinterpret_cast<float4*>(lds) + (half * NWN + wn) * HALF_U4 + lane;
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const f32x4_t v = half == 0 ? acc[t][2 + j] : acc[t][j];
        out[(t * 2 + j) * 64] = make_float4(v[0], v[1], v[2], v[3]);
      }
    __syncthreads();
    const float4* in = reinterpret_cast<const float4*>(lds) + ((1 - half) * NWN + wn) * HALF_U4 + lane;
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const float4 v = in[(t * 2 + j) * 64];
        const f32x4_t mine = half == 0 ? acc[t][j] : acc[t][2 + j];
        acc[t][j] = mine + f32x4_t{v.x, v.y, v.z, v.w};
      }
  }
  DED_STAMP(3)
  const float row_scale = ssq_scale(epi, lane, 2 * NWN, s_ssq);
  const bool store_ok = ng_raw < NG;
  if (splits == 1) {
    if (store_ok) run_epilogue<EPI, 2>(epi, ng, N, rb0, rb0 + half * 2, row_scale, lane, acc);
  } else {
    // every wavefront writes the two row blocks it holds; in the last workgroup it fetches the same two row
    // blocks of the other slices and finishes them
    if (store_ok) store_slice_rows<2>(part + (int64_t)split * part_stride, NG, ng, rb0, half * 2, lane, acc);
    if (take_ticket(splits, counters, &s_flag) && store_ok) {
      sum_slices_keep_own<2>(part, part_stride, split, splits, NG, ng, rb0, half * 2, lane, acc);
      DED_STAMP(6)
      run_epilogue<EPI, 2>(epi, ng, N, rb0, rb0 + half * 2, row_scale, lane, acc);
    }
  }
  DED_STAMP(7)
}

// ------------------------------------------------------------------------------------------
// Large-row kernel (rows_pad >= 256: batched trees).  With hundreds of rows per weight the projection is
// bound by the matrix cores, not by the weight stream, so this is an ordinary tiled GEMM on the same
// fragment layouts: a workgroup of 8 wavefronts owns FGS feature groups x RGS row groups (FGS * RGS == 8;
// a wavefront owns GPW = 2 feature groups x 1 row group: 256 features x 256 rows per workgroup), in units of
// the 64 x 64 tile the other kernels give a wavefront, so the split-K hand-over and the epilogues are shared.
// A stage holds CH k steps of the workgroup's weights and activations in LDS (double buffered, one barrier
// per stage; global loads run two stages ahead in registers).  Per k step a wavefront reads 8 weight and
// 4 x PLANES activation fragments from LDS for 32 x PLANES matrix instructions: LDS read bandwidth, the
// limit of a smaller wavefront tile (64 x 64: 52 % of the f16 peak), is a third lower per instruction.
// ------------------------------------------------------------------------------------------
__device__ inline float ssq_direct(const GemmEpilogue& e, int rb0, int lane) {
  if (!e.ssq_in) return 1.f;
  const float2* p = reinterpret_cast<const float2*>(e.ssq_in + (int64_t)(rb0 * 16 + lane) * e.ssq_groups);
  float s = 0.f;
#pragma unroll 8
  for (int g = 0; g < (e.ssq_groups >> 1); ++g) s += p[g].x + p[g].y;
  return 1.0f / sqrtf(s * e.inv_k + e.eps);
}

// Two shapes (plan.nwn 8 and 9): GPW = 1 feature group per wavefront, wavefront grid 4 x 2 (256 features x 128
// rows per workgroup: more workgroups, for a few hundred rows and for single-plane inputs), and GPW = 2,
// wavefront grid 2 x 4 (256 features x 256 rows: fewer LDS bytes per matrix instruction).
constexpr int LARGE_FEAT_GROUPS = 4;  // feature groups per workgroup (x 64 features), both shapes
constexpr int large_row_groups(int gpw) { return gpw == 1 ? 2 : 4; }  // 64-row groups per workgroup

template <int PLANES, int EPI, int GPW>
__global__ __launch_bounds__(512) void gemm_large_kernel(float* __restrict__ part, int64_t part_stride,
                                                         const uint4* __restrict__ xp, const uint4* __restrict__ wp,
                                                         int RB, int N, int KT, int splits,
                                                         int* __restrict__ counters, GemmEpilogue epi, int x_off,
                                                         int slice_ng) {
  // x_off / slice_ng: a launch may cover only the feature tiles from x_off on (the remainder launch of a plan whose
  // last scheduling round would be mostly empty; it splits k where the main launch does not); its slices are indexed
  // by the feature group's offset inside that range, slice_ng groups per row group
  constexpr int FGS = LARGE_FEAT_GROUPS / GPW, RGS = large_row_groups(GPW);
  constexpr int CH = (PLANES == 2 && GPW == 2) ? 1 : 2;  // k steps per LDS stage
  static_assert(FGS * RGS == 8, "8 wavefronts");
  constexpr int W_U4 = FGS * GPW * TN * 64;         // weights of one k step
  constexpr int X_U4 = RGS * 4 * PLANES * 64;       // activations of one k step
  constexpr int STEP_U4 = W_U4 + X_U4;
  constexpr int STAGE_U4 = CH * STEP_U4;
  constexpr int UPS = STEP_U4 / 512;                // staged units per thread and k step
  constexpr int WUPS = W_U4 / 512;                  // ... of which weights (the first ones)
  constexpr int NU = CH * UPS;
  static_assert(STEP_U4 % 512 == 0 && W_U4 % 512 == 0 && NU <= 8, "units must not straddle operand kinds");
  static_assert(PD % CH == 0, "a k range holds whole stages");
  __shared__ uint4 lds[2][STAGE_U4];
  __shared__ int s_flag;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int fg = wave % FGS, rg = wave / FGS;
  const int NG = (N + 16 * TN - 1) / (16 * TN);
  const int bx = blockIdx.x + x_off;
  const int g_off = x_off * (FGS * GPW);
  const int g_first = (bx * FGS + fg) * GPW;  // first feature group of this wavefront
  const int split = blockIdx.y;
  const int rb_tile = blockIdx.z * (RGS * 4);
  const int rbw = rb_tile + rg * 4;                 // first row block of this wavefront
  const int groups = KT / PD;
  const int k_begin = (int)((int64_t)split * groups / splits) * PD;
  const int k_end = (int)((int64_t)(split + 1) * groups / splits) * PD;
  const int n_stages = (k_end - k_begin) / CH;      // >= PD / CH >= 2

  // Unit i of a thread (u = tid + 512 i inside a stage): k step i / UPS of the stage; inside the step the
  // first WUPS units are weights, the others activations (the kind depends on i only).  off[i] = offset of
  // the unit from the operand's address at the stage's first k step.
  const int64_t xstride = (int64_t)RB << 7;         // activations of one k step (all row blocks, 2 planes)
  int64_t off[NU];
#pragma unroll
  for (int i = 0; i < NU; ++i) {
    const int ks = i / UPS, j = i % UPS;
    if (j < WUPS) {
      const int v = tid + j * 512;
      const int g_raw = bx * (FGS * GPW) + (v >> 8);
      off[i] = ((((int64_t)(g_raw < NG ? g_raw : NG - 1) * KT + ks) * TN) << 6) + (v & 255);
    } else {
      const int xu = tid + (j - WUPS) * 512;
      const int rbl = xu / (PLANES * 64), rem = xu - rbl * (PLANES * 64);
      const int rb = rb_tile + rbl < RB ? rb_tile + rbl : RB - 1;  // ragged last row tile: re-read a valid block
      off[i] = ks * xstride + (rb * 2 + rem / 64) * 64 + (rem & 63);
    }
  }
  struct Stage {  // named members keep the staged units in registers
    uint4 u0, u1, u2, u3, u4, u5, u6, u7;
  };
#define DED_EACH_UNIT(F) F(0, u0) F(1, u1) F(2, u2) F(3, u3) F(4, u4) F(5, u5) F(6, u6) F(7, u7)
  auto load_stage = [&](int kt) {
    Stage st;
    const uint4* wk = wp + ((int64_t)kt * TN << 6);
    const uint4* xk = xp + kt * xstride;
#define DED_LOAD(i, m) \
    if constexpr (i < NU) st.m = ((i % UPS) < WUPS ? wk : xk)[off[i < NU ? i : 0]];
    DED_EACH_UNIT(DED_LOAD)
#undef DED_LOAD
    return st;
  };
  auto store_stage = [&](int buf, const Stage& st) {
    uint4* d = lds[buf] + tid;
#define DED_STORE(i, m) \
    if constexpr (i < NU) d[i * 512] = st.m;
    DED_EACH_UNIT(DED_STORE)
#undef DED_STORE
  };
#undef DED_EACH_UNIT

  Acc acc[GPW];
#pragma unroll
  for (int gw = 0; gw < GPW; ++gw)
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) acc[gw][t][rb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  auto compute = [&](int buf) {
#pragma unroll
    for (int ks = 0; ks < CH; ++ks) {
      const uint4* lw = lds[buf] + ks * STEP_U4 + fg * (GPW * TN * 64) + lane;
      const uint4* lx = lds[buf] + ks * STEP_U4 + W_U4 + rg * (4 * PLANES * 64) + lane;
      f16x8_t b[4 * PLANES];
#pragma unroll
      for (int i = 0; i < 4 * PLANES; ++i) b[i] = __builtin_bit_cast(f16x8_t, lx[i << 6]);
#pragma unroll
      for (int gw = 0; gw < GPW; ++gw)
#pragma unroll
        for (int t = 0; t < TN; ++t) {
          f16x8_t a = __builtin_bit_cast(f16x8_t, lw[(gw * TN + t) << 6]);
#pragma unroll
          for (int p = 0; p < PLANES; ++p)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
              acc[gw][t][rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b[rb * PLANES + p], acc[gw][t][rb], 0, 0, 0);
        }
    }
  };

  // Stage c + 2 is fetched while stage c is computed and stage c + 1 is parked in LDS.
  Stage s0 = load_stage(k_begin);
  Stage s1 = load_stage(k_begin + CH);
  store_stage(0, s0);
  __syncthreads();
  int buf = 0;
  for (int c = 0; c + 2 < n_stages; ++c) {
    Stage s2 = load_stage(k_begin + (c + 2) * CH);
    compute(buf);
    store_stage(buf ^ 1, s1);
    __syncthreads();
    s1 = s2;
    buf ^= 1;
  }
  compute(buf);  // second-last stage
  store_stage(buf ^ 1, s1);
  __syncthreads();
  compute(buf ^ 1);  // last stage

  // every wavefront finishes its own GPW tiles of 64 features x 64 rows
  const bool rows_ok = rbw < RB;
  const float row_scale = ssq_direct(epi, rows_ok ? rbw : 0, lane);
  bool last = true;
  if (splits > 1) {
#pragma unroll
    for (int gw = 1; gw < GPW; ++gw)
      if (rows_ok && g_first + gw < NG)
        store_slice(part + (int64_t)split * part_stride, slice_ng, g_first + gw - g_off, rbw, lane, acc[gw]);
    last = finish_split(part, part_stride, split, splits, counters, slice_ng, (g_first < NG ? g_first : NG - 1) - g_off, rbw,
                        lane, rows_ok && g_first < NG, acc[0], &s_flag);
  }
  if (last && rows_ok) {
#pragma unroll
    for (int gw = 0; gw < GPW; ++gw) {
      const int ng = g_first + gw;
      if (ng >= NG) continue;
      if (splits > 1) load_slices<4>(part, part_stride, splits, slice_ng, ng - g_off, rbw, 0, lane, acc[gw]);
      run_epilogue<EPI, 4>(epi, ng, N, rbw, rbw, row_scale, lane, acc[gw]);
    }
  }
}

// Sweep knob, compiled in only with -DDED_GEMM_TUNE_ENV (never in the library build): the environment variable
// DED_GEMM_TUNE="nwn,splits" forces the kernel shape (nwn 0 = stream kernel).
struct Tune {
  int nwn = -1, splits = 0;
  Tune() {
#ifdef DED_GEMM_TUNE_ENV
    if (const char* e = getenv("DED_GEMM_TUNE")) {
      int a = -1, b = 0;
      if (sscanf(e, "%d,%d", &a, &b) == 2 && a >= 0 && a <= 4 && b >= 1) {
        nwn = a;
        splits = b;
      }
    }
#endif
  }
};

constexpr int kCUs = 256;

// relative cost of a shape: weight stream slowed down by activation reloads and uneven CU filling,
// plus the split-K slices that are written and read back inside the kernel
double shape_cost(int64_t w_bytes, int64_t slice_bytes, int wgs, double x_per_w, int splits) {
  int rounds = (wgs + kCUs - 1) / kCUs;
  double eff = (double)wgs / (double)(rounds * kCUs);
  double stream = (double)w_bytes * (1.0 + 0.35 * x_per_w) / eff;
  return stream + 2.0 * (double)slice_bytes * (splits > 1 ? splits : 0);
}

template <int PLANES, int EPI>
bool launch_shape(const GemmPlan& plan, dim3 grid_stream, dim3 grid_wide, float* part, int64_t part_stride,
                  const uint4* xp, const uint4* wp, int RB, int N, int KT, int* counters, const GemmEpilogue& epi,
                  int nw, hipStream_t s) {
  const int splits = plan.splits;
#define DED_ARGS part, part_stride, xp, wp, RB, N, KT, splits, counters, epi
  if (plan.nwn == 8 || plan.nwn == 9) {
    const int rgs = large_row_groups(plan.nwn - 7);
    const int NG = (N + 16 * TN - 1) / (16 * TN);
    const int X = (NG + LARGE_FEAT_GROUPS - 1) / LARGE_FEAT_GROUPS, Z = (RB + 4 * rgs - 1) / (4 * rgs);
    auto go = [&](dim3 grid, int64_t stride, int n_splits, int x_off, int slice_ng) {
      if (plan.nwn == 8)
        hipLaunchKernelGGL((gemm_large_kernel<PLANES, EPI, 1>), grid, dim3(512), 0, s, part, stride, xp, wp, RB, N, KT,
                           n_splits, counters, epi, x_off, slice_ng);
      else
        hipLaunchKernelGGL((gemm_large_kernel<PLANES, EPI, 2>), grid, dim3(512), 0, s, part, stride, xp, wp, RB, N, KT,
                           n_splits, counters, epi, x_off, slice_ng);
    };
    if (plan.x_main > 0) {
      // whole rounds unsplit, then the remaining feature tiles with k split so that they fill one more round
      const int rem_ng = NG - plan.x_main * LARGE_FEAT_GROUPS;
      go(dim3(plan.x_main, 1, Z), part_stride, 1, 0, NG);
      go(dim3(X - plan.x_main, plan.rem_splits, Z), (int64_t)RB * 16 * rem_ng * (16 * TN), plan.rem_splits, plan.x_main, rem_ng);
    } else {
      go(dim3(X, splits, Z), part_stride, splits, 0, NG);
    }
    return true;
  }
  // the logits epilogues read a single plane only where the projection is matrix-bound (the large-row kernel above)
  if constexpr (PLANES == 1 && (EPI == EPI_LOGITS || EPI == EPI_TOP2)) {
    return false;
  } else {
  const bool once = RB == 4;  // one 64-row group: every weight byte is read once
#define DED_SKINNY(KERNEL, A, GRID, THREADS)                                                          \
  if (once) hipLaunchKernelGGL((KERNEL<A, PLANES, EPI, true>), GRID, dim3(THREADS), 0, s, DED_ARGS);   \
  else hipLaunchKernelGGL((KERNEL<A, PLANES, EPI, false>), GRID, dim3(THREADS), 0, s, DED_ARGS);
  if (plan.nwn == 0) {
    if (nw == 4) { DED_SKINNY(gemm_stream_kernel, 4, grid_stream, 256) }
    else if (nw == 2) { DED_SKINNY(gemm_stream_kernel, 2, grid_stream, 128) }
    else { DED_SKINNY(gemm_stream_kernel, 1, grid_stream, 64) }
    return true;
  }
  if (plan.nwn == 4) { DED_SKINNY(gemm_wide_kernel, 4, grid_wide, 512) }
  else if (plan.nwn == 3) { DED_SKINNY(gemm_wide_kernel, 3, grid_wide, 384) }
  else if (plan.nwn == 2) { DED_SKINNY(gemm_wide_kernel, 2, grid_wide, 256) }
  else return false;
#undef DED_SKINNY
#undef DED_ARGS
  return true;
  }
}

}  // namespace

GemmPlan bf16_gemm_plan(int rows_pad, int N, int K, int planes, int max_splits) {
  static const Tune tune;
  const int NG = (N + 16 * TN - 1) / (16 * TN), groups = K / (32 * PD), rg = rows_pad / 64;
  const int64_t w_bytes = (int64_t)NG * 64 * K * 2, slice = (int64_t)rows_pad * N * 4;
  if (rows_pad >= 256) {  // matrix-core bound: the large-row kernel
    // One workgroup per CU is resident, so a launch runs in ceil(workgroups / CUs) rounds.
    // Two wavefront tiles: one feature group per wavefront (256 features x 128 rows per workgroup: more workgroups)
    // or two (256 x 256: a quarter to a third fewer LDS bytes per matrix instruction, which is what bounds this
    // kernel; measured 15-18 % faster at equal CU filling with two-plane inputs, ~30 % with single-plane ones, whose
    // small tile reads twice the LDS bytes per matrix instruction).  k is split only as far as it takes to fill the
    // last round (a split costs its slices: ~15 % per extra slice).  From 512 rows both tiles are weighed; the narrow
    // single-plane projections (N = d) keep the small one - the large tile leaves them so few workgroups that k has
    // to be split, which measured slower (Llama-3-8B shape, 2048 rows: O 101 -> 130 us) -, the LM head takes the
    // large one (3.1 -> 2.2 ms per step at that shape).
    GemmPlan best{8, 1, 1};
    double best_cost = 1e300;
    for (int gpw = 1; gpw <= (rows_pad >= 512 ? 2 : 1); ++gpw) {
      const int tiles = ((NG + LARGE_FEAT_GROUPS - 1) / LARGE_FEAT_GROUPS) *
                        ((rows_pad + 64 * large_row_groups(gpw) - 1) / (64 * large_row_groups(gpw)));
      for (int s = 1; s <= 4 && s <= max_splits && s <= groups; ++s) {
        const int wgs = tiles * s, rounds = (wgs + kCUs - 1) / kCUs;
        const double c = (double)rounds * kCUs / wgs * (1.0 + 0.15 * (s - 1)) * (gpw == 1 ? 1.15 : 1.0);
        if (c < best_cost) {
          best_cost = c;
          best = GemmPlan{7 + gpw, 1, s};
        }
      }
      // A last round that is at most half full: the whole rounds stay unsplit and only the feature tiles of the
      // last one split k, 2 - 4 ways, into one more (shorter) round of their own (a second launch).  The cut has to
      // fall between feature tiles: whole rounds x CUs must be a multiple of the row tiles.
      const int X = (NG + LARGE_FEAT_GROUPS - 1) / LARGE_FEAT_GROUPS, Z = tiles / X, full = tiles / kCUs;
      if (max_splits >= 2 && full >= 1 && (full * kCUs) % Z == 0 && full * kCUs < tiles) {
        const int x_main = full * kCUs / Z, rem = tiles - full * kCUs;
        const int rs = std::min(std::min(4, groups), kCUs / rem);
        if (rs >= 2) {
          const double c = (full + (1.0 + 0.15 * (rs - 1)) / rs + 0.05) * kCUs / tiles * (gpw == 1 ? 1.15 : 1.0);
          if (c < best_cost) {
            best_cost = c;
            best = GemmPlan{7 + gpw, 1, 1};
            best.x_main = x_main;
            best.rem_splits = rs;
          }
        }
      }
    }
    return best;
  }
  GemmPlan best{0, 1, 1};
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
        x_per_w = (double)planes / nwn + 0.7;  // + barriers and LDS traffic of the wide kernel (calibrated)
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

int bf16_gemm_tiles(int rows_pad, int N, const GemmPlan& plan) {
  const int NG = (N + 16 * TN - 1) / (16 * TN);
  if (plan.nwn >= 8) {
    const int rgs = large_row_groups(plan.nwn - 7);
    return ((NG + LARGE_FEAT_GROUPS - 1) / LARGE_FEAT_GROUPS) * ((rows_pad + 64 * rgs - 1) / (64 * rgs));
  }
  const int gx = plan.nwn == 0 ? NG : (NG + plan.nwn - 1) / plan.nwn;
  return gx * (rows_pad / 64);
}

bool bf16_gemm(float* part, int64_t part_stride, const bf16_t* x_packed, const bf16_t* w_packed, int rows_pad,
               int N, int K, int planes, const GemmPlan& plan, int* counters, const GemmEpilogue& epi,
               hipStream_t s) {
  if (rows_pad <= 0 || rows_pad % 64 || N % 16 || K % (32 * PD) || (planes != 1 && planes != 2)) return false;
  const int RB = rows_pad / 16, KT = K / 32, groups = KT / PD;
  const int NG = (N + 16 * TN - 1) / (16 * TN);
  const int splits = plan.splits;
  if (splits < 1 || splits > groups || !counters) return false;
  if (plan.nwn != 0 && plan.nwn < 8 && groups / splits < 2) return false;
  if (plan.nwn > 9) return false;
  if (plan.x_main > 0) {  // remainder launch: its 2 - 4 compact slices must fit into one slice of the whole matrix
    const int X = (NG + LARGE_FEAT_GROUPS - 1) / LARGE_FEAT_GROUPS;
    if (plan.nwn < 8 || splits != 1 || plan.x_main >= X || plan.rem_splits < 2 || plan.rem_splits > 4 ||
        plan.rem_splits > groups)
      return false;
    const int64_t rem_ng = NG - (int64_t)plan.x_main * LARGE_FEAT_GROUPS;
    if (plan.rem_splits * rows_pad * rem_ng * (16 * TN) > part_stride) return false;
  }
  if (splits > 1 && part_stride < (int64_t)rows_pad * NG * 16 * TN) return false;
  if ((epi.kind == EPI_RESIDUAL || epi.kind == EPI_QKV || epi.kind == EPI_SILU) && N % 64) return false;
  int nw = plan.nw >= 4 ? 4 : plan.nw >= 2 ? 2 : 1;
  while (nw > 1 && splits * nw > groups) nw /= 2;  // every wavefront needs at least one k group
  const uint4* xp = reinterpret_cast<const uint4*>(x_packed);
  const uint4* wp = reinterpret_cast<const uint4*>(w_packed);
  dim3 gs(NG, splits, RB / 4), gw(plan.nwn ? (NG + plan.nwn - 1) / plan.nwn : 1, splits, RB / 4);
#define DED_GO(P, E) return launch_shape<P, E>(plan, gs, gw, part, part_stride, xp, wp, RB, N, KT, counters, epi, nw, s)
  switch (epi.kind) {
    case EPI_LOGITS:
      if (planes == 2) DED_GO(2, EPI_LOGITS);
      if (plan.nwn >= 8) DED_GO(1, EPI_LOGITS);
      return false;
    case EPI_TOP2:
      if (planes == 2) DED_GO(2, EPI_TOP2);
      if (plan.nwn >= 8) DED_GO(1, EPI_TOP2);
      return false;
    case EPI_QKV:
      if (planes == 2) DED_GO(2, EPI_QKV);
      return false;
    case EPI_SILU:
      if (planes == 2) DED_GO(2, EPI_SILU);
      return false;
    case EPI_RESIDUAL:
      if (planes == 1) DED_GO(1, EPI_RESIDUAL);
      return false;
  }
#undef DED_GO
  return false;
}

}  // namespace ded
