// Tree-masked attention for the 16-bit path (f16 K/V cache, head_dim 128), split over the key axis.
//
// Work unit: (sequence, kv head, tile of 64 "virtual rows", key range).  The virtual rows of a kv head
// are its G query heads x n_step tree rows (vr = g * n_step + node), so grouped-query heads share
// every K/V byte that is fetched.  A workgroup of 4 wavefronts streams its key range in tiles of 64
// keys: the K and V^T fragments of a tile (32 KiB, contiguous in the cache) are fetched with fully
// coalesced 16-byte loads, parked in LDS (double buffered) and consumed by all four wavefronts, each
// of which owns 16 of the 64 rows:
//     S^T = K . Q^T           v_mfma_f32_16x16x32_f16, A = key fragment (LDS), B = query fragment (VGPR)
//     online soft-max          per lane: 1 row, 16 keys of the tile; row max via two wavefront shuffles
//     O^T += V^T . P^T         A = value fragment (LDS), B = probabilities straight from the S^T registers
// The key rows of a 32-key group are interleaved inside the two 16-row tiles (see packk_index) so that
// after the first product a lane holds 8 consecutive keys - exactly the B-operand slice the second
// product needs, with no cross-lane traffic.  The ancestor mask is a per-row bitmask over tree slots;
// tiles that lie entirely inside the prefix skip all mask work.
// Each workgroup writes (running max, sum, unnormalised output) per row; a second kernel merges the
// key ranges in a fixed order and writes the output as hi/lo f16 in PackX for the O projection.
#include <algorithm>

#include "bf16_layout.h"
#include "ded_kernels.h"

namespace ded {

namespace {

constexpr int TILE = 64;         // keys per tile
constexpr int TILE_U4 = 1024;    // uint4 units of one K (or V) tile: 64 keys * 128 dims * 2 B / 16
constexpr float NEG_BIG = -1.0e30f;

#ifdef DED_ATTN_TRACE
__device__ unsigned long long* g_atrace = nullptr;  // [workgroup][4] wall-clock stamps (debug builds only)
#define DED_ASTAMP(i)                                                                                         \
  if (g_atrace && threadIdx.x == 0)                                                                           \
    g_atrace[(((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 4 + (i)] = wall_clock64();
__device__ unsigned long long* g_aphase = nullptr;  // [workgroup][4] accumulated phase times of wave 0
#define DED_APHASE_DECL unsigned long long ph_t = 0, ph_acc[4] = {0, 0, 0, 0};
#define DED_APHASE_START ph_t = wall_clock64();
#define DED_APHASE(i) { unsigned long long now_ = wall_clock64(); ph_acc[i] += now_ - ph_t; ph_t = now_; }
#define DED_APHASE_FLUSH                                                                                      \
  if (g_aphase && threadIdx.x == 0)                                                                           \
    for (int i_ = 0; i_ < 4; ++i_)                                                                            \
      g_aphase[(((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 4 + i_] = ph_acc[i_];
#else
#define DED_ASTAMP(i)
#define DED_APHASE_DECL
#define DED_APHASE_START
#define DED_APHASE(i)
#define DED_APHASE_FLUSH
#endif

__global__ __launch_bounds__(256) void tree_attn_partial_kernel(
    const uint4* __restrict__ qp, const uint4* __restrict__ kc, const uint4* __restrict__ vc,
    float* __restrict__ part_o, float2* __restrict__ part_ml, const uint64_t* __restrict__ mask,
    const int32_t* __restrict__ seq_p, const int32_t* __restrict__ seq_n, int n_step, int H, int Hkv, int cap,
    int n_splits, float scale_log2e) {
  __shared__ uint4 lds[2][2 * TILE_U4];  // [buffer][K tile | V tile], 2 x 32 KiB
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int split = blockIdx.x, row_tile = blockIdx.y, bz = blockIdx.z;
  const int b = bz / Hkv, kvh = bz - b * Hkv;
  const int G = H / Hkv;
  const int P = seq_p[b], N = seq_n[b], T = P + N;
  const int n_tiles = (T + TILE - 1) / TILE;
  // key ranges of equal cost: a tile that holds tree keys (mask work) counts as two prefix tiles
  const int n_plain = P / TILE;  // tiles entirely inside the prefix
  const int cost_total = n_plain + 2 * (n_tiles - n_plain);
  auto tile_at_cost = [&](int c) { return c <= n_plain ? c : n_plain + (c - n_plain + 1) / 2; };
  const int t_begin = tile_at_cost((int)((int64_t)split * cost_total / n_splits));
  const int t_end = split + 1 == n_splits ? n_tiles : tile_at_cost((int)((int64_t)(split + 1) * cost_total / n_splits));
  const int VR = G * n_step;
  const int vrb = row_tile * 4 + wave;
  const bool active = vrb * 16 < VR;  // wavefront owns real rows
  const int vr = vrb * 16 + (lane & 15);
  const int quad = lane >> 4;
  const int g = active ? vr / n_step : 0;
  const int node = active ? vr - g * n_step : 0;
  const uint4* kbase = kc + (int64_t)bz * cap * 16;  // 16 uint4 per key
  const uint4* vbase = vc + (int64_t)bz * cap * 16;

  // global -> register -> LDS staging of one tile (kept in eight named registers per thread)
  struct Stage {
    uint4 k0, k1, k2, k3, v0, v1, v2, v3;
  };
  auto load_tile = [&](int t) {
    const uint4* ks = kbase + (int64_t)t * TILE_U4 + tid;
    const uint4* vs = vbase + (int64_t)t * TILE_U4 + tid;
    Stage st;
    st.k0 = ks[0];
    st.k1 = ks[256];
    st.k2 = ks[512];
    st.k3 = ks[768];
    st.v0 = vs[0];
    st.v1 = vs[256];
    st.v2 = vs[512];
    st.v3 = vs[768];
    return st;
  };
  // the first tile is requested before anything else (mask row, queries): it has the longest way to come
  Stage st_first;
  if (t_begin < t_end) st_first = load_tile(t_begin);

  // this lane's row of the ancestor bitmask (4 words cover 256 tree slots), kept in registers
  const uint64_t* mrow = mask + ((int64_t)b * n_step + node) * 4;
  const uint64_t mw0 = mrow[0], mw1 = mrow[1], mw2 = mrow[2], mw3 = mrow[3];

  f16x8_t q[8];  // [head-dim chunk kk][plane hi / lo]
  if (active) {
    const uint4* qsrc = qp + (((int64_t)bz * (VR / 16) + vrb) * 8 << 6) + lane;
#pragma unroll
    for (int i = 0; i < 8; ++i) q[i] = __builtin_bit_cast(f16x8_t, qsrc[i << 6]);
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) q[i] = __builtin_bit_cast(f16x8_t, make_uint4(0, 0, 0, 0));
  }

  f32x4_t o[8];
#pragma unroll
  for (int hb = 0; hb < 8; ++hb) o[hb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float m_run = NEG_BIG, l_run = 0.f;

  auto store_tile = [&](int buf, const Stage& st) {
    uint4* d = lds[buf] + tid;
    d[0] = st.k0;
    d[256] = st.k1;
    d[512] = st.k2;
    d[768] = st.k3;
    d[TILE_U4] = st.v0;
    d[TILE_U4 + 256] = st.v1;
    d[TILE_U4 + 512] = st.v2;
    d[TILE_U4 + 768] = st.v3;
  };

  DED_APHASE_DECL
  auto compute_tile = [&](int buf, int t) {
    DED_APHASE_START
    const uint4* lk = lds[buf];
    const uint4* lv = lds[buf] + TILE_U4;
    // S^T: s[kb][c][i] = score of key  t*64 + kb*32 + quad*8 + c*4 + i  against this lane's row
    f32x4_t s[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
        f32x4_t acc_lo = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          f16x8_t a = __builtin_bit_cast(f16x8_t, lk[(((kb * 2 + c) * 4 + kk) << 6) + lane]);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, q[2 * kk], acc, 0, 0, 0);
          acc_lo = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, q[2 * kk + 1], acc_lo, 0, 0, 0);
        }
        s[kb][c] = acc + acc_lo;
      }
    DED_APHASE(0)
    const int key0 = t * TILE;
    float p[2][8];
    float mx = NEG_BIG;
    if (key0 + TILE <= P) {  // whole tile inside the prefix: every key visible
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          p[kb][j] = s[kb][j >> 2][j & 3] * scale_log2e;
          mx = fmaxf(mx, p[kb][j]);
        }
    } else {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          int key = key0 + kb * 32 + quad * 8 + j;
          const int tt = key - P;  // tree slot of this key (negative inside the prefix)
          const int wi = tt >> 6;
          const uint64_t word = wi == 0 ? mw0 : wi == 1 ? mw1 : wi == 2 ? mw2 : mw3;
          const bool vis = (key < P) | ((key < T) & (bool)((word >> (tt & 63)) & 1ull));  // no short circuit: no branches
          float v = vis ? s[kb][j >> 2][j & 3] * scale_log2e : NEG_BIG;
          p[kb][j] = v;
          mx = fmaxf(mx, v);
        }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    float lsum = 0.f;
    f16x8_t pb[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float e = p[kb][j] > 0.5f * NEG_BIG ? __builtin_amdgcn_exp2f(p[kb][j] - m_new) : 0.f;
        _Float16 h = (_Float16)e;
        lsum += (float)h;  // the sum uses the rounded weights the product uses
        pb[kb][j] = h;
      }
    }
    l_run = l_run * alpha + lsum;
    m_run = m_new;
    DED_APHASE(1)
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int hb = 0; hb < 8; ++hb) o[hb] *= alpha;
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int hb = 0; hb < 8; ++hb) {
        f16x8_t a = __builtin_bit_cast(f16x8_t, lv[((kb * 8 + hb) << 6) + lane]);
        o[hb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, pb[kb], o[hb], 0, 0, 0);
      }
    DED_APHASE(2)
  };

  DED_ASTAMP(0)
  if (t_begin < t_end) {
    store_tile(0, st_first);
    __syncthreads();
    DED_ASTAMP(1)
    int buf = 0;
    for (int t = t_begin; t < t_end; ++t) {
      // the last iteration re-fetches its own tile (in bounds, L2 hit) so that the loop body is branch free
      const int t_next = t + 1 < t_end ? t + 1 : t;
      Stage st = load_tile(t_next);
      if (active) compute_tile(buf, t);
      store_tile(buf ^ 1, st);
      __syncthreads();
      buf ^= 1;
    }
  }

  DED_ASTAMP(2)
  DED_APHASE_FLUSH
  if (active) {
    float l = l_run;
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    const int h = kvh * G + g;
    const int64_t prow = (((int64_t)b * H + h) * n_splits + split) * n_step + node;
    float* po = part_o + prow * 128 + quad * 4;
#pragma unroll
    for (int hb = 0; hb < 8; ++hb)
      *reinterpret_cast<float4*>(po + hb * 16) = make_float4(o[hb][0], o[hb][1], o[hb][2], o[hb][3]);
    if (quad == 0) part_ml[prow] = make_float2(m_run, l);
  }
  DED_ASTAMP(3)
}

// One thread per (row, query head, 4 head dims).  The key ranges are folded in index order, eight at a time, with
// all loads of a batch of eight in flight together; the result does not depend on the launch shape.
__global__ __launch_bounds__(256) void tree_attn_merge_kernel(bf16_t* __restrict__ op, int RB,
                                                              const float* __restrict__ part_o,
                                                              const float2* __restrict__ part_ml, int n_splits,
                                                              int n_step, int H, int total) {
  const int gid = blockIdx.x * 256 + threadIdx.x;
  if (gid >= total) return;
  const int d4 = gid & 31, rh = gid >> 5;
  const int r = rh / H, h = rh - r * H;
  const int b = r / n_step, node = r - b * n_step;
  const int64_t base = (((int64_t)b * H + h) * n_splits) * n_step + node;
  float M = NEG_BIG, L = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s0 = 0; s0 < n_splits; s0 += 8) {
    float2 ml[8];
    float4 po[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int64_t row = base + (int64_t)min(s0 + j, n_splits - 1) * n_step;  // clamped: in bounds, weight 0 below
      ml[j] = part_ml[row];
      po[j] = *reinterpret_cast<const float4*>(part_o + row * 128 + d4 * 4);
    }
    float Mc = M;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (s0 + j < n_splits) Mc = fmaxf(Mc, ml[j].x);
    const float keep = __builtin_amdgcn_exp2f(M - Mc);
    L *= keep;
    acc.x *= keep, acc.y *= keep, acc.z *= keep, acc.w *= keep;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float w = s0 + j < n_splits ? __builtin_amdgcn_exp2f(ml[j].x - Mc) : 0.f;
      L += ml[j].y * w;
      acc.x += po[j].x * w, acc.y += po[j].y * w, acc.z += po[j].z * w, acc.w += po[j].w * w;
    }
    M = Mc;
  }
  const float inv = 1.0f / L;
  const float v[4] = {acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv};
  uint16_t hi[4], lo[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) split_f16(v[i], hi[i], lo[i]);
  // four consecutive features sit side by side inside a PackX fragment
  const int64_t ihi = packx_index(r, h * 128 + d4 * 4, RB, 0), ilo = packx_index(r, h * 128 + d4 * 4, RB, 1);
  *reinterpret_cast<uint2*>(op + ihi) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
  *reinterpret_cast<uint2*>(op + ilo) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
}

}  // namespace

int bf16_attn_pick_splits(const StepMeta& m, const ModelDims& md, int max_p, int64_t part_rows_cap) {
  const int G = md.H / md.Hkv;
  const int row_tiles = (G * m.n_step + 63) / 64;
  const int tiles = (max_p + m.n_step + TILE - 1) / TILE;
  const int base = m.batch * md.Hkv * row_tiles;
  int ns = std::max(1, 512 / std::max(base, 1));
  ns = std::min(ns, std::max(1, tiles / 2));  // keep >= 2 tiles (128 keys) per range: each range re-reads the queries
  while (ns > 1 && (int64_t)m.batch * md.H * ns * m.n_step > part_rows_cap) --ns;
  return ns;
}

void bf16_tree_attention_partial(const bf16_t* q_packed, const bf16_t* kc, const bf16_t* vc, float* part_o,
                                 float2* part_ml, int n_splits, const StepMeta& m, const ModelDims& md,
                                 hipStream_t s) {
  if (md.hd != 128 || n_splits < 1 || m.rows <= 0) return;
  const int G = md.H / md.Hkv;
  const int row_tiles = (G * m.n_step + 63) / 64;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)md.hd);
  hipLaunchKernelGGL(tree_attn_partial_kernel, dim3(n_splits, row_tiles, m.batch * md.Hkv), dim3(256), 0, s,
                     reinterpret_cast<const uint4*>(q_packed), reinterpret_cast<const uint4*>(kc),
                     reinterpret_cast<const uint4*>(vc), part_o, part_ml, m.mask, m.seq_p, m.seq_n, m.n_step, md.H,
                     md.Hkv, md.cap, n_splits, scale_log2e);
}

void bf16_tree_attention_merge(bf16_t* o_packed, int rows_pad, const float* part_o, const float2* part_ml,
                               int n_splits, const StepMeta& m, const ModelDims& md, hipStream_t s) {
  if (m.rows <= 0) return;
  const int total = m.rows * md.H * 32;
  hipLaunchKernelGGL(tree_attn_merge_kernel, dim3((total + 255) / 256), dim3(256), 0, s, o_packed, rows_pad / 16,
                     part_o, part_ml, n_splits, m.n_step, md.H, total);
}

}  // namespace ded
