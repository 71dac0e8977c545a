// 16-bit path, what is neither a contraction nor a GEMM epilogue: weight re-layout, embedding gather,
// cache compaction and the plain <-> fragment layout conversions.  Number formats: see bf16_layout.h.
#include <algorithm>

#include "bf16_layout.h"
#include "ded_kernels.h"

namespace ded {

namespace {

__device__ inline float wave_sum(float v) {
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ inline float block_sum_256(float v, float* sh) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  return sh[0] + sh[1] + sh[2] + sh[3];
}

struct F8 {
  float v[8];
};
__device__ inline F8 load8(const float* p) {
  F8 r;
  float4 a = *reinterpret_cast<const float4*>(p);
  float4 b = *reinterpret_cast<const float4*>(p + 4);
  r.v[0] = a.x; r.v[1] = a.y; r.v[2] = a.z; r.v[3] = a.w;
  r.v[4] = b.x; r.v[5] = b.y; r.v[6] = b.z; r.v[7] = b.w;
  return r;
}
__device__ inline void store8(float* p, const F8& r) {
  *reinterpret_cast<float4*>(p) = make_float4(r.v[0], r.v[1], r.v[2], r.v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(r.v[4], r.v[5], r.v[6], r.v[7]);
}
__device__ inline uint32_t pk(uint16_t lo, uint16_t hi) { return (uint32_t)lo | ((uint32_t)hi << 16); }
// eight floats -> eight f16 (one 16-byte unit)
__device__ inline uint4 to_f16x8(const F8& r) {
  return make_uint4(pk(f32_to_f16(r.v[0]), f32_to_f16(r.v[1])), pk(f32_to_f16(r.v[2]), f32_to_f16(r.v[3])),
                    pk(f32_to_f16(r.v[4]), f32_to_f16(r.v[5])), pk(f32_to_f16(r.v[6]), f32_to_f16(r.v[7])));
}
// eight floats -> hi and lo planes
__device__ inline void to_f16x8_split(const F8& r, uint4& hi, uint4& lo) {
  uint16_t h[8], l[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) split_f16(r.v[i], h[i], l[i]);
  hi = make_uint4(pk(h[0], h[1]), pk(h[2], h[3]), pk(h[4], h[5]), pk(h[6], h[7]));
  lo = make_uint4(pk(l[0], l[1]), pk(l[2], l[3]), pk(l[4], l[5]), pk(l[6], l[7]));
}
// sum over split-K slices in slice order (fixed order -> deterministic)
__device__ inline F8 sum_parts8(const float* part, int n_part, int64_t part_stride, int64_t off) {
  F8 acc = load8(part + off);
  for (int s = 1; s < n_part; ++s) {
    F8 t = load8(part + (int64_t)s * part_stride + off);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc.v[i] += t.v[i];
  }
  return acc;
}

}  // namespace

// ------------------------------------------------------------------------------------------
// Source feature of packed feature n (see PERM_* in ded_kernels.h).  F = half the row count for PERM_GATE_UP.
__device__ inline int packw_source_row(int n, int perm, int F) {
  if (perm == PERM_NONE) return n;
  const int t = (n >> 4) & 3, e = n & 15;
  if (perm == PERM_ROPE) {  // per 128-dim head: group j holds dims [32j, 32j+32) and their partners + 64
    const int head = n >> 7, j = (n >> 6) & 1;
    const int dim = 32 * j + 16 * (t & 1) + e + (t >= 2 ? 64 : 0);
    return head * 128 + dim;
  }
  const int f = 32 * (n >> 6) + 16 * (t & 1) + e;  // PERM_GATE_UP: gate f in tiles 0,1, up f in tiles 2,3
  return t >= 2 ? F + f : f;
}

// dst: PackW (f16) with the feature count padded to a multiple of 64 (padding features are zero)
__global__ void pack_weight_kernel(uint4* __restrict__ dst, const bf16_t* __restrict__ src, int N, int K, int perm) {
  int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // destination 16-byte unit
  int64_t total = (int64_t)((N + 63) / 64 * 64) * K / 8;
  if (u >= total) return;
  int lane = (int)(u & 63);
  int64_t frag = u >> 6;
  int KT = K >> 5;
  int t = (int)(frag % PACKW_TILES);
  int64_t gk = frag / PACKW_TILES;
  int kt = (int)(gk % KT), ng = (int)(gk / KT);
  int n = ng * 64 + t * 16 + (lane & 15);
  int k = kt * 32 + (lane >> 4) * 8;
  uint4 out = make_uint4(0, 0, 0, 0);
  if (n < N) {
    int row = packw_source_row(n, perm, N / 2);
    uint4 in = *reinterpret_cast<const uint4*>(src + (int64_t)row * K + k);
    uint32_t w[4] = {in.x, in.y, in.z, in.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = pk(bf16_to_f16((uint16_t)(w[i] & 0xffffu)), bf16_to_f16((uint16_t)(w[i] >> 16)));
    out = make_uint4(w[0], w[1], w[2], w[3]);
  }
  dst[u] = out;
}
void bf16_pack_weight(bf16_t* dst, const bf16_t* src, int N, int K, int perm, hipStream_t s) {
  int64_t units = (int64_t)((N + 63) / 64 * 64) * K / 8;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s,
                     reinterpret_cast<uint4*>(dst), src, N, K, perm);
}

// ------------------------------------------------------------------------------------------
// Embedding gather: x = emb[token] (fp32 residual stream), y = (x * gain) as hi/lo f16 in PackX for the first
// GEMM, ssq[r][g] = sum of x^2 over the 64 features of group g (the consumer turns that into 1/rms).
__global__ __launch_bounds__(256) void bf16_embed_kernel(float* __restrict__ x, uint4* __restrict__ y,
                                                         float* __restrict__ ssq, const bf16_t* __restrict__ emb,
                                                         const float* __restrict__ gain,
                                                         const int32_t* __restrict__ token, int rows, int RB, int d) {
  int r = blockIdx.x;
  const bool real = r < rows;  // padding rows (up to the 64-row granule of the GEMMs) are cleared
  const bf16_t* src = emb + (int64_t)(real ? token[r] : 0) * d;
  for (int u = threadIdx.x; u < d / 8; u += 256) {  // d % 64 == 0: whole wavefront iterations only
    uint4 in = real ? *reinterpret_cast<const uint4*>(src + u * 8) : make_uint4(0, 0, 0, 0);
    uint32_t w[4] = {in.x, in.y, in.z, in.w};
    F8 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v.v[2 * i] = bf16_to_f32((uint16_t)(w[i] & 0xffffu));
      v.v[2 * i + 1] = bf16_to_f32((uint16_t)(w[i] >> 16));
    }
    store8(x + (int64_t)r * d + u * 8, v);
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) ss += v.v[i] * v.v[i];
    ss += __shfl_xor(ss, 1);  // 8 consecutive lanes = one 64-feature group
    ss += __shfl_xor(ss, 2);
    ss += __shfl_xor(ss, 4);
    if ((threadIdx.x & 7) == 0) ssq[(int64_t)r * (d / 64) + (u >> 3)] = ss;
    F8 g = load8(gain + u * 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) v.v[i] *= g.v[i];
    uint4 hi, lo;
    to_f16x8_split(v, hi, lo);
    y[packx_index(r, u * 8, RB, 0) >> 3] = hi;
    y[packx_index(r, u * 8, RB, 1) >> 3] = lo;
  }
}
void bf16_embed(float* x, bf16_t* y_packed, float* ssq, const bf16_t* emb, const float* gain, const StepMeta& m,
                int rows_pad, int d, hipStream_t s) {
  hipLaunchKernelGGL(bf16_embed_kernel, dim3(rows_pad), dim3(256), 0, s, x, reinterpret_cast<uint4*>(y_packed), ssq, emb,
                     gain, m.token, m.rows, rows_pad / 16, d);
}

// ------------------------------------------------------------------------------------------
// Compaction in the fragment layouts.  Threads 0..15 move the sixteen 16-byte key units of a slot,
// threads 16..143 one value element each; every thread walks the path upwards (see the fp32 kernel).
__global__ __launch_bounds__(192) void bf16_kv_compact_kernel(bf16_t* const* __restrict__ kc,
                                                              bf16_t* const* __restrict__ vc,
                                                              const int32_t* __restrict__ path,
                                                              const int32_t* __restrict__ n_acc,
                                                              const int32_t* __restrict__ seq_p, int Hkv, int cap,
                                                              int stride) {
  const int hd = 128;
  int layer = blockIdx.x, bh = blockIdx.y;
  int b = bh / Hkv;
  int len = n_acc[b], P = seq_p[b];
  const int32_t* pth = path + (int64_t)b * stride;
  int t = threadIdx.x;
  if (t < 16) {
    bf16_t* K = kc[layer] + (int64_t)bh * cap * hd;
    for (int j = 0; j < len; ++j) {
      int src = pth[j];
      if (src != j)
        *reinterpret_cast<uint4*>(K + packk_index(P + j, t * 8)) =
            *reinterpret_cast<const uint4*>(K + packk_index(P + src, t * 8));
    }
  } else if (t < 16 + hd) {
    bf16_t* V = vc[layer] + (int64_t)bh * cap * hd;
    int hdim = t - 16;
    for (int j = 0; j < len; ++j) {
      int src = pth[j];
      if (src != j) V[packvt_index(P + j, hdim)] = V[packvt_index(P + src, hdim)];
    }
  }
}
void bf16_kv_compact(bf16_t* const* kc, bf16_t* const* vc, const int32_t* path, const int32_t* n_acc,
                     const StepMeta& m, const ModelDims& md, int stride, hipStream_t s) {
  hipLaunchKernelGGL(bf16_kv_compact_kernel, dim3(md.n_layers, m.batch * md.Hkv), dim3(192), 0, s, kc, vc, path,
                     n_acc, m.seq_p, md.Hkv, md.cap, stride);
}

// ------------------------------------------------------------------------------------------
// plain bf16 [Hkv][n][hd]  <->  f16 cache fragments (to the cache: exact widening; back: round to bf16)
__global__ void bf16_kv_copy_kernel(bf16_t* __restrict__ kcache, bf16_t* __restrict__ vcache,
                                    bf16_t* __restrict__ kp, bf16_t* __restrict__ vp, int to_cache, int seq,
                                    int first, int n, int Hkv, int cap) {
  const int hd = 128;
  int j = blockIdx.x, g = blockIdx.y, i = threadIdx.x;
  int64_t cbase = ((int64_t)seq * Hkv + g) * cap * hd;
  int64_t pidx = ((int64_t)g * n + j) * hd + i;
  int64_t ki = cbase + packk_index(first + j, i), vi = cbase + packvt_index(first + j, i);
  if (to_cache) {
    if (kp) kcache[ki] = bf16_to_f16(kp[pidx]);
    if (vp) vcache[vi] = bf16_to_f16(vp[pidx]);
  } else {
    if (kp) kp[pidx] = f32_to_bf16(f16_to_f32(kcache[ki]));
    if (vp) vp[pidx] = f32_to_bf16(f16_to_f32(vcache[vi]));
  }
}
void bf16_kv_copy(bf16_t* kcache, bf16_t* vcache, bf16_t* k_plain, bf16_t* v_plain, bool to_cache, int seq,
                  int first, int n, const ModelDims& md, hipStream_t s) {
  if (n <= 0) return;
  hipLaunchKernelGGL(bf16_kv_copy_kernel, dim3(n, md.Hkv), dim3(128), 0, s, kcache, vcache, k_plain, v_plain,
                     to_cache ? 1 : 0, seq, first, n, md.Hkv, md.cap);
}

// zero the slots [first, first + n) of one sequence (keys and values) in the fragment layouts
__global__ void bf16_kv_clear_kernel(bf16_t* __restrict__ kcache, bf16_t* __restrict__ vcache, int seq, int first,
                                     int Hkv, int cap) {
  const int hd = 128;
  int j = blockIdx.x, g = blockIdx.y, i = threadIdx.x;
  int64_t cbase = ((int64_t)seq * Hkv + g) * cap * hd;
  kcache[cbase + packk_index(first + j, i)] = 0;
  vcache[cbase + packvt_index(first + j, i)] = 0;
}
void bf16_kv_clear(bf16_t* kcache, bf16_t* vcache, int seq, int first, int n, const ModelDims& md, hipStream_t s) {
  if (n <= 0) return;
  hipLaunchKernelGGL(bf16_kv_clear_kernel, dim3(n, md.Hkv), dim3(128), 0, s, kcache, vcache, seq, first, md.Hkv, md.cap);
}

__global__ void bf16_scatter_tree_kv_kernel(bf16_t* __restrict__ kc, bf16_t* __restrict__ vc,
                                            const bf16_t* __restrict__ kt, const bf16_t* __restrict__ vt,
                                            const int32_t* __restrict__ seq_p, const int32_t* __restrict__ seq_n,
                                            int Hkv, int cap, int max_nodes) {
  const int hd = 128;
  int node = blockIdx.x, bh = blockIdx.y, i = threadIdx.x;
  int b = bh / Hkv;
  if (node >= seq_n[b]) return;
  int64_t src = ((int64_t)bh * max_nodes + node) * hd + i;
  int64_t cbase = (int64_t)bh * cap * hd;
  int slot = seq_p[b] + node;
  kc[cbase + packk_index(slot, i)] = bf16_to_f16(kt[src]);
  vc[cbase + packvt_index(slot, i)] = bf16_to_f16(vt[src]);
}
void bf16_scatter_tree_kv(bf16_t* kc, bf16_t* vc, const bf16_t* k_tree, const bf16_t* v_tree, const StepMeta& m,
                          const ModelDims& md, int max_nodes, hipStream_t s) {
  hipLaunchKernelGGL(bf16_scatter_tree_kv_kernel, dim3(max_nodes, m.batch * md.Hkv), dim3(128), 0, s, kc, vc,
                     k_tree, v_tree, m.seq_p, m.seq_n, md.Hkv, md.cap, max_nodes);
}

// q plain bf16 [B][max_nodes][H][hd] -> PackQ (hi = exact f16, lo = 0; rows of absent nodes become zero)
__global__ void bf16_pack_q_kernel(bf16_t* __restrict__ qp, const bf16_t* __restrict__ q,
                                   const int32_t* __restrict__ seq_n, int n_step, int H, int Hkv, int max_nodes) {
  const int hd = 128;
  int r = blockIdx.x, h = blockIdx.y, i = threadIdx.x;
  int b = r / n_step, node = r - b * n_step;
  int G = H / Hkv, kvh = h / G, g = h - kvh * G;
  uint16_t hi = 0, lo = 0;
  if (node < seq_n[b]) split_f16(bf16_to_f32(q[(((int64_t)b * max_nodes + node) * H + h) * hd + i]), hi, lo);
  bf16_t* base = qp + ((int64_t)b * Hkv + kvh) * ((int64_t)G * n_step * hd * 2);
  base[packq_index(g * n_step + node, i, 0)] = hi;
  base[packq_index(g * n_step + node, i, 1)] = lo;
}
void bf16_pack_q(bf16_t* q_packed, const bf16_t* q_plain, const StepMeta& m, const ModelDims& md, int max_nodes,
                 hipStream_t s) {
  hipLaunchKernelGGL(bf16_pack_q_kernel, dim3(m.rows, md.H), dim3(128), 0, s, q_packed, q_plain, m.seq_n, m.n_step,
                     md.H, md.Hkv, max_nodes);
}

// PackX(o) hi + lo [rows_pad][H*hd] -> plain bf16 [B][max_nodes][H][hd]
__global__ void bf16_unpack_o_kernel(bf16_t* __restrict__ out, const bf16_t* __restrict__ op,
                                     const int32_t* __restrict__ seq_n, int n_step, int H, int RB, int max_nodes) {
  const int hd = 128;
  int r = blockIdx.x, h = blockIdx.y, i = threadIdx.x;
  int b = r / n_step, node = r - b * n_step;
  if (node >= seq_n[b]) return;
  float v = f16_to_f32(op[packx_index(r, h * hd + i, RB, 0)]) + f16_to_f32(op[packx_index(r, h * hd + i, RB, 1)]);
  out[(((int64_t)b * max_nodes + node) * H + h) * hd + i] = f32_to_bf16(v);
}
void bf16_unpack_o(bf16_t* out_plain, const bf16_t* o_packed, int rows_pad, const StepMeta& m, const ModelDims& md,
                   int max_nodes, hipStream_t s) {
  hipLaunchKernelGGL(bf16_unpack_o_kernel, dim3(m.rows, md.H), dim3(128), 0, s, out_plain, o_packed, m.seq_n,
                     m.n_step, md.H, rows_pad / 16, max_nodes);
}

}  // namespace ded
