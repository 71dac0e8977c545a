// fp32 storage path: plain row-major buffers, cache [B][Hkv][cap][hd].  This path serves the small
// latency-bound configurations; it is written for clarity and determinism, not for the matrix cores.
#include "ded_kernels.h"

namespace ded {

__device__ inline float wave_sum(float v) {
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ inline float wave_max(float v) {
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}

// block-wide reductions for 256 threads; `sh` needs 4 floats
__device__ inline float block_sum_256(float v, float* sh) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  return sh[0] + sh[1] + sh[2] + sh[3];
}
__device__ inline float block_max_256(float v, float* sh) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
}

// ------------------------------------------------------------------------------------------
__global__ void f32_embed_kernel(float* __restrict__ x, const float* __restrict__ emb,
                                 const int32_t* __restrict__ token, int d) {
  int r = blockIdx.x;
  const float* src = emb + (int64_t)token[r] * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) x[(int64_t)r * d + i] = src[i];
}
void f32_embed(float* x, const float* emb, const StepMeta& m, int d, hipStream_t s) {
  hipLaunchKernelGGL(f32_embed_kernel, dim3(m.rows), dim3(256), 0, s, x, emb, m.token, d);
}

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void f32_rmsnorm_kernel(float* __restrict__ y, const float* __restrict__ x,
                                                          const float* __restrict__ gain, int d, float eps) {
  __shared__ float sh[4];
  const float* xr = x + (int64_t)blockIdx.x * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) ss += xr[i] * xr[i];
  ss = block_sum_256(ss, sh);
  float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += 256) y[(int64_t)blockIdx.x * d + i] = xr[i] * inv * gain[i];
}
void f32_rmsnorm(float* y, const float* x, const float* gain, int rows, int d, float eps, hipStream_t s) {
  hipLaunchKernelGGL(f32_rmsnorm_kernel, dim3(rows), dim3(256), 0, s, y, x, gain, d, eps);
}

// ------------------------------------------------------------------------------------------
// One wavefront per (output feature n, tile of 16 rows); lanes stride over k.
__global__ __launch_bounds__(256) void f32_gemm_kernel(float* __restrict__ Y, const float* __restrict__ X,
                                                       const float* __restrict__ W, int rows, int N, int K,
                                                       int accumulate) {
  int lane = threadIdx.x & 63;
  int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  int r0 = blockIdx.y * 16;
  if (n >= N) return;
  int nr = min(16, rows - r0);
  float acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  const float* w = W + (int64_t)n * K;
  for (int k = lane; k < K; k += 64) {
    float wv = w[k];
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if (i < nr) acc[i] += wv * X[(int64_t)(r0 + i) * K + k];
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    float v = wave_sum(acc[i]);
    if (lane == 0 && i < nr) {
      int64_t o = (int64_t)(r0 + i) * N + n;
      Y[o] = accumulate ? Y[o] + v : v;
    }
  }
}
void f32_gemm(float* Y, const float* X, const float* W, int rows, int N, int K, bool accumulate, hipStream_t s) {
  if (rows <= 0) return;
  hipLaunchKernelGGL(f32_gemm_kernel, dim3((N + 3) / 4, (rows + 15) / 16), dim3(256), 0, s, Y, X, W, rows, N,
                     K, accumulate ? 1 : 0);
}

// ------------------------------------------------------------------------------------------
// Rotate q (in place) and k, append k/v of real nodes to cache slot P + node.
__global__ void f32_rope_kv_kernel(float* __restrict__ qkv, float* __restrict__ kc, float* __restrict__ vc,
                                   const float2* __restrict__ tab, const int32_t* __restrict__ seq_p,
                                   const int32_t* __restrict__ seq_n, int n_step, int H, int Hkv, int hd,
                                   int cap) {
  int r = blockIdx.x, hs = blockIdx.y;
  int b = r / n_step, node = r - b * n_step;
  int half = hd / 2;
  int width = (H + 2 * Hkv) * hd;
  float* v = qkv + (int64_t)r * width + (int64_t)hs * hd;
  bool real = node < seq_n[b];
  int64_t slot = (int64_t)seq_p[b] + node;
  if (hs < H + Hkv) {
    float* dst = nullptr;
    if (hs >= H && real) dst = kc + (((int64_t)b * Hkv + (hs - H)) * cap + slot) * hd;
    for (int i = threadIdx.x; i < half; i += blockDim.x) {
      float2 cs = tab[(int64_t)r * half + i];
      float a = v[i], c = v[i + half];
      float ra = a * cs.x - c * cs.y;
      float rc = c * cs.x + a * cs.y;
      if (hs < H) {
        v[i] = ra;
        v[i + half] = rc;
      } else if (dst) {
        dst[i] = ra;
        dst[i + half] = rc;
      }
    }
  } else if (real) {
    float* dst = vc + (((int64_t)b * Hkv + (hs - H - Hkv)) * cap + slot) * hd;
    for (int i = threadIdx.x; i < hd; i += blockDim.x) dst[i] = v[i];
  }
}
void f32_rope_kv(float* qkv, float* kc, float* vc, const float2* tab, const StepMeta& m,
                 const ModelDims& md, hipStream_t s) {
  hipLaunchKernelGGL(f32_rope_kv_kernel, dim3(m.rows, md.H + 2 * md.Hkv), dim3(64), 0, s, qkv, kc, vc, tab,
                     m.seq_p, m.seq_n, m.n_step, md.H, md.Hkv, md.hd, md.cap);
}

// ------------------------------------------------------------------------------------------
// Tree-masked attention, one workgroup per (row, query head).  Keys are taken in chunks of 1024:
// scores -> running max -> probabilities -> value accumulation (thread = (dim, key-part)).
// Needs hd <= 256 and 256 % hd == 0.
#define F32_ATT_CHUNK 1024
__global__ __launch_bounds__(256) void f32_tree_attention_kernel(
    float* __restrict__ o, const float* __restrict__ qkv, int q_stride, const float* __restrict__ kc,
    const float* __restrict__ vc, const uint64_t* __restrict__ mask, const int32_t* __restrict__ seq_p,
    const int32_t* __restrict__ seq_n, int n_step, int H, int Hkv, int hd, int cap) {
  __shared__ float sq[256];
  __shared__ float sp[F32_ATT_CHUNK];
  __shared__ float sred[4];
  __shared__ float sacc[256];
  int r = blockIdx.x, h = blockIdx.y;
  int b = r / n_step, node = r - b * n_step;
  float* out = o + ((int64_t)r * H + h) * hd;
  int nb = seq_n[b];
  if (node >= nb) {
    for (int i = threadIdx.x; i < hd; i += 256) out[i] = 0.f;
    return;
  }
  int P = seq_p[b];
  int T = P + nb;
  int g = (h * Hkv) / H;
  const float* K = kc + ((int64_t)b * Hkv + g) * cap * hd;
  const float* V = vc + ((int64_t)b * Hkv + g) * cap * hd;
  const uint64_t* mrow = mask + (int64_t)r * 4;
  for (int i = threadIdx.x; i < hd; i += 256) sq[i] = qkv[(int64_t)r * q_stride + (int64_t)h * hd + i];
  __syncthreads();
  float scale = 1.0f / sqrtf((float)hd);
  int parts = 256 / hd;
  int dim = threadIdx.x % hd, part = threadIdx.x / hd;
  float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
  for (int c0 = 0; c0 < T; c0 += F32_ATT_CHUNK) {
    int cn = min(F32_ATT_CHUNK, T - c0);
    float lmax = -INFINITY;
    for (int j = threadIdx.x; j < cn; j += 256) {
      int key = c0 + j;
      bool vis = key < P;
      if (!vis) {
        int t = key - P;
        vis = (mrow[t >> 6] >> (t & 63)) & 1ull;
      }
      float sc = -INFINITY;
      if (vis) {
        const float* kr = K + (int64_t)key * hd;
        float d = 0.f;
        for (int i = 0; i < hd; ++i) d += sq[i] * kr[i];
        sc = d * scale;
      }
      sp[j] = sc;
      lmax = fmaxf(lmax, sc);
    }
    float cmax = block_max_256(lmax, sred);
    float m_new = fmaxf(m_run, cmax);
    float alpha = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
    float lsum = 0.f;
    if (m_new != -INFINITY) {
      for (int j = threadIdx.x; j < cn; j += 256) {
        float sc = sp[j];
        float p = (sc == -INFINITY) ? 0.f : expf(sc - m_new);
        sp[j] = p;
        lsum += p;
      }
    } else {
      for (int j = threadIdx.x; j < cn; j += 256) sp[j] = 0.f;
    }
    float csum = block_sum_256(lsum, sred);  // also orders the sp[] writes before the reads below
    l_run = l_run * alpha + csum;
    acc *= alpha;
    for (int j = part; j < cn; j += parts) acc += sp[j] * V[(int64_t)(c0 + j) * hd + dim];
    m_run = m_new;
    __syncthreads();
  }
  sacc[threadIdx.x] = acc;
  __syncthreads();
  if (threadIdx.x < hd) {
    float t = 0.f;
    for (int p = 0; p < parts; ++p) t += sacc[p * hd + threadIdx.x];
    out[threadIdx.x] = t / l_run;
  }
}
void f32_tree_attention(float* o, const float* qkv, int q_stride, const float* kc, const float* vc,
                        const StepMeta& m, const ModelDims& md, hipStream_t s) {
  hipLaunchKernelGGL(f32_tree_attention_kernel, dim3(m.rows, md.H), dim3(256), 0, s, o, qkv, q_stride, kc, vc,
                     m.mask, m.seq_p, m.seq_n, m.n_step, md.H, md.Hkv, md.hd, md.cap);
}

// ------------------------------------------------------------------------------------------
__global__ void f32_silu_mul_kernel(float* __restrict__ h, const float* __restrict__ gu, int F) {
  int r = blockIdx.y;
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= F) return;
  float g = gu[(int64_t)r * 2 * F + i], u = gu[(int64_t)r * 2 * F + F + i];
  h[(int64_t)r * F + i] = g / (1.0f + expf(-g)) * u;
}
void f32_silu_mul(float* h, const float* gu, int rows, int F, hipStream_t s) {
  hipLaunchKernelGGL(f32_silu_mul_kernel, dim3((F + 255) / 256, rows), dim3(256), 0, s, h, gu, F);
}

// ------------------------------------------------------------------------------------------
// Compaction: slot P + path[j] -> slot P + j for j = 0..len-1.  path is increasing with path[j] >= j,
// so each thread walks j upwards and only ever overwrites slots it has already consumed.
__global__ void f32_kv_compact_kernel(float* const* __restrict__ kc, float* const* __restrict__ vc,
                                      const int32_t* __restrict__ path, const int32_t* __restrict__ n_acc,
                                      const int32_t* __restrict__ seq_p, int Hkv, int hd, int cap, int stride) {
  int layer = blockIdx.x, bh = blockIdx.y;
  int b = bh / Hkv;
  int len = n_acc[b];
  int P = seq_p[b];
  const int32_t* pth = path + (int64_t)b * stride;
  float* K = kc[layer] + (int64_t)bh * cap * hd;
  float* V = vc[layer] + (int64_t)bh * cap * hd;
  for (int i = threadIdx.x; i < hd; i += blockDim.x) {
    for (int j = 0; j < len; ++j) {
      int src = pth[j];
      if (src != j) {
        K[(int64_t)(P + j) * hd + i] = K[(int64_t)(P + src) * hd + i];
        V[(int64_t)(P + j) * hd + i] = V[(int64_t)(P + src) * hd + i];
      }
    }
  }
}
void f32_kv_compact(float* const* kc, float* const* vc, const int32_t* path, const int32_t* n_acc,
                    const StepMeta& m, const ModelDims& md, int stride, hipStream_t s) {
  hipLaunchKernelGGL(f32_kv_compact_kernel, dim3(md.n_layers, m.batch * md.Hkv), dim3(64), 0, s, kc, vc, path,
                     n_acc, m.seq_p, md.Hkv, md.hd, md.cap, stride);
}

// ------------------------------------------------------------------------------------------
__global__ void f32_kv_copy_kernel(float* __restrict__ cache, float* __restrict__ plain, int to_cache,
                                   int seq, int first, int n, int Hkv, int hd, int cap) {
  int j = blockIdx.x, g = blockIdx.y;
  float* c = cache + (((int64_t)seq * Hkv + g) * cap + first + j) * hd;
  float* p = plain + ((int64_t)g * n + j) * hd;
  for (int i = threadIdx.x; i < hd; i += blockDim.x) {
    if (to_cache) c[i] = p[i];
    else p[i] = c[i];
  }
}
void f32_kv_copy(float* cache, float* plain, bool to_cache, int seq, int first, int n,
                 const ModelDims& md, hipStream_t s) {
  if (n <= 0) return;
  hipLaunchKernelGGL(f32_kv_copy_kernel, dim3(n, md.Hkv), dim3(64), 0, s, cache, plain, to_cache ? 1 : 0, seq,
                     first, n, md.Hkv, md.hd, md.cap);
}

// zero the slots [first, first + n) of one sequence (keys and values)
__global__ void f32_kv_clear_kernel(float* __restrict__ kc, float* __restrict__ vc, int seq, int first, int Hkv,
                                    int hd, int cap) {
  int j = blockIdx.x, g = blockIdx.y;
  int64_t at = (((int64_t)seq * Hkv + g) * cap + first + j) * hd;
  for (int i = threadIdx.x; i < hd; i += blockDim.x) {
    kc[at + i] = 0.f;
    vc[at + i] = 0.f;
  }
}
void f32_kv_clear(float* kc, float* vc, int seq, int first, int n, const ModelDims& md, hipStream_t s) {
  if (n <= 0) return;
  hipLaunchKernelGGL(f32_kv_clear_kernel, dim3(n, md.Hkv), dim3(64), 0, s, kc, vc, seq, first, md.Hkv, md.hd, md.cap);
}

// k_tree / v_tree: [B][Hkv][max_nodes][hd] -> cache slot P + node
__global__ void f32_scatter_tree_kv_kernel(float* __restrict__ kc, float* __restrict__ vc,
                                           const float* __restrict__ kt, const float* __restrict__ vt,
                                           const int32_t* __restrict__ seq_p, const int32_t* __restrict__ seq_n,
                                           int Hkv, int hd, int cap, int max_nodes) {
  int node = blockIdx.x, bh = blockIdx.y;
  int b = bh / Hkv;
  if (node >= seq_n[b]) return;
  int64_t src = ((int64_t)bh * max_nodes + node) * hd;
  int64_t dst = ((int64_t)bh * cap + seq_p[b] + node) * hd;
  for (int i = threadIdx.x; i < hd; i += blockDim.x) {
    kc[dst + i] = kt[src + i];
    vc[dst + i] = vt[src + i];
  }
}
void f32_scatter_tree_kv(float* kc, float* vc, const float* k_tree, const float* v_tree,
                         const StepMeta& m, const ModelDims& md, int max_nodes, hipStream_t s) {
  hipLaunchKernelGGL(f32_scatter_tree_kv_kernel, dim3(max_nodes, m.batch * md.Hkv), dim3(64), 0, s, kc, vc,
                     k_tree, v_tree, m.seq_p, m.seq_n, md.Hkv, md.hd, md.cap, max_nodes);
}

// rows of real nodes between the caller's [B][max_nodes][width] and the padded [R][width] buffers
__global__ void f32_gather_rows_kernel(float* __restrict__ dst, const float* __restrict__ src,
                                       const int32_t* __restrict__ seq_n, int n_step, int max_nodes, int width,
                                       int to_padded) {
  int r = blockIdx.x;
  int b = r / n_step, node = r - b * n_step;
  bool real = node < seq_n[b];
  int64_t pad = (int64_t)r * width, ext = ((int64_t)b * max_nodes + node) * width;
  for (int i = threadIdx.x; i < width; i += blockDim.x) {
    if (to_padded) dst[pad + i] = real ? src[ext + i] : 0.f;
    else if (real) dst[ext + i] = src[pad + i];
  }
}
void f32_gather_rows(float* dst, const float* src, const StepMeta& m, int max_nodes, int width,
                     bool to_padded, hipStream_t s) {
  hipLaunchKernelGGL(f32_gather_rows_kernel, dim3(m.rows), dim3(256), 0, s, dst, src, m.seq_n, m.n_step,
                     max_nodes, width, to_padded ? 1 : 0);
}

}  // namespace ded
