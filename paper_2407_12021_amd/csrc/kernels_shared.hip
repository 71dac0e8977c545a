// Kernels used by both storage types: rotary table, per-node argmax, logits export, approval walk.
#include "ded_kernels.h"

namespace ded {

// ------------------------------------------------------------------------------------------
// Rotary table.  The angle pos * base^(-2i/hd) is formed in fp64 so that long contexts do not lose
// phase accuracy; the rotation itself is applied in fp32 by the consumers.
// ------------------------------------------------------------------------------------------
__global__ void rope_table_kernel(float2* __restrict__ tab, const int32_t* __restrict__ pos, int rows,
                                  int half, double neg2_over_hd_log2base) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= rows * half) return;
  int r = idx / half, i = idx - r * half;
  double theta = exp2((double)i * neg2_over_hd_log2base);
  double ang = (double)pos[r] * theta;
  tab[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

void launch_rope_table(float2* tab, const int32_t* pos, int rows, int hd, float base, hipStream_t s) {
  int half = hd / 2;
  int n = rows * half;
  if (n <= 0) return;
  double c = -2.0 / (double)hd * log2((double)base);
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, tab, pos, rows, half, c);
}

// ------------------------------------------------------------------------------------------
// Argmax with top-2 margin.  One workgroup per row; candidates are merged with a fixed rule
// (larger value wins, equal values -> lower index), so the result does not depend on the
// reduction order.
// ------------------------------------------------------------------------------------------
struct Top2 {
  float v1;
  int i1;
  float v2;
};

__device__ inline void top2_push(Top2& t, float v, int i) {
  if (v > t.v1 || (v == t.v1 && i < t.i1)) {
    t.v2 = t.v1;
    t.v1 = v;
    t.i1 = i;
  } else if (v > t.v2) {
    t.v2 = v;
  }
}

__device__ inline void top2_merge(Top2& a, const Top2& b) {
  if (b.v1 > a.v1 || (b.v1 == a.v1 && b.i1 < a.i1)) {
    a.v2 = fmaxf(a.v1, b.v2);
    a.v1 = b.v1;
    a.i1 = b.i1;
  } else {
    a.v2 = fmaxf(a.v2, b.v1);
  }
}

__global__ __launch_bounds__(256) void argmax_kernel(const float* __restrict__ logits, int64_t row_stride,
                                                     int V, int32_t* __restrict__ amax,
                                                     float* __restrict__ margin) {
  const float* row = logits + (int64_t)blockIdx.x * row_stride;
  Top2 t = {-INFINITY, 0x7fffffff, -INFINITY};
  int nv4 = ((reinterpret_cast<uintptr_t>(row) & 15) == 0) ? (V / 4) : 0;
  const float4* row4 = reinterpret_cast<const float4*>(row);
  for (int i = threadIdx.x; i < nv4; i += 256) {
    float4 v = row4[i];
    top2_push(t, v.x, 4 * i);
    top2_push(t, v.y, 4 * i + 1);
    top2_push(t, v.z, 4 * i + 2);
    top2_push(t, v.w, 4 * i + 3);
  }
  for (int i = nv4 * 4 + threadIdx.x; i < V; i += 256) top2_push(t, row[i], i);
  for (int off = 32; off >= 1; off >>= 1) {
    Top2 o;
    o.v1 = __shfl_xor(t.v1, off);
    o.i1 = __shfl_xor(t.i1, off);
    o.v2 = __shfl_xor(t.v2, off);
    top2_merge(t, o);
  }
  __shared__ Top2 sh[4];
  int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) sh[wave] = t;
  __syncthreads();
  if (threadIdx.x == 0) {
    Top2 r = sh[0];
    for (int w = 1; w < 4; ++w) top2_merge(r, sh[w]);
    amax[blockIdx.x] = r.i1;
    margin[blockIdx.x] = r.v1 - r.v2;
  }
}

void launch_argmax(const float* logits, int64_t row_stride, int rows, int V, int32_t* amax,
                   float* margin, hipStream_t s) {
  if (rows <= 0) return;
  hipLaunchKernelGGL(argmax_kernel, dim3(rows), dim3(256), 0, s, logits, row_stride, V, amax, margin);
}

// ------------------------------------------------------------------------------------------
__global__ void export_logits_kernel(float* __restrict__ dst, const float* __restrict__ src,
                                     int64_t src_stride, const int32_t* __restrict__ seq_n, int n_step,
                                     int max_nodes, int V) {
  int r = blockIdx.x;
  int b = r / n_step, node = r - b * n_step;
  if (node >= seq_n[b]) return;
  const float* s = src + (int64_t)r * src_stride;
  float* d = dst + ((int64_t)b * max_nodes + node) * V;
  for (int i = threadIdx.x; i < V; i += blockDim.x) d[i] = s[i];
}

void launch_export_logits(float* dst, const float* src, int64_t src_stride, const StepMeta& m,
                          int max_nodes, int V, hipStream_t s) {
  hipLaunchKernelGGL(export_logits_kernel, dim3(m.rows), dim3(256), 0, s, dst, src, src_stride, m.seq_n,
                     m.n_step, max_nodes, V);
}

// ------------------------------------------------------------------------------------------
// Approval walk, one wavefront per sequence.  Node i is approved iff every node v on the path
// root..i (v != root) carries the model's token of its parent.  The end node is the deepest
// approved node, lowest index among equals.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void accept_walk_kernel(const int32_t* __restrict__ token,
                                                         const int32_t* __restrict__ parent,
                                                         const int32_t* __restrict__ depth,
                                                         const int32_t* __restrict__ seq_n,
                                                         const int32_t* __restrict__ amax, int n_step,
                                                         int mode, int32_t* __restrict__ out_n,
                                                         int32_t* __restrict__ out_path,
                                                         int32_t* __restrict__ out_tok, int stride) {
  int b = blockIdx.x;
  int n = seq_n[b];
  const int32_t* tok = token + (int64_t)b * n_step;
  const int32_t* par = parent + (int64_t)b * n_step;
  const int32_t* dep = depth + (int64_t)b * n_step;
  const int32_t* am = amax + (int64_t)b * n_step;
  int best = -1;  // key = depth * 1024 + (1023 - node)
  if (mode == 1) {
    best = (n - 1) * 1024 + (1023 - (n - 1));
  } else {
    for (int i = threadIdx.x; i < n; i += 64) {
      bool ok = true;
      int v = i;
      for (int guard = 0; guard < n && ok; ++guard) {
        int p = par[v];
        if (p < 0) break;
        ok = (tok[v] == am[p]);
        v = p;
      }
      if (ok) {
        int key = dep[i] * 1024 + (1023 - i);
        best = key > best ? key : best;
      }
    }
    for (int off = 32; off >= 1; off >>= 1) {
      int o = __shfl_xor(best, off);
      best = o > best ? o : best;
    }
  }
  if (threadIdx.x == 0) {
    int end = 1023 - (best & 1023);
    int len = dep[end] + 1;
    int32_t* path = out_path + (int64_t)b * stride;
    int32_t* acc = out_tok + (int64_t)b * stride;
    int v = end;
    for (int j = len - 1; j >= 0; --j) {
      path[j] = v;
      if (j > 0) acc[j - 1] = tok[v];
      v = par[v];
    }
    acc[len - 1] = am[end];
    out_n[b] = len;
  }
}

void launch_accept_walk(const StepMeta& m, const int32_t* amax, int mode, int32_t* out_n,
                        int32_t* out_path, int32_t* out_tok, int stride, hipStream_t s) {
  hipLaunchKernelGGL(accept_walk_kernel, dim3(m.batch), dim3(64), 0, s, m.token, m.parent, m.depth,
                     m.seq_n, amax, m.n_step, mode, out_n, out_path, out_tok, stride);
}

}  // namespace ded
