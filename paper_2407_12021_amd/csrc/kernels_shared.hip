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
// Measurement aid: a plain streaming read of a device buffer: every wavefront walks a contiguous region of its own
// with 16-byte non-temporal loads, four in flight per lane (the access pattern of the weight-streaming GEMMs; the
// non-temporal hint is worth ~12 % on this chip: 6.8 against 6.0 TB/s).  Its rate is the ceiling that a weight- or
// cache-streaming kernel can be held against on the same chip in the same run.  The XOR of everything read goes
// to sink[0] so that the loads cannot be dropped.
typedef unsigned probe_u32x4_t __attribute__((ext_vector_type(4)));
__device__ inline uint4 probe_load(const uint4* q) {
  const probe_u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const probe_u32x4_t*>(q));
  return make_uint4(r.x, r.y, r.z, r.w);
}
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, int64_t n_u4,
                                                          uint32_t* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), n_waves = (int64_t)gridDim.x * 4;
  const int64_t per = n_u4 / n_waves / 256 * 256;  // 16-byte units per wavefront, whole turns of 4 x 64 only
  uint4 a = make_uint4(0, 0, 0, 0);
  const uint4* q = src + wave * per + lane;
  for (int64_t i = 0; i < per; i += 256) {
    const uint4 v0 = probe_load(q + i), v1 = probe_load(q + i + 64), v2 = probe_load(q + i + 128), v3 = probe_load(q + i + 192);
    a.x ^= v0.x ^ v1.x ^ v2.x ^ v3.x;
    a.y ^= v0.y ^ v1.y ^ v2.y ^ v3.y;
    a.z ^= v0.z ^ v1.z ^ v2.z ^ v3.z;
    a.w ^= v0.w ^ v1.w ^ v2.w ^ v3.w;
  }
  for (int64_t i = n_waves * per + wave * 64 + lane; i < n_u4; i += n_waves * 64) {  // what the regions leave over
    const uint4 v = src[i];
    a.x ^= v.x;
    a.y ^= v.y;
    a.z ^= v.z;
    a.w ^= v.w;
  }
  uint32_t x = a.x ^ a.y ^ a.z ^ a.w;
  for (int off = 32; off >= 1; off >>= 1) x ^= __shfl_xor(x, off);
  if (lane == 0 && x == 0x9e3779b9u) sink[0] = x;  // practically never true: the store is the data dependence
}

void launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s) {
  const int64_t n = (int64_t)(bytes / 16);
  if (n <= 0) return;
  hipLaunchKernelGGL(stream_read_kernel, dim3(1024), dim3(256), 0, s, reinterpret_cast<const uint4*>(src), n, sink);
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

// NaN and +-inf: a row that holds one has no meaningful argmax; it is reported through the row's flag
__device__ inline int nonfinite(float v) { return !(fabsf(v) <= 3.402823466e38f); }

// combine the 256 threads' candidates of one row and write the row's verdict
__device__ inline void top2_block_finish(Top2 t, int bad, int32_t* amax, float* margin, int32_t* flag) {
  for (int off = 32; off >= 1; off >>= 1) {
    Top2 o;
    o.v1 = __shfl_xor(t.v1, off);
    o.i1 = __shfl_xor(t.i1, off);
    o.v2 = __shfl_xor(t.v2, off);
    top2_merge(t, o);
    bad |= __shfl_xor(bad, off);
  }
  __shared__ Top2 sh[4];
  __shared__ int sh_bad[4];
  int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    sh[wave] = t;
    sh_bad[wave] = bad;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    Top2 r = sh[0];
    for (int w = 1; w < 4; ++w) top2_merge(r, sh[w]);
    amax[blockIdx.x] = r.i1;
    margin[blockIdx.x] = r.v1 - r.v2;
    flag[blockIdx.x] = sh_bad[0] | sh_bad[1] | sh_bad[2] | sh_bad[3];
  }
}

__global__ __launch_bounds__(256) void argmax_kernel(const float* __restrict__ logits, int64_t row_stride,
                                                     int V, int32_t* __restrict__ amax,
                                                     float* __restrict__ margin, int32_t* __restrict__ flag) {
  const float* row = logits + (int64_t)blockIdx.x * row_stride;
  Top2 t = {-INFINITY, 0x7fffffff, -INFINITY};
  int bad = 0;
  int nv4 = ((reinterpret_cast<uintptr_t>(row) & 15) == 0) ? (V / 4) : 0;
  const float4* row4 = reinterpret_cast<const float4*>(row);
  for (int i = threadIdx.x; i < nv4; i += 256) {
    float4 v = row4[i];
    bad |= nonfinite(v.x) | nonfinite(v.y) | nonfinite(v.z) | nonfinite(v.w);
    top2_push(t, v.x, 4 * i);
    top2_push(t, v.y, 4 * i + 1);
    top2_push(t, v.z, 4 * i + 2);
    top2_push(t, v.w, 4 * i + 3);
  }
  for (int i = nv4 * 4 + threadIdx.x; i < V; i += 256) {
    bad |= nonfinite(row[i]);
    top2_push(t, row[i], i);
  }
  top2_block_finish(t, bad, amax, margin, flag);
}

void launch_argmax(const float* logits, int64_t row_stride, int rows, int V, int32_t* amax,
                   float* margin, int32_t* flag, hipStream_t s) {
  if (rows <= 0) return;
  hipLaunchKernelGGL(argmax_kernel, dim3(rows), dim3(256), 0, s, logits, row_stride, V, amax, margin, flag);
}

// The same verdict from per-(row, 64-feature group) candidates that the LM-head GEMM's epilogue left instead of
// logits: part[r][g] = (top-1 value, its id, top-2 value, non-finite flag) as four 32-bit words.  The merge rule
// does not depend on the order, so the result equals argmax_kernel's on the materialised row bit for bit.
__global__ __launch_bounds__(256) void top2_reduce_kernel(const uint4* __restrict__ part, int groups,
                                                          int32_t* __restrict__ amax, float* __restrict__ margin,
                                                          int32_t* __restrict__ flag) {
  const uint4* row = part + (int64_t)blockIdx.x * groups;
  Top2 t = {-INFINITY, 0x7fffffff, -INFINITY};
  int bad = 0;
  for (int g = threadIdx.x; g < groups; g += 256) {
    const uint4 p = row[g];
    Top2 o = {__uint_as_float(p.x), (int)p.y, __uint_as_float(p.z)};
    top2_merge(t, o);
    bad |= (int)p.w;
  }
  top2_block_finish(t, bad, amax, margin, flag);
}

void launch_top2_reduce(const void* part, int groups, int rows, int32_t* amax, float* margin, int32_t* flag,
                        hipStream_t s) {
  if (rows <= 0) return;
  hipLaunchKernelGGL(top2_reduce_kernel, dim3(rows), dim3(256), 0, s, reinterpret_cast<const uint4*>(part), groups,
                     amax, margin, flag);
}

// ------------------------------------------------------------------------------------------
// Temperature / top-p sampling of the model's token at every node (stochastic approval, Sec. 2.4: a token
// is sampled from the model's distribution and compared with the draft; Sec. 4.4 varies temperature and
// top-p).  One workgroup per row.  p_i = softmax(logits / T); the nucleus is the smallest set of most
// probable tokens reaching top_p, ties with its last member included; the token is the inverse CDF of the
// caller's uniform number over the nucleus in token-id order.
// p is monotone in the logit, so the nucleus is {logit >= t*} with t* the largest threshold under which the
// set still reaches top_p: found by bisection over the order-preserving integer image of fp32 (<= 32
// passes over the row, which stays in L2).  Sums are formed in a fixed order (per thread, wavefront
// shuffles, wavefront order), so the result is reproducible.
constexpr int SAMPLE_THREADS = 1024;

__device__ inline uint32_t ordered_key(float v) {
  const uint32_t b = __float_as_uint(v);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ inline float block_sum(float v, float* sh) {
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = 0.f;
  for (int w = 0; w < SAMPLE_THREADS / 64; ++w) r += sh[w];
  return r;
}

// exclusive prefix of v over the threads of the block and the block total, in a fixed order (wavefront scan by
// shuffles, then the wavefront totals one after the other)
__device__ inline float block_exclusive_scan(float v, float* sh_w, float& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float inc = v;
  for (int off = 1; off < 64; off <<= 1) {
    const float o = __shfl_up(inc, off);
    if (lane >= off) inc += o;
  }
  __syncthreads();
  if (lane == 63) sh_w[wave] = inc;
  __syncthreads();
  float before = 0.f, all = 0.f;
  for (int w = 0; w < SAMPLE_THREADS / 64; ++w) {
    if (w < wave) before += sh_w[w];
    all += sh_w[w];
  }
  total = all;
  return before + (inc - v);
}

__global__ __launch_bounds__(SAMPLE_THREADS) void sample_top_p_kernel(const float* __restrict__ logits,
                                                                      int64_t row_stride, int V, float inv_temp,
                                                                      float top_p, const float* __restrict__ uniform,
                                                                      int32_t* __restrict__ token_out) {
  __shared__ float sh[SAMPLE_THREADS / 64];
  __shared__ uint32_t sh_k[2 * (SAMPLE_THREADS / 64)];
  __shared__ int sh_owner;
  const float* row = logits + (int64_t)blockIdx.x * row_stride;
  const int tid = threadIdx.x;
  // pass 1: extreme keys
  uint32_t kmax = 0u, kmin = 0xffffffffu;
  for (int i = tid; i < V; i += SAMPLE_THREADS) {
    const uint32_t k = ordered_key(row[i]);
    kmax = k > kmax ? k : kmax;
    kmin = k < kmin ? k : kmin;
  }
  for (int off = 32; off >= 1; off >>= 1) {
    const uint32_t a = __shfl_xor(kmax, off), b = __shfl_xor(kmin, off);
    kmax = a > kmax ? a : kmax;
    kmin = b < kmin ? b : kmin;
  }
  if ((tid & 63) == 0) {
    sh_k[tid >> 6] = kmax;
    sh_k[SAMPLE_THREADS / 64 + (tid >> 6)] = kmin;
  }
  __syncthreads();
  for (int w = 0; w < SAMPLE_THREADS / 64; ++w) {
    kmax = sh_k[w] > kmax ? sh_k[w] : kmax;
    kmin = sh_k[SAMPLE_THREADS / 64 + w] < kmin ? sh_k[SAMPLE_THREADS / 64 + w] : kmin;
  }
  const uint32_t bmax = (kmax & 0x80000000u) ? (kmax & 0x7fffffffu) : ~kmax;
  const float m = __uint_as_float(bmax);  // row maximum
  // weight of the tokens whose key is >= t  (t = 0: all)
  auto mass = [&](uint32_t t) {
    float s = 0.f;
    for (int i = tid; i < V; i += SAMPLE_THREADS) {
      const float l = row[i];
      if (ordered_key(l) >= t) s += __expf((l - m) * inv_temp);
    }
    return block_sum(s, sh);
  };
  const float Z = mass(0u);
  const float need = top_p * Z;
  // largest t with mass(t) >= need:  mass(lo) >= need holds (lo = smallest key), mass(hi) < need (hi beyond the largest)
  uint32_t lo = kmin, hi = kmax + 1u;  // logits are finite, so kmax + 1 does not wrap
  while (hi - lo > 1u) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    if (mass(mid) >= need) lo = mid;
    else hi = mid;
  }
  // inverse CDF over the nucleus in id order: thread t owns the ids [t * chunk, (t + 1) * chunk)
  const int chunk = (V + SAMPLE_THREADS - 1) / SAMPLE_THREADS;
  const int i0 = tid * chunk, i1 = min(V, i0 + chunk);
  float own = 0.f;
  int last_kept = -1;
  for (int i = i0; i < i1; ++i) {
    const float l = row[i];
    if (ordered_key(l) >= lo) {
      own += __expf((l - m) * inv_temp);
      last_kept = i;
    }
  }
  if (tid == 0) sh_owner = -1;
  float total;
  const float before = block_exclusive_scan(own, sh, total);  // its barriers also publish sh_owner
  const float target = uniform[blockIdx.x] * total;
  // The chunk that holds the target is the last one that starts at or below it (`before` never decreases with
  // the thread index).  Its thread takes the first id whose running sum passes the target - or, when its own
  // running sum (rounded in another order than the scan) stops short of it, the chunk's last nucleus id.
  if (own > 0.f && before <= target) atomicMax(&sh_owner, tid);
  __syncthreads();
  if (tid == sh_owner) {
    float run = before;
    int pick = last_kept;
    for (int i = i0; i < i1; ++i) {
      const float l = row[i];
      if (ordered_key(l) >= lo) {
        run += __expf((l - m) * inv_temp);
        if (run > target) {
          pick = i;
          break;
        }
      }
    }
    token_out[blockIdx.x] = pick;
  }
}

// Same sampler for vocabularies that fit LDS: the weights exp((l - max) / T) are computed once and kept in LDS
// (they are monotone in the logit, so the bisection runs on their bit patterns), which turns the ~34 passes
// over the row into LDS traffic.
constexpr int SAMPLE_LDS_V = 36864;  // 144 KiB of weights

__global__ __launch_bounds__(SAMPLE_THREADS) void sample_top_p_lds_kernel(const float* __restrict__ logits,
                                                                          int64_t row_stride, int V, float inv_temp,
                                                                          float top_p, const float* __restrict__ uniform,
                                                                          int32_t* __restrict__ token_out) {
  __shared__ float e[SAMPLE_LDS_V];
  __shared__ float sh[SAMPLE_THREADS / 64];
  __shared__ int sh_owner;
  const float* row = logits + (int64_t)blockIdx.x * row_stride;
  const int tid = threadIdx.x;
  float m = -INFINITY;
  for (int i = tid; i < V; i += SAMPLE_THREADS) m = fmaxf(m, row[i]);
  for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  if ((tid & 63) == 0) sh[tid >> 6] = m;
  __syncthreads();
  for (int w = 0; w < SAMPLE_THREADS / 64; ++w) m = fmaxf(m, sh[w]);
  float z = 0.f;
  uint32_t kmin = 0xffffffffu;
  for (int i = tid; i < V; i += SAMPLE_THREADS) {
    const float w = __expf((row[i] - m) * inv_temp);  // in [0, 1]: its bit pattern orders like its value
    e[i] = w;
    z += w;
    kmin = min(kmin, __float_as_uint(w));
  }
  const float Z = block_sum(z, sh);
  for (int off = 32; off >= 1; off >>= 1) kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off));
  __shared__ uint32_t sh_k[SAMPLE_THREADS / 64];
  if ((tid & 63) == 0) sh_k[tid >> 6] = kmin;
  __syncthreads();
  for (int w = 0; w < SAMPLE_THREADS / 64; ++w) kmin = min(kmin, sh_k[w]);
  // largest t with mass(t) >= need, mass(t) = weight of {bits(w) >= t}: 8-way search, seven thresholds per pass
  // over the LDS copy (one block reduction per pass instead of three)
  __shared__ float sh7[7][SAMPLE_THREADS / 64];
  const float need = top_p * Z;
  uint32_t lo = kmin, hi = 0x3f800000u + 1u;  // mass(lo) >= need; the largest weight is exp(0) = 1, so mass(hi) = 0
  while (hi - lo > 1u) {
    const uint32_t span = hi - lo;
    uint32_t t[7];
#pragma unroll
    for (int j = 0; j < 7; ++j) t[j] = lo + (uint32_t)(((uint64_t)span * (j + 1)) >> 3);  // lo <= t[j] < hi, non-decreasing
    float sj[7] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int i = tid; i < V; i += SAMPLE_THREADS) {
      const float w = e[i];
      const uint32_t k = __float_as_uint(w);
#pragma unroll
      for (int j = 0; j < 7; ++j) sj[j] += k >= t[j] ? w : 0.f;
    }
#pragma unroll
    for (int j = 0; j < 7; ++j)
      for (int off = 32; off >= 1; off >>= 1) sj[j] += __shfl_xor(sj[j], off);
    __syncthreads();
    if ((tid & 63) == 0) {
#pragma unroll
      for (int j = 0; j < 7; ++j) sh7[j][tid >> 6] = sj[j];
    }
    __syncthreads();
    uint32_t nlo = lo, nhi = hi;
#pragma unroll
    for (int j = 0; j < 7; ++j) {
      float f = 0.f;
      for (int w = 0; w < SAMPLE_THREADS / 64; ++w) f += sh7[j][w];
      if (f >= need) nlo = t[j] > nlo ? t[j] : nlo;         // thresholds that still reach the target move lo up
      else nhi = t[j] < nhi ? t[j] : nhi;                    // the first that does not becomes hi
    }
    if (nlo == lo && nhi == hi) break;  // cannot happen while span > 1 (t[6] > lo or t[0] == lo handled), safety only
    lo = nlo;
    hi = nhi;
  }
  const int chunk = (V + SAMPLE_THREADS - 1) / SAMPLE_THREADS;
  const int i0 = tid * chunk, i1 = min(V, i0 + chunk);
  float own = 0.f;
  int last_kept = -1;
  for (int i = i0; i < i1; ++i) {
    const float w = e[i];
    if (__float_as_uint(w) >= lo) {
      own += w;
      last_kept = i;
    }
  }
  if (tid == 0) sh_owner = -1;
  float total;
  const float before = block_exclusive_scan(own, sh, total);  // its barriers also publish sh_owner
  const float target = uniform[blockIdx.x] * total;
  // as in sample_top_p_kernel: the last chunk that starts at or below the target holds it
  if (own > 0.f && before <= target) atomicMax(&sh_owner, tid);
  __syncthreads();
  if (tid == sh_owner) {
    float run = before;
    int pick = last_kept;
    for (int i = i0; i < i1; ++i) {
      const float w = e[i];
      if (__float_as_uint(w) >= lo) {
        run += w;
        if (run > target) {
          pick = i;
          break;
        }
      }
    }
    token_out[blockIdx.x] = pick;
  }
}

void launch_sample_top_p(const float* logits, int64_t row_stride, int rows, int V, float temperature, float top_p,
                         const float* uniform, int32_t* token_out, hipStream_t s) {
  if (rows <= 0) return;
  if (V <= SAMPLE_LDS_V)
    hipLaunchKernelGGL(sample_top_p_lds_kernel, dim3(rows), dim3(SAMPLE_THREADS), 0, s, logits, row_stride, V,
                       1.0f / temperature, top_p, uniform, token_out);
  else
    hipLaunchKernelGGL(sample_top_p_kernel, dim3(rows), dim3(SAMPLE_THREADS), 0, s, logits, row_stride, V,
                       1.0f / temperature, top_p, uniform, token_out);
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
                                                         const int32_t* __restrict__ amax,
                                                         const int32_t* __restrict__ row_flag, int n_step,
                                                         int mode, int32_t* __restrict__ out_n,
                                                         int32_t* __restrict__ out_flag,
                                                         int32_t* __restrict__ out_path,
                                                         int32_t* __restrict__ out_tok, int stride) {
  int b = blockIdx.x;
  int n = seq_n[b];
  const int32_t* tok = token + (int64_t)b * n_step;
  const int32_t* par = parent + (int64_t)b * n_step;
  const int32_t* dep = depth + (int64_t)b * n_step;
  const int32_t* am = amax + (int64_t)b * n_step;
  // a step with a non-finite logit at a real node of any sequence has no verdict: every sequence gets path
  // length 0 (nothing is compacted) and its flag raised
  int bad = 0;
  for (int b2 = 0; b2 < gridDim.x; ++b2)
    for (int i = threadIdx.x; i < seq_n[b2]; i += 64) bad |= row_flag[(int64_t)b2 * n_step + i];
  bad = __any(bad != 0);
  if (bad) {
    if (threadIdx.x == 0) {
      out_n[b] = 0;
      out_flag[b] = 1;
    }
    return;
  }
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
    out_flag[b] = 0;
  }
}

void launch_accept_walk(const StepMeta& m, const int32_t* amax, const int32_t* row_flag, int mode, int32_t* out_n,
                        int32_t* out_flag, int32_t* out_path, int32_t* out_tok, int stride, hipStream_t s) {
  hipLaunchKernelGGL(accept_walk_kernel, dim3(m.batch), dim3(64), 0, s, m.token, m.parent, m.depth,
                     m.seq_n, amax, row_flag, m.n_step, mode, out_n, out_flag, out_path, out_tok, stride);
}

}  // namespace ded
