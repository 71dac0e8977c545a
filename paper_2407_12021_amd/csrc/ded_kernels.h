// Internal launcher interface between the host scheduler (ded_api.hip) and the kernel files.
// Every launcher enqueues on the given stream and checks its shapes on the host first; the
// kernels themselves assume those shapes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ded {

// Device-resident description of the current step (one verification forward).
// Row r = b * n_step + node; n_step = the step's padded tree size (multiple of 16).
struct StepMeta {
  const int32_t* token;   // [R]   token id of the row (padding rows repeat the root token)
  const int32_t* parent;  // [R]   parent node index inside the sequence, -1 for root / padding
  const int32_t* depth;   // [R]
  const int32_t* pos;     // [R]   absolute position prefix_len + depth
  const uint64_t* mask;   // [R][4] ancestor-or-self bitmask over node indices (bit j = node j)
  const int32_t* seq_p;   // [B]   prefix_len per sequence
  const int32_t* seq_n;   // [B]   real tree rows per sequence
  int32_t batch, n_step, rows;  // rows = batch * n_step
};

struct ModelDims {
  int32_t n_layers, d, H, Hkv, hd, F, V, cap;
  float rope_base, eps;
};

// ---- shared (both dtypes) --------------------------------------------------------------
// cos/sin of pos[r] * base^(-2i/hd), i < hd/2, angles formed in fp64.  tab: [R][hd/2] float2.
void launch_rope_table(float2* tab, const int32_t* pos, int rows, int hd, float base, hipStream_t s);
// Measurement aid: streams `bytes` (multiple of 16) of device memory through the CUs once.
void launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s);
// Per-row argmax (lowest index on exact ties) and top-1 minus top-2 over V fp32 logits; flag[r] != 0 when the
// row holds a NaN or an infinity.
void launch_argmax(const float* logits, int64_t row_stride, int rows, int V, int32_t* amax,
                   float* margin, int32_t* flag, hipStream_t s);
// The same from the candidates the LM-head GEMM leaves with EPI_TOP2: part [rows][groups] x 16 bytes.
void launch_top2_reduce(const void* part, int groups, int rows, int32_t* amax, float* margin, int32_t* flag,
                        hipStream_t s);
// Per-row temperature / top-p sample (inverse CDF of uniform[r] over the nucleus in id order) -> token_out[r].
void launch_sample_top_p(const float* logits, int64_t row_stride, int rows, int V, float temperature, float top_p,
                         const float* uniform, int32_t* token_out, hipStream_t s);
// Copy rows of real nodes to the caller's [batch][max_nodes][V] logits buffer.
void launch_export_logits(float* dst, const float* src, int64_t src_stride, const StepMeta& m,
                          int max_nodes, int V, hipStream_t s);
// Approval walk (one wavefront per sequence).  mode 0 greedy, mode 1 keep the whole chain.
// out_n [B], out_path / out_tok [B][stride].  If a real row of any sequence is flagged, every sequence gets out_n = 0, out_flag = 1.
void launch_accept_walk(const StepMeta& m, const int32_t* amax, const int32_t* row_flag, int mode, int32_t* out_n,
                        int32_t* out_flag, int32_t* out_path, int32_t* out_tok, int stride, hipStream_t s);

// ---- fp32 path (plain row-major everywhere; cache [B][Hkv][cap][hd]) ---------------------
void f32_embed(float* x, const float* emb, const StepMeta& m, int d, hipStream_t s);
void f32_rmsnorm(float* y, const float* x, const float* gain, int rows, int d, float eps, hipStream_t s);
// Y[r][n] (+)= sum_k X[r][k] W[n][k]
void f32_gemm(float* Y, const float* X, const float* W, int rows, int N, int K, bool accumulate, hipStream_t s);
void f32_rope_kv(float* qkv, float* kc, float* vc, const float2* tab, const StepMeta& m,
                 const ModelDims& md, hipStream_t s);
void f32_tree_attention(float* o, const float* qkv, int q_stride, const float* kc, const float* vc,
                        const StepMeta& m, const ModelDims& md, hipStream_t s);
void f32_silu_mul(float* h, const float* gu, int rows, int F, hipStream_t s);
void f32_kv_compact(float* const* kc, float* const* vc, const int32_t* path, const int32_t* n_acc,
                    const StepMeta& m, const ModelDims& md, int stride, hipStream_t s);
// plain [Hkv][n][hd] <-> cache
void f32_kv_copy(float* cache, float* plain, bool to_cache, int seq, int first, int n,
                 const ModelDims& md, hipStream_t s);
void f32_kv_clear(float* kc, float* vc, int seq, int first, int n, const ModelDims& md, hipStream_t s);
void f32_scatter_tree_kv(float* kc, float* vc, const float* k_tree, const float* v_tree,
                         const StepMeta& m, const ModelDims& md, int max_nodes, hipStream_t s);
// q [B][max_nodes][H][hd] -> qkv-style rows [R][H*hd]; and back for the output
void f32_gather_rows(float* dst, const float* src, const StepMeta& m, int max_nodes, int width,
                     bool to_padded, hipStream_t s);

// ---- 16-bit path (bf16 weights in, f16 matrix-core operands; see bf16_layout.h) -----------------
// Operand-fragment layouts (units: 2-byte elements; a fragment = 64 lanes x 8 elements = 1 KiB):
//  PackW  W[N][K]   : frag (ng = n/64, kt = k/32, t = (n/16)%4) at (ng*(K/32)+kt)*4+t; lane = ((k%32)/8)*16 + n%16;
//                      elem k%8; N padded to a multiple of 64 with zero features
//  PackX  X[R][K]   : frag (kt, rb = r/16, plane hi/lo) at (kt*RB+rb)*2+plane; lane = ((k%32)/8)*16 + r%16; elem k%8
//  PackQ  per (b,kvh): frag (vrb, kk = hd/32, plane) at (vrb*4+kk)*2+plane, virtual row vr = g*n_step + node
//  PackK  per (b,kvh): 32-key group kb; frag (kb, c, kk) at (kb*2+c)*4+kk; key%32 = q8*8 + c*4 + i
//                      -> lane = ((hdim%32)/8)*16 + q8*4 + i; elem hdim%8
//  PackVt per (b,kvh): frag (kb, hb = hdim/16) at kb*8+hb; lane = ((key%32)/8)*16 + hdim%16; elem key%8
typedef uint16_t bf16_t;

// How the features (rows) of a weight matrix are ordered inside PackW.  The paired orders put partner
// features into tiles t and t + 2 of one 64-feature group so that one wavefront holds both.
enum { PERM_NONE = 0, PERM_ROPE = 1 /* per head: dims i and i + 64 */, PERM_GATE_UP = 2 /* gate f and up f */ };
void bf16_pack_weight(bf16_t* dst, const bf16_t* src, int N, int K, int perm, hipStream_t s);
// x = emb[token]; y = (x * gain) as hi/lo f16 in PackX; ssq[r][g] = sum of x^2 over feature group g (64 wide)
void bf16_embed(float* x, bf16_t* y_packed, float* ssq, const bf16_t* emb, const float* gain, const StepMeta& m,
                int rows_pad, int d, hipStream_t s);

// What a GEMM does with its result tile (fused epilogue).  RMSNorm is deferred: producers write
// x * gain and sum(x^2) per 64-feature group, consumers multiply their output rows by 1/rms.
enum { EPI_LOGITS = 0, EPI_QKV = 1, EPI_SILU = 2, EPI_RESIDUAL = 3, EPI_TOP2 = 4 };
struct GemmEpilogue {
  int kind;
  // row scale of the GEMM input (null: 1): scale[r] = rsqrt(sum_g ssq_in[r][g] * inv_k + eps)
  const float* ssq_in;
  int ssq_groups;
  float inv_k, eps;
  int rows;      // real rows (the rest up to rows_pad is padding)
  int rb_total;  // rows_pad / 16 of the PackX buffers
  // EPI_LOGITS: out[r][n] = scale * Y
  float* out;
  int64_t out_stride;
  // EPI_TOP2: instead of the logits, per (row, 64-feature group) the best value, its feature index, the second
  // best value and a non-finite flag: top2_part[r * top2_groups + group] (16 bytes each)
  void* top2_part;
  int top2_groups;
  // EPI_QKV: rotary embedding at the row's position, queries -> PackQ (hi/lo), keys / values -> cache
  bf16_t *q_packed, *k_cache, *v_cache;
  const float2* rope_tab;
  const int32_t *seq_p, *seq_n;
  int n_step, H, Hkv, cap;
  // EPI_SILU: y_packed(hi) = silu(scale*gate) * (scale*up);  EPI_RESIDUAL: x += Y, y_packed = x*gain (hi/lo), ssq_out
  bf16_t* y_packed;
  float* x;
  const float* gain;
  float* ssq_out;
};

// Skinny GEMM on the matrix cores with a fused epilogue.  planes = 2 uses X = hi + lo, planes = 1 only the
// hi plane.  rows_pad % 64 == 0, N % 16 == 0 (N % 64 for the paired epilogues), K % 128 == 0.  `part` holds
// plan.splits slices of part_stride >= rows_pad * round_up(N, 64) floats, `counters` one zeroed int per output tile (left zeroed).
// Returns false (nothing launched) on an unsupported shape.
struct GemmPlan {
  int nwn;     // 0: stream kernel (one feature group per workgroup); 2..4: wide kernel, groups per workgroup;
               // 8, 9: large-row kernel (256 features x 128 / 256 rows per workgroup)
  int nw;      // stream kernel: wavefronts splitting the k range
  int splits;  // split-K slices
  // large-row kernel only: x_main > 0 = two launches, the first x_main feature tiles (whole scheduling rounds)
  // unsplit, the others with k split rem_splits ways so that they fill one more round
  int x_main = 0, rem_splits = 0;
};
GemmPlan bf16_gemm_plan(int rows_pad, int N, int K, int planes, int max_splits = 8);
int bf16_gemm_tiles(int rows_pad, int N, const GemmPlan& plan);
bool bf16_gemm(float* part, int64_t part_stride, const bf16_t* x_packed, const bf16_t* w_packed, int rows_pad,
               int N, int K, int planes, const GemmPlan& plan, int* counters, const GemmEpilogue& epi,
               hipStream_t s);
// Tree-masked attention: split-KV partials (running max, sum, unnormalised output per key range), then - when
// there is more than one key range - the merge; the result is written as PackX(o), hi/lo, for the O projection.
// n_splits from bf16_attn_pick_splits.  part_o: [B][H][n_splits][n_step][hd] fp32, part_ml: [B][H][n_splits][n_step]
// float2 (max, sum).  q_planes: 2 = the queries are hi + lo pairs, 1 = their lo plane is known to be zero
// (queries given as bf16).
int bf16_attn_pick_splits(const StepMeta& m, const ModelDims& md, int max_p, int64_t part_rows_cap);
// Query planes the model path hands to the attention: 2, except 1 (hi plane only) when 512 or more rows share each
// K / V byte (grouped query heads x tree rows per kv head): there the attention is bound by the matrix cores and the lo
// plane is a third of their work, while the keys are stored with the same 11-bit rounding anyway, so the score error
// grows by at most sqrt(2).
int bf16_attn_query_planes(const StepMeta& m, const ModelDims& md);
void bf16_tree_attention(bf16_t* o_packed, int rows_pad, const bf16_t* q_packed, const bf16_t* kc, const bf16_t* vc,
                         float* part_o, float2* part_ml, int n_splits, int q_planes, const StepMeta& m,
                         const ModelDims& md, hipStream_t s);
void bf16_kv_compact(bf16_t* const* kc, bf16_t* const* vc, const int32_t* path, const int32_t* n_acc,
                     const StepMeta& m, const ModelDims& md, int stride, hipStream_t s);
void bf16_kv_copy(bf16_t* kcache, bf16_t* vcache, bf16_t* k_plain, bf16_t* v_plain, bool to_cache,
                  int seq, int first, int n, const ModelDims& md, hipStream_t s);
void bf16_kv_clear(bf16_t* kcache, bf16_t* vcache, int seq, int first, int n, const ModelDims& md, hipStream_t s);
void bf16_scatter_tree_kv(bf16_t* kc, bf16_t* vc, const bf16_t* k_tree, const bf16_t* v_tree,
                          const StepMeta& m, const ModelDims& md, int max_nodes, hipStream_t s);
void bf16_pack_q(bf16_t* q_packed, const bf16_t* q_plain, const StepMeta& m, const ModelDims& md,
                 int max_nodes, hipStream_t s);
void bf16_unpack_o(bf16_t* out_plain, const bf16_t* o_packed, int rows_pad, const StepMeta& m,
                   const ModelDims& md, int max_nodes, hipStream_t s);

}  // namespace ded
