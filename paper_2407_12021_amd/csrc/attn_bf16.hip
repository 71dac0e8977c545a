// Tree-masked attention for the 16-bit path (f16 K/V cache, head_dim 128), split over the key axis.
//
// Work unit: (sequence, kv head, tile of "virtual rows", key range).  The virtual rows of a kv head are its G
// query heads x n_step tree rows (vr = g * n_step + node), so grouped-query heads share every K/V byte that is
// fetched.  A workgroup streams its key range in tiles of 64 keys: the K and V^T fragments of a tile (32 KiB,
// contiguous in the cache) are fetched with fully coalesced 16-byte loads, parked in LDS (double buffered) and
// consumed by the wavefronts, each of which owns one or two blocks of 16 rows:
//     S^T = K . Q^T           v_mfma_f32_16x16x32_f16, A = key fragment (LDS), B = query fragment (VGPR, hi + lo)
//     online soft-max          per lane: 1 row, 8 keys of a 32-key chunk; row max via two lane swaps
//     O^T += V^T . P^T         A = value fragment (LDS), B = weights straight from the S^T registers
//     l   += 1^T . P^T         the weights' sum, by the matrix cores as well (a row of ones)
// The key rows of a 32-key group are interleaved inside the two 16-row tiles (see packk_index) so that after the
// first product a lane holds 8 consecutive keys - exactly the B-operand slice the second product needs, with no
// cross-lane traffic.  The ancestor mask is a per-row bitmask over tree slots; chunks that lie entirely inside
// the prefix skip all mask work and take the short soft-max path (3 arithmetic instructions per score).
// Each workgroup writes (running max, sum, unnormalised output) per row; a second kernel merges the key ranges
// in a fixed order and writes the output as hi/lo f16 in PackX for the O projection.
#include <algorithm>
#include <type_traits>

#include "bf16_layout.h"
#include "ded_kernels.h"

namespace ded {

namespace {

constexpr int TILE = 64;         // keys per tile
constexpr int TILE_U4 = 1024;    // uint4 units of one K (or V) tile: 64 keys * 128 dims * 2 B / 16
constexpr float NEG_BIG = -1.0e30f;

constexpr int CHUNK = 32;  // keys per chunk: the contraction length of one matrix instruction of the second product

// maximum over the four lanes (lane ^ 16, lane ^ 32, lane ^ 48) that hold the keys of one row, by the row / half
// swaps of this GPU: after swapping with a copy of itself, one result holds the even rows (lower half) twice, the
// other the odd rows (upper half) twice
__device__ __forceinline__ float quad_max(float v) {
  unsigned u = __float_as_uint(v);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float m = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  u = __float_as_uint(m);
  const auto b = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

// Online soft-max step of ONE row block (16 rows, one per lane & 15) over ONE 32-key chunk.  s[c2][i] is the raw
// score (q . k, unscaled) of key key0 + quad * 8 + c2 * 4 + i against the lane's row.  Updates the row's running
// maximum m_run (in units of score * scale * log2 e), returns the factor alpha by which everything accumulated
// so far has to be multiplied, and the chunk's weights exp2(score' - m) as the f16 B operand of the second
// product (the lane's eight consecutive keys).  The weights' sum is NOT formed here: the matrix cores add it up
// (a row of ones in front of V^T), from the same rounded weights that they multiply with V.
// plain = the chunk lies inside the prefix, every key is visible: max over the raw scores (the scale is
// positive), then one fused multiply-add, one exponential and half a packed conversion (round towards zero; the
// normaliser sees the same rounding) per score.  Otherwise the ancestor mask row (4 words over tree slots) decides
// per key, and a row that has seen no visible key yet keeps weights of exactly zero.
__device__ __forceinline__ void softmax_chunk(const f32x4_t (&s)[2], bool plain, int key0, int quad, int P, int T,
                                              const uint64_t* mrow, float scale_log2e, float& m_run, float& alpha,
                                              f16x8_t& pb) {
  typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
  if (plain) {
    float mx = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                     fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
    mx = quad_max(mx);
    const float m_new = fmaxf(m_run, mx * scale_log2e);
    alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    const float neg_m = -m_new;
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
      const float e0 = __builtin_amdgcn_exp2f(fmaf(s[j >> 2][j & 3], scale_log2e, neg_m));
      const float e1 = __builtin_amdgcn_exp2f(fmaf(s[j >> 2][(j & 3) + 1], scale_log2e, neg_m));
      const h2_t h = __builtin_bit_cast(h2_t, __builtin_amdgcn_cvt_pkrtz(e0, e1));
      pb[j] = h[0];
      pb[j + 1] = h[1];
    }
  } else {
    const uint64_t w0 = mrow[0], w1 = mrow[1], w2 = mrow[2], w3 = mrow[3];
    float p[8];
    float mx = NEG_BIG;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int key = key0 + quad * 8 + j;
      const int tt = key - P;  // tree slot of this key (negative inside the prefix)
      const int wi = tt >> 6;
      const uint64_t word = wi == 0 ? w0 : wi == 1 ? w1 : wi == 2 ? w2 : w3;
      const bool vis = (key < P) | ((key < T) & (bool)((word >> (tt & 63)) & 1ull));  // no short circuit: no branches
      const float v = vis ? s[j >> 2][j & 3] * scale_log2e : NEG_BIG;
      p[j] = v;
      mx = fmaxf(mx, v);
    }
    mx = quad_max(mx);
    const float m_new = fmaxf(m_run, mx);
    alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
      const float e0 = p[j] > 0.5f * NEG_BIG ? __builtin_amdgcn_exp2f(p[j] - m_new) : 0.f;
      const float e1 = p[j + 1] > 0.5f * NEG_BIG ? __builtin_amdgcn_exp2f(p[j + 1] - m_new) : 0.f;
      const h2_t h = __builtin_bit_cast(h2_t, __builtin_amdgcn_cvt_pkrtz(e0, e1));
      pb[j] = h[0];
      pb[j + 1] = h[1];
    }
  }
}

__device__ __forceinline__ f16x8_t f16_ones() {
  f16x8_t v;
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (_Float16)1.0f;
  return v;
}


// ------------------------------------------------------------------------------------------
// Tiled kernel.  Work unit: (sequence, kv head, row tile, key range).  The K / V tiles of 64 keys (32 KiB,
// contiguous in the cache) go global -> register -> LDS (double buffered, one barrier per tile) once per
// workgroup.  A wavefront owns RBW row blocks of 16 rows.  With RBW = 2 a key or value fragment read from LDS
// feeds two (four with the lo query plane) matrix instructions, queries take 32 / 64 registers and the output tile
// 64, so two wavefronts still fit a SIMD and one's soft-max arithmetic runs under the other's matrix instructions.
// NW wavefronts form NW / KS row groups x KS key groups: with KS = 1 every wavefront takes both 32-key chunks of
// a tile; with KS = 2 a wavefront takes one chunk of every tile, so that few rows still spread over all
// wavefronts, and the two key groups' (max, sum, O) are merged through LDS at the end, in key-group order.
// Shapes in use (rows per workgroup tile = NW / KS * RBW * 16):
//   64 rows  = 8 wavefronts as 4 row groups of 16 rows x 2 key groups: trees of one sequence;
//   128 rows = 8 wavefronts as 4 row groups of 32 rows x 2 key groups, or (one key range) 8 wavefronts x 16 rows;
//   256 rows = 8 wavefronts x 32 rows, all keys each: many rows per kv head (batched trees, grouped-query heads),
//              where the matrix cores bound the operation and LDS bytes per matrix instruction decide how busy
//              they are.
// Workgroup indices are remapped so that neighbours in (key range, row tile) order - which fetch the same K / V -
// run on the same XCD and meet in its L2.
// ------------------------------------------------------------------------------------------
// (PIPE: the prefix tiles of shapes in which every wavefront takes all keys go through the software pipeline below)
template <int QP, int NW, int KS, int RBW>
__global__ __launch_bounds__(NW * 64, 2) void tree_attn_tiled_kernel(
    const uint4* __restrict__ qp, const uint4* __restrict__ kc, const uint4* __restrict__ vc,
    float* __restrict__ part_o, float2* __restrict__ part_ml, const uint64_t* __restrict__ mask,
    const int32_t* __restrict__ seq_p, const int32_t* __restrict__ seq_n, int n_step, int H, int Hkv, int cap,
    int n_splits, float scale_log2e, bf16_t* __restrict__ o_final, int RB_total) {
  constexpr int NT = NW * 64;          // threads
  constexpr int RG = NW / KS;          // row groups (of RBW * 16 rows) per workgroup
  constexpr int UPT = 2 * TILE_U4 / NT;  // staged 16-byte units per thread and tile (K and V)
  static_assert(KS == 1 || KS == 2, "a tile holds two chunks");
  static_assert(UPT == 4 || UPT == 8, "4 or 8 wavefronts");
  __shared__ uint4 lds[2][2 * TILE_U4];  // [buffer][K tile | V tile], 2 x 32 KiB; reused for the key-group merge
  __shared__ float2 lds_ml[KS == 2 ? RG * RBW * 64 : 1];  // (max, sum) of key group 1 for that merge
  constexpr bool PIPE = KS == 1 && ((RBW == 2 && QP == 1) || RBW == 1);
  __shared__ uint4 lds_k3[PIPE ? TILE_U4 : 1];  // third K slot of the pipelined prefix loop
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rg = wave % RG, kg = wave / RG;
  // XCD-aware order: hardware hands consecutive workgroup ids to the 8 XCDs in turn
  int lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  const int total = gridDim.x * gridDim.y * gridDim.z;
  if ((total & 7) == 0) lin = (lin & 7) * (total >> 3) + (lin >> 3);
  const int split = lin % n_splits;
  const int row_tile = (lin / n_splits) % gridDim.y, bz = lin / (n_splits * gridDim.y);
  const int b = bz / Hkv, kvh = bz - b * Hkv;
  const int G = H / Hkv;
  const int P = seq_p[b], N = seq_n[b], T = P + N;
  const int n_tiles = (T + TILE - 1) / TILE;
  const int n_plain = P / TILE;  // tiles entirely inside the prefix
  // key ranges of equal cost: a tile that holds tree keys (mask work) counts as two prefix tiles
  const int cost_total = n_plain + 2 * (n_tiles - n_plain);
  auto tile_at_cost = [&](int c) { return c <= n_plain ? c : n_plain + (c - n_plain + 1) / 2; };
  const int t_begin = tile_at_cost((int)((int64_t)split * cost_total / n_splits));
  const int t_end = split + 1 == n_splits ? n_tiles : tile_at_cost((int)((int64_t)(split + 1) * cost_total / n_splits));
  const int VR = G * n_step;
  const int vrb0 = (row_tile * RG + rg) * RBW;              // first row block of this wavefront
  const int nrb = max(0, min(RBW, VR / 16 - vrb0));         // row blocks that hold rows
  const int row_in = lane & 15, quad = lane >> 4;
  const uint4* kbase = kc + (int64_t)bz * cap * 16;
  const uint4* vbase = vc + (int64_t)bz * cap * 16;

  struct Stage {
    uint4 k0, k1, k2, k3, v0, v1, v2, v3;  // UPT / 2 of each kind are used
  };
  auto load_tile = [&](int t) {
    const uint4* ks = kbase + (int64_t)t * TILE_U4 + tid;
    const uint4* vs = vbase + (int64_t)t * TILE_U4 + tid;
    Stage st;
    st.k0 = ks[0], st.k1 = ks[NT];
    st.v0 = vs[0], st.v1 = vs[NT];
    if (UPT == 8) {
      st.k2 = ks[2 * NT], st.k3 = ks[3 * NT];
      st.v2 = vs[2 * NT], st.v3 = vs[3 * NT];
    }
    return st;
  };
  auto store_tile = [&](int buf, const Stage& st) {
    uint4* d = lds[buf] + tid;
    d[0] = st.k0, d[NT] = st.k1;
    d[TILE_U4] = st.v0, d[TILE_U4 + NT] = st.v1;
    if (UPT == 8) {
      d[2 * NT] = st.k2, d[3 * NT] = st.k3;
      d[TILE_U4 + 2 * NT] = st.v2, d[TILE_U4 + 3 * NT] = st.v3;
    }
  };
  // the first tile is requested before anything else (queries, mask rows): it has the longest way to come
  Stage st_first;
  if (t_begin < t_end) st_first = load_tile(t_begin);

  f16x8_t q[RBW][4 * QP];
  int node_of[RBW], g_of[RBW];
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) {
    const int vrb = rb < nrb ? vrb0 + rb : 0;
    const uint4* qsrc = qp + (((int64_t)bz * (VR / 16) + vrb) * 8 << 6) + lane;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int pl = 0; pl < QP; ++pl) q[rb][kk * QP + pl] = __builtin_bit_cast(f16x8_t, qsrc[(kk * 2 + pl) << 6]);
    const int vr = vrb * 16 + row_in;
    g_of[rb] = vr / n_step;
    node_of[rb] = vr - g_of[rb] * n_step;
  }
  // o_l = ones . P^T: the running sum of each row's weights, present in every element
  f32x4_t o[RBW][8], o_l[RBW];
  float m_run[RBW];
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) {
    m_run[rb] = NEG_BIG;
    o_l[rb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int hb = 0; hb < 8; ++hb) o[rb][hb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }
  const f16x8_t ones = f16_ones();

  // one 32-key chunk (kb = 0, 1) of the tile in LDS buffer `buf` against the wavefront's rows
  auto compute_chunk = [&](int buf, int t, int kb) {
    const uint4* lk = lds[buf] + ((kb * 8) << 6) + lane;
    const uint4* lv = lds[buf] + TILE_U4 + ((kb * 8) << 6) + lane;
    const int key0 = t * TILE + kb * CHUNK;
    const bool plain = key0 + CHUNK <= P;  // whole chunk inside the prefix: every key visible to every row
    f16x8_t kf[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) kf[i] = __builtin_bit_cast(f16x8_t, lk[i << 6]);
    f16x8_t pb[RBW];
    float alpha[RBW];
    bool rescale = false;
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
      // S^T: s[c2][i] = score of key  key0 + quad*8 + c2*4 + i  against row (vrb0 + rb)*16 + row_in
      f32x4_t s[2];
#pragma unroll
      for (int c2 = 0; c2 < 2; ++c2) {
        f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
        f32x4_t acc_lo = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[c2 * 4 + kk], q[rb][kk * QP], acc, 0, 0, 0);
          if (QP == 2) acc_lo = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[c2 * 4 + kk], q[rb][kk * QP + QP - 1], acc_lo, 0, 0, 0);
        }
        s[c2] = QP == 2 ? acc + acc_lo : acc;
      }
      softmax_chunk(s, plain, key0, quad, P, T, mask + ((int64_t)b * n_step + node_of[rb]) * 4, scale_log2e,
                    m_run[rb], alpha[rb], pb[rb]);
      rescale |= alpha[rb] != 1.0f;
    }
    if (__any(rescale)) {
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) {
        o_l[rb] *= alpha[rb];
#pragma unroll
        for (int hb = 0; hb < 8; ++hb) o[rb][hb] *= alpha[rb];
      }
    }
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) o_l[rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones, pb[rb], o_l[rb], 0, 0, 0);
#pragma unroll
    for (int hb = 0; hb < 8; ++hb) {
      const f16x8_t a = __builtin_bit_cast(f16x8_t, lv[hb << 6]);
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) o[rb][hb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, pb[rb], o[rb][hb], 0, 0, 0);
    }
  };

  auto compute_tile = [&](int buf, int t) {
    if (nrb > 0) {
      if (KS == 2) {
        compute_chunk(buf, t, kg);
      } else {
#pragma unroll 1
        for (int kb = 0; kb < 2; ++kb) compute_chunk(buf, t, kb);
      }
    }
  };
  if (t_begin < t_end) {
    const int t_last = t_end - 1;  // fetches past the range re-read its last tile: in bounds, and no branches
    store_tile(0, st_first);
    __syncthreads();
    int buf = 0;
    int t = t_begin;
    if constexpr (PIPE) {
      // Many rows per kv head: the matrix cores and the soft-max arithmetic bound the kernel, each busy about half
      // of the time when a wavefront runs  scores -> soft-max -> second product  strictly one after the other.  The
      // tiles that lie inside the prefix (no mask work) therefore go through a software pipeline, one 32-key chunk
      // per stage: while chunk c gets its weights (exp2, conversion) and its second product, the scores of chunk
      // c + 1 are already there and their exponents and row maxima are formed behind the second product's matrix
      // instructions; nothing in a stage waits for a matrix result issued in the same stage.  For that the K half of a
      // tile is parked in LDS one tile ahead of its V half (three K slots, two V slots).
      // The running maximum becomes a REFERENCE that is raised only when a row's exponent exceeds 8 (weights stay
      // below 2^8 in f16; numerator and normaliser carry the same reference, so the quotient is unchanged): the
      // rescale of the output tile is a rarely taken branch between the stages, not arithmetic in every chunk.  The
      // scores are kept as exponents relative to the reference, so a row maximum is taken over results of fused
      // multiply-adds (canonical numbers, no quieting moves), across the four lanes of a row with this GPU's lane
      // swaps (no LDS round trip), and only in that branch: the test itself looks at each lane's own eight keys.
      // Measured on the Llama-3-8B shape (8 x 256 nodes, 16384-key prefixes): 704 -> 548 us per layer.
      const int t_pipe = min(t_end, n_plain);  // tiles [t_begin, t_pipe) hold prefix keys only
      const bool wg_full = (row_tile + 1) * (RG * RBW) <= VR / 16;  // the same for every wavefront (barriers differ)
      if (wg_full && t_pipe - t_begin >= 2) {
        static_assert(!PIPE || UPT == 4, "two units of K and two of V per thread and tile");
        typedef f32x4_t Scores[RBW][2];
        struct Half {
          uint4 a, b;
        };
        auto load_half = [&](const uint4* base, int tt) {
          const uint4* src = base + (int64_t)tt * TILE_U4 + tid;
          Half h;
          h.a = src[0], h.b = src[NT];
          return h;
        };
        auto store_half = [&](uint4* slot, const Half& h) {
          uint4* d = slot + tid;
          d[0] = h.a, d[NT] = h.b;
        };
        // raw scores -> soft-max exponents relative to the rows' present reference, in place, and the largest
        // exponent among each lane's eight keys (the fused multiply-adds' results are canonical numbers, so the maxima
        // need no quieting moves; the four lanes of a row are only combined if some lane asks for a new reference)
        auto exponents = [&](Scores& s, float (&mx)[RBW]) {
#pragma unroll
          for (int rb = 0; rb < RBW; ++rb) {
            const float neg_m = -m_run[rb];
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
              for (int i = 0; i < 4; ++i) s[rb][c2][i] = fmaf(s[rb][c2][i], scale_log2e, neg_m);
            const float v = fmaxf(fmaxf(fmaxf(s[rb][0][0], s[rb][0][1]), fmaxf(s[rb][0][2], s[rb][0][3])),
                                  fmaxf(fmaxf(s[rb][1][0], s[rb][1][1]), fmaxf(s[rb][1][2], s[rb][1][3])));
            mx[rb] = v;
          }
        };
        auto weights = [&](const Scores& s, f16x8_t (&pb)[RBW]) {
          typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
#pragma unroll
          for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
            for (int j = 0; j < 8; j += 2) {
              const float e0 = __builtin_amdgcn_exp2f(s[rb][j >> 2][j & 3]);
              const float e1 = __builtin_amdgcn_exp2f(s[rb][j >> 2][(j & 3) + 1]);
              const h2_t h = __builtin_bit_cast(h2_t, __builtin_amdgcn_cvt_pkrtz(e0, e1));
              pb[rb][j] = h[0];
              pb[rb][j + 1] = h[1];
            }
        };
        auto v_frags = [&](int b_, int kb, f16x8_t (&vf)[8]) {
          const uint4* lv = lds[b_] + TILE_U4 + ((kb * 8) << 6) + lane;
#pragma unroll
          for (int hb = 0; hb < 8; ++hb) vf[hb] = __builtin_bit_cast(f16x8_t, lv[hb << 6]);
        };
        auto pv = [&](const f16x8_t (&vf)[8], const f16x8_t (&pb)[RBW]) {
#pragma unroll
          for (int rb = 0; rb < RBW; ++rb) o_l[rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones, pb[rb], o_l[rb], 0, 0, 0);
#pragma unroll
          for (int hb = 0; hb < 8; ++hb)
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) o[rb][hb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf[hb], pb[rb], o[rb][hb], 0, 0, 0);
        };
        // a row with an exponent above 8 gets a new reference (its present maximum): the output tile and the pending
        // exponents of that row move with it
        auto raise = [&](const float (&mx)[RBW], Scores& s) {
          bool need = false;
#pragma unroll
          for (int rb = 0; rb < RBW; ++rb) need |= mx[rb] > 8.0f;
          if (__any(need)) {
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) {
              const float row_mx = quad_max(mx[rb]);
              const float delta = row_mx > 8.0f ? row_mx : 0.f;
              const float alpha = __builtin_amdgcn_exp2f(-delta);
              m_run[rb] += delta;
              o_l[rb] *= alpha;
#pragma unroll
              for (int hb = 0; hb < 8; ++hb) o[rb][hb] *= alpha;
#pragma unroll
              for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                for (int i = 0; i < 4; ++i) s[rb][c2][i] -= delta;
            }
          }
        };
        Scores sa, sb;  // scores of a tile's first / second chunk
        float mx[RBW];
        f16x8_t pb[RBW];
        // K halves of tiles t, t + 1 and (being written) t + 2; the V half of tile t sits in lds[buf], t + 1 goes to
        // lds[buf ^ 1].  A third K slot, because both K(t) (second chunk) and K(t + 1) (first chunk) are read in the
        // iteration that parks K(t + 2).
        uint4 *k_cur = lds[0], *k_next = lds[1], *k_free = lds_k3;
        auto qk = [&](const uint4* kslot, int kb, Scores& s) {
          const uint4* lk = kslot + ((kb * 8) << 6) + lane;
          f16x8_t kf[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) kf[i] = __builtin_bit_cast(f16x8_t, lk[i << 6]);
#pragma unroll
          for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) {
              f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
              for (int kk = 0; kk < 4; ++kk) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[c2 * 4 + kk], q[rb][kk * QP], acc, 0, 0, 0);
              if constexpr (QP == 2) {  // the lo query plane in a chain of its own, as in the general loop
                f32x4_t acc_lo = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                  acc_lo = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[c2 * 4 + kk], q[rb][kk * QP + 1], acc_lo, 0, 0, 0);
                acc = acc + acc_lo;
              }
              s[rb][c2] = acc;
            }
        };
        {
          const Half kn = load_half(kbase, min(t + 1, t_last));
          qk(k_cur, 0, sa);
#pragma unroll
          for (int rb = 0; rb < RBW; ++rb) {  // first reference of a row: the maximum of its first chunk
            const float v = fmaxf(fmaxf(fmaxf(sa[rb][0][0], sa[rb][0][1]), fmaxf(sa[rb][0][2], sa[rb][0][3])),
                                  fmaxf(fmaxf(sa[rb][1][0], sa[rb][1][1]), fmaxf(sa[rb][1][2], sa[rb][1][3])));
            m_run[rb] = quad_max(v) * scale_log2e;
          }
          exponents(sa, mx);
          store_half(k_next, kn);
          __syncthreads();
        }
        auto tile_body = [&](auto last_tag) {
          constexpr bool LAST = decltype(last_tag)::value;  // last prefix tile: nothing of tile t + 1 is computed here
          Half kn, vn;
          if constexpr (!LAST) {
            kn = load_half(kbase, min(t + 2, t_last));
            vn = load_half(vbase, min(t + 1, t_last));
          }
          // first chunk of tile t, scores of its second chunk
          {
            f16x8_t vf[8];
            qk(k_cur, 1, sb);
            v_frags(buf, 0, vf);
            __builtin_amdgcn_sched_barrier(0);  // the V fragments are requested before the exponentials start
            weights(sa, pb);
            pv(vf, pb);
          }
          exponents(sb, mx);
          raise(mx, sb);
          // second chunk of tile t, scores of the first chunk of tile t + 1
          {
            f16x8_t vf[8];
            if constexpr (!LAST) qk(k_next, 0, sa);
            v_frags(buf, 1, vf);
            __builtin_amdgcn_sched_barrier(0);
            weights(sb, pb);
            pv(vf, pb);
          }
          if constexpr (!LAST) {
            exponents(sa, mx);
            store_half(k_free, kn);
            store_half(lds[buf ^ 1] + TILE_U4, vn);
          }
          __syncthreads();
          if constexpr (!LAST) raise(mx, sa);
        };
        for (; t + 1 < t_pipe; ++t) {
          tile_body(std::false_type{});
          uint4* const k_old = k_cur;
          k_cur = k_next, k_next = k_free, k_free = k_old;
          buf ^= 1;
        }
        tile_body(std::true_type{});
        ++t;
        if (t < t_end) {  // the general loop expects its first tile whole in lds[0]
          store_tile(0, load_tile(t));
          __syncthreads();
          buf = 0;
        }
      }
    }
    for (; t < t_end; ++t) {
      const Stage st = load_tile(min(t + 1, t_last));
      compute_tile(buf, t);
      store_tile(buf ^ 1, st);
      __syncthreads();
      buf ^= 1;
    }
  }

  if (KS == 2) {
    // key group 1 hands its (max, sum, O) to key group 0 of the same rows through LDS (every workgroup barrier of
    // the loop has been passed by all wavefronts, so the tile buffers are free)
    float4* xo = reinterpret_cast<float4*>(&lds[0][0]);  // [rg][rb][hb][lane]: RG * 16 KiB <= the two tile buffers
    float2* xml = lds_ml;                                // [rg][rb][lane]
    if (kg == 1) {
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) {
        xml[(rg * RBW + rb) * 64 + lane] = make_float2(m_run[rb], o_l[rb][0]);
#pragma unroll
        for (int hb = 0; hb < 8; ++hb)
          xo[((rg * RBW + rb) * 8 + hb) * 64 + lane] = make_float4(o[rb][hb][0], o[rb][hb][1], o[rb][hb][2], o[rb][hb][3]);
      }
    }
    __syncthreads();
    if (kg == 1) return;
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
      const float2 other = xml[(rg * RBW + rb) * 64 + lane];
      const float M = fmaxf(m_run[rb], other.x);
      const float w0 = __builtin_amdgcn_exp2f(m_run[rb] - M), w1 = __builtin_amdgcn_exp2f(other.x - M);
      o_l[rb][0] = o_l[rb][0] * w0 + other.y * w1;
      m_run[rb] = M;
#pragma unroll
      for (int hb = 0; hb < 8; ++hb) {
        const float4 v = xo[((rg * RBW + rb) * 8 + hb) * 64 + lane];
        o[rb][hb] = o[rb][hb] * w0 + f32x4_t{v.x, v.y, v.z, v.w} * w1;
      }
    }
  }

#pragma unroll
  for (int rb = 0; rb < RBW; ++rb) {
    if (rb >= nrb) continue;
    const float l = o_l[rb][0];  // every element of the ones-row product holds the row's sum
    const int h = kvh * G + g_of[rb];
    if (o_final) {
      // a single key range: nothing to merge, the row is normalised here and written as the O projection's input
      // (hi / lo f16 in PackX; four consecutive features sit side by side inside a fragment)
      const float inv = 1.0f / l;
      const int r = b * n_step + node_of[rb];
#pragma unroll
      for (int hb = 0; hb < 8; ++hb) {
        uint16_t hi[4], lo[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) split_f16(o[rb][hb][i] * inv, hi[i], lo[i]);
        const int feat = h * 128 + hb * 16 + quad * 4;
        *reinterpret_cast<uint2*>(o_final + packx_index(r, feat, RB_total, 0)) =
            make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
        *reinterpret_cast<uint2*>(o_final + packx_index(r, feat, RB_total, 1)) =
            make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
      }
      continue;
    }
    const int64_t prow = (((int64_t)b * H + h) * n_splits + split) * n_step + node_of[rb];
    float* po = part_o + prow * 128 + quad * 4;
#pragma unroll
    for (int hb = 0; hb < 8; ++hb)
      *reinterpret_cast<float4*>(po + hb * 16) = make_float4(o[rb][hb][0], o[rb][hb][1], o[rb][hb][2], o[rb][hb][3]);
    if (quad == 0) part_ml[prow] = make_float2(m_run[rb], l);
  }
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

// Kernel shape by the rows per kv head (grouped query heads x padded tree rows): see tree_attn_tiled_kernel.
// Up to 64 rows: 4 row groups of 16 rows x 2 key groups; up to 128: 4 row groups of 32 rows x 2 key groups;
// beyond: 8 row groups of 32 rows.  Eight wavefronts per workgroup in every shape: with four, the 64-row shape
// left half of each CU's issue slots empty while it waited on the K/V stream (config 2: 25.6 -> 24.5 us).
enum { ATTN_T64 = 0, ATTN_T128 = 1, ATTN_T256 = 2 };
static int attn_kernel_for(const StepMeta& m, const ModelDims& md) {
  const int VR = (md.H / md.Hkv) * m.n_step;
  return VR <= 64 ? ATTN_T64 : VR <= 128 ? ATTN_T128 : ATTN_T256;
}
static int attn_tile_rows(int kind) { return kind == ATTN_T256 ? 256 : kind == ATTN_T128 ? 128 : 64; }

int bf16_attn_query_planes(const StepMeta& m, const ModelDims& md) {
  return (md.H / md.Hkv) * m.n_step >= 512 ? 1 : 2;
}

int bf16_attn_pick_splits(const StepMeta& m, const ModelDims& md, int max_p, int64_t part_rows_cap) {
  const int G = md.H / md.Hkv;
  const int kind = attn_kernel_for(m, md);
  const int row_tiles = (G * m.n_step + attn_tile_rows(kind) - 1) / attn_tile_rows(kind);
  const int base = std::max(1, m.batch * md.Hkv * row_tiles);
  const int tiles = (max_p + m.n_step + TILE - 1) / TILE;
  // One workgroup per CU is resident (8 wavefronts of 150-250 registers), so a launch runs in rounds of 256
  // workgroups; a round lasts its tiles plus a start-up of ~2.5 tile times (queries, first tile).  Splitting the
  // keys costs the merge launch (~3 tile times) and the partials, written once and read once through memory
  // (1 KiB per row and range at ~5.5 TB/s; a tile time is ~2 us).  Calibrated on configs 2-4: config 2 is 1 us
  // faster with 8 ranges than with 16, the benchmark step's attention 4 % faster with 6 than with 8, and 160
  // workgroups of 34 tiles with 128 rows each (config 4) are faster unsplit than as 480 workgroups of 12.
  const int ns_max = std::min(16, std::max(1, tiles / (kind == ATTN_T256 ? 4 : 2)));  // >= 2 (4) tiles per range
  const double rows_total = (double)m.batch * md.H * m.n_step;
  int ns = 1;
  double best = 1e300;
  for (int n = 1; n <= ns_max; ++n) {
    if (n > 1 && rows_total * n > (double)part_rows_cap) break;
    const int rounds = (base * n + 255) / 256;
    const double cost = rounds * ((tiles + n - 1) / n + 2.5) + (n > 1 ? 3.0 + n * rows_total * 1024.0 / 5.5e6 / 2.0 : 0.0);
    if (cost < best) {
      best = cost;
      ns = n;
    }
  }
  return ns;
}

void bf16_tree_attention(bf16_t* o_packed, int rows_pad, const bf16_t* q_packed, const bf16_t* kc, const bf16_t* vc,
                         float* part_o, float2* part_ml, int n_splits, int q_planes, const StepMeta& m,
                         const ModelDims& md, hipStream_t s) {
  if (md.hd != 128 || n_splits < 1 || m.rows <= 0) return;
  const int G = md.H / md.Hkv;
  const int VR = G * m.n_step;
  const int kind = attn_kernel_for(m, md);
  const int row_tiles = (VR + attn_tile_rows(kind) - 1) / attn_tile_rows(kind);
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)md.hd);
  const dim3 grid(n_splits, row_tiles, m.batch * md.Hkv);
  bf16_t* o_final = n_splits == 1 ? o_packed : nullptr;  // one key range: the kernel finishes the rows itself
#define DED_ATTN_ARGS                                                                                              \
  reinterpret_cast<const uint4*>(q_packed), reinterpret_cast<const uint4*>(kc), reinterpret_cast<const uint4*>(vc), \
      part_o, part_ml, m.mask, m.seq_p, m.seq_n, m.n_step, md.H, md.Hkv, md.cap, n_splits, scale_log2e, o_final,   \
      rows_pad / 16
#define DED_ATTN_GO(NW, KS, RBW)                                                                                       \
  if (q_planes == 1) hipLaunchKernelGGL((tree_attn_tiled_kernel<1, NW, KS, RBW>), grid, dim3(NW * 64), 0, s, DED_ATTN_ARGS); \
  else hipLaunchKernelGGL((tree_attn_tiled_kernel<2, NW, KS, RBW>), grid, dim3(NW * 64), 0, s, DED_ATTN_ARGS);
  if (kind == ATTN_T256) {
    DED_ATTN_GO(8, 1, 2)
  } else if (kind == ATTN_T128) {
    // one key range per workgroup (enough sequences and heads to fill the chip: batched trees): 8 wavefronts x 16
    // rows, all keys each, whose prefix tiles run through the software pipeline (69 -> 63 us per layer at 4 x 128 rows
    // on 2048-key prefixes); split ranges are short and keep the shape that reads every K / V fragment from LDS once
    // per two row blocks
    if (n_splits == 1) {
      DED_ATTN_GO(8, 1, 1)
    } else {
      DED_ATTN_GO(8, 2, 2)
    }
  } else {
    DED_ATTN_GO(8, 2, 1)
  }
#undef DED_ATTN_GO
#undef DED_ATTN_ARGS
  if (n_splits > 1) {
    const int total = m.rows * md.H * 32;
    hipLaunchKernelGGL(tree_attn_merge_kernel, dim3((total + 255) / 256), dim3(256), 0, s, o_packed, rows_pad / 16,
                       part_o, part_ml, n_splits, m.n_step, md.H, total);
  }
}

}  // namespace ded
