// Greedy acceptance fused with the LM head (arXiv 2408.15562, Methodology, "LM Head": the last
// linear map from the target's features to the vocabulary; Preliminaries, validation phase;
// Experiments "Settings": temperature 0). The [rows, V] logits are never written: a skinny
// bf16 GEMM (rows = B*N <= a few hundred, K = hidden size, V columns) keeps every logit in the
// accumulators of the matrix cores and leaves only (max, first argmax) per row and vocabulary
// slice; a second, small kernel merges the slices and walks the tree. gfx950 (CDNA4) only.
//
// The GEMM is bound by streaming the V x K weight matrix once (262 MB for a 32000 x 4096 head);
// the hidden states (a few hundred KB) are re-read by every workgroup through LDS.
//
// Workgroup = 128 vocabulary rows x up to 128 hidden-state rows x all of K; eight wavefronts of 16
// vocabulary rows each. With `v_mfma_f32_16x16x32_bf16` and A = 16 weight rows, B = 16 hidden
// rows, both operands are "8 consecutive k per lane", i.e. plain 16-byte loads of row-major data:
// the weights go from HBM straight into registers (a ring of 16 k-steps = 16 KB requested ahead per wavefront),
// the hidden states are staged through LDS (XOR-swizzled by 16-byte chunk so that a 16-row operand
// read touches 16 different bank groups), double-buffered, one barrier per stage of 256 or 512 k. D[vocab][row] puts one hidden-state row per lane column, so the argmax over the
// vocabulary is a per-lane scan plus two lane exchanges.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "fspad.h"
#include "greedy_walk.h"
#include "stream_gemm.h"

namespace {

using fspad_detail::bf16x8;
using fspad_detail::f32x4;
using fspad_detail::StreamGemm;
typedef const __attribute__((address_space(1))) void* GlobalPtr;
typedef __attribute__((address_space(3))) void* LdsPtr;

constexpr int kVocabPerWg = 128;                            // vocabulary rows per workgroup, in every shape below
constexpr int kNone = 0x7fffffff;
constexpr int kWalkThreads = 1024;

struct LmHeadParams {
  const char* hidden;   // [M][K] bf16
  const char* weights;  // [V][K] bf16, row-major or (PACKED) in the tile order of fspad_pack_weight
  float* part_max;      // greedy: [n_slices][M]; sampling: [M][n_slices]
  int32_t* part_idx;    // greedy: [n_slices][M]
  double* part_sum;     // sampling: [M][n_slices], sum of exp((l - part_max) / T) over the slice
  float* tile_sum;      // sampling: [M][n_slices][8], the same sum per 16 tokens of the slice
  float* node_logit;    // sampling: [M], the logit of node c's own token under its parent's row
  const int32_t* draft_tokens;   // sampling: the tree, to know which logits the walk will ask for
  const int32_t* parent;
  const int32_t* n_nodes;
  int32_t M, V, K, n_slices, n_passes, rows_per_pass;
  int32_t stagger;      // stages by which consecutive workgroups are offset along k (0: all start at k = 0)
  int32_t Nmax;
  float inv_t_log2e;    // sampling: log2(e) / T
};

// (value, index) with "larger value, then lower index" order
__device__ __forceinline__ void take_better(float& v, int& i, float ov, int oi) {
  if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
}

// The LM head: MT, SPS, kRing, WAVES, VT as above; WAVES x VT = 8, i.e. 128 vocabulary rows per
// workgroup: eight wavefronts of one weight tile, two per SIMD, in every shape in use (four
// wavefronts of two tiles, one per SIMD with the whole register file, halve the LDS reads per
// product but measured slower at 256 rows: 178 against 152 us on a 32000 x 6656 head).
// MODE 0: per slice and row (max, first argmax) for the greedy walk. MODE 1: per slice and row
// (max, sum of exponentials) and the logits of the draft tokens, for the sampling walk.
template <int MT, int SPS, int kRing, int WAVES, int VT, int MODE, bool PACKED>
__global__ __launch_bounds__(64 * WAVES, (WAVES == 8 ? 2 : 1)) void lm_head_argmax_kernel(const LmHeadParams p) {
  static_assert(WAVES * VT * 16 == kVocabPerWg, "workgroup shape");
  typedef StreamGemm<MT, SPS, kRing, WAVES, VT, PACKED> G;
  constexpr int kStageBytes = G::kStageBytes;
  __shared__ __attribute__((aligned(16))) char xs[2 * kStageBytes];
  __shared__ float red_val[WAVES][MT * 16];
  __shared__ int red_idx[WAVES][MT * 16];

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, g = lane >> 4;
  const int slice = blockIdx.x / p.n_passes, pass = blockIdx.x - slice * p.n_passes;
  const int row0 = pass * p.rows_per_pass;
  const int v0 = slice * kVocabPerWg + wave * (16 * VT);
  const int n_steps = p.K >> 5;
  // workgroup `slice` walks k from stage `first_stage` on and wraps around
  const int first_step = p.stagger ? (int)(((unsigned)slice * (unsigned)p.stagger) % (unsigned)(n_steps / SPS)) * SPS : 0;

  f32x4 acc[MT][VT];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int nv = 0; nv < VT; ++nv) acc[t][nv] = f32x4{0.f, 0.f, 0.f, 0.f};
  // (the tile order pads the vocabulary to whole tiles of 16 rows)
  G::run(xs, p.hidden, p.weights, (size_t)p.K * 2, p.M, PACKED ? (p.V + 15) / 16 * 16 : p.V, row0, v0, n_steps, first_step, acc);

  if constexpr (MODE == 1) {
    // The stages are dead: the workgroup's 16*MT x 128 logits go there, as fp32, row by row
    // (16-byte chunk c of row r at chunk c ^ (r & 15): sixteen rows written at once hit different banks).
    constexpr int kRows = MT * 16;
    static_assert(kRows * 512 <= 2 * kStageBytes, "the logits of a workgroup fit the two stages");
    __syncthreads();
    float* dump = reinterpret_cast<float*>(xs);
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int nv = 0; nv < VT; ++nv) {
        const int r = t * 16 + n, chunk = (wave * (16 * VT) + 16 * nv + 4 * g) >> 2;
        *reinterpret_cast<f32x4*>(dump + r * 128 + ((chunk ^ (r & 15)) << 2)) = acc[t][nv];
      }
    __syncthreads();
    // slice statistics: sixteen lanes per row, eight logits each
    const int sub = lane & 15;
    const int slice0 = slice * kVocabPerWg;
    for (int r = threadIdx.x >> 4; r < kRows; r += 4 * WAVES) {   // uniform per 16 lanes
      float x[8];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int chunk = sub + 16 * h;
        const f32x4 v4 = *reinterpret_cast<const f32x4*>(dump + r * 128 + ((chunk ^ (r & 15)) << 2));
#pragma unroll
        for (int i = 0; i < 4; ++i) x[4 * h + i] = (slice0 + 4 * chunk + i < p.V && v4[i] == v4[i]) ? v4[i] : -INFINITY;
      }
      float m = x[0];
#pragma unroll
      for (int i = 1; i < 8; ++i) m = fmaxf(m, x[i]);
#pragma unroll
      for (int d = 1; d < 16; d <<= 1) m = fmaxf(m, __shfl_xor(m, d));
      float half[2] = {0.f, 0.f};   // this lane's share of tiles sub/4 and 4 + sub/4 (16 tokens each)
      if (m > -INFINITY) {
#pragma unroll
        for (int i = 0; i < 8; ++i) half[i >> 2] += __builtin_amdgcn_exp2f((x[i] - m) * p.inv_t_log2e);
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        half[h] += __shfl_xor(half[h], 1);
        half[h] += __shfl_xor(half[h], 2);
      }
      double dsum = (sub & 3) == 0 ? (double)half[0] + (double)half[1] : 0.0;
#pragma unroll
      for (int d = 4; d < 16; d <<= 1) dsum += __shfl_xor(dsum, d);
      if (row0 + r < p.M) {
        const size_t slot = (size_t)(row0 + r) * p.n_slices + slice;
        if ((sub & 3) == 0) {
          p.tile_sum[slot * 8 + (sub >> 2)] = half[0];
          p.tile_sum[slot * 8 + 4 + (sub >> 2)] = half[1];
        }
        if (sub == 0) {
          p.part_max[slot] = m;
          p.part_sum[slot] = dsum;
        }
      }
    }
    // the logits the walk will test: node c's token under the row of c's parent
    for (int cnode = threadIdx.x; cnode < p.M; cnode += 64 * WAVES) {
      const int b = cnode / p.Nmax, i = cnode - b * p.Nmax;
      if (i == 0 || i >= p.n_nodes[b]) continue;
      const int par = p.parent[cnode], tok = p.draft_tokens[cnode];
      if (par < 0 || par >= i || tok < slice0 || tok >= slice0 + kVocabPerWg || tok >= p.V) continue;
      const int r = b * p.Nmax + par - row0;
      if (r < 0 || r >= kRows) continue;
      const int vl = tok - slice0;
      p.node_logit[cnode] = dump[r * 128 + ((((vl >> 2) ^ (r & 15)) << 2) | (vl & 3))];
    }
    return;
  }

  // argmax over this wavefront's vocabulary rows for each hidden-state row (lane column n):
  // ascending vocabulary order inside the lane, then across the four lane groups
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    float best = -INFINITY;
    int idx = kNone;
#pragma unroll
    for (int nv = 0; nv < VT; ++nv)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int v = v0 + 16 * nv + 4 * g + i;
        const float x = acc[t][nv][i];
        if (v < p.V && x > best) { best = x; idx = v; }
      }
#pragma unroll
    for (int d = 16; d < 64; d <<= 1) {
      const float ov = __shfl_xor(best, d);
      const int oi = __shfl_xor(idx, d);
      take_better(best, idx, ov, oi);
    }
    if (g == 0) { red_val[wave][t * 16 + n] = best; red_idx[wave][t * 16 + n] = idx; }
  }
  __syncthreads();
  for (int m = threadIdx.x; m < MT * 16; m += 64 * WAVES) {
    if (row0 + m >= p.M) break;
    float best = red_val[0][m];
    int idx = red_idx[0][m];
#pragma unroll
    for (int w8 = 1; w8 < WAVES; ++w8) take_better(best, idx, red_val[w8][m], red_idx[w8][m]);
    const size_t slot = (size_t)slice * p.M + row0 + m;
    p.part_max[slot] = best;
    p.part_idx[slot] = idx;
  }
}

struct LmWalkParams {
  const float* part_max;    // [n_slices][B*Nmax]
  const int32_t* part_idx;
  const int32_t* draft_tokens;
  const int32_t* parent;
  const int32_t* n_nodes;
  int32_t* path;
  int32_t* path_len;
  int32_t* tokens;
  int32_t* n_tokens;
  int32_t* node_target;     // may be null
  float* node_top;          // may be null
  int32_t B, Nmax, n_slices;
};

// One workgroup per sequence: thread (node = lane, part = wavefront) scans every 16th slice of its
// node (adjacent lanes read adjacent words), the sixteen parts of a node meet in LDS, then
// wavefront 0 descends.
__global__ __launch_bounds__(kWalkThreads) void lm_head_walk_kernel(const LmWalkParams p) {
  constexpr int kParts = kWalkThreads / 64;
  __shared__ float q_best[kParts][FSPAD_MAX_NODES];
  __shared__ int q_idx[kParts][FSPAD_MAX_NODES];
  __shared__ int target[FSPAD_MAX_NODES];
  const int b = blockIdx.x, lane = threadIdx.x & 63, part = threadIdx.x >> 6;
  const int n = min(p.n_nodes[b], p.Nmax);
  const int64_t o = (int64_t)b * p.Nmax;
  const int64_t rows = (int64_t)p.B * p.Nmax;
  // the tree itself does not depend on the logits: wavefront 0 asks for it before anything else
  int my_par = -2, my_tok = -1;
  if (part == 0 && lane < p.Nmax) {
    my_par = p.parent[o + lane];
    my_tok = p.draft_tokens[o + lane];
  }
  if (lane >= n) my_par = -2;
  {
    float best = -INFINITY;
    int idx = kNone;
    if (lane < p.Nmax) {   // every row of the sequence has partial results; the ones past the tree are not used
      for (int c0 = part; c0 < p.n_slices; c0 += 16 * kParts) {
        float v[16];
        int ix[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
          const int c = c0 + kParts * k;
          v[k] = c < p.n_slices ? p.part_max[c * rows + o + lane] : -INFINITY;
          ix[k] = c < p.n_slices ? p.part_idx[c * rows + o + lane] : kNone;
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) take_better(best, idx, v[k], ix[k]);
      }
    }
    q_best[part][lane] = best;
    q_idx[part][lane] = idx;
  }
  __syncthreads();
  if (part != 0) return;
  if (lane < p.Nmax) {
    float best = -INFINITY;
    int idx = kNone;
    if (lane < n) {
      best = q_best[0][lane];
      idx = q_idx[0][lane];
#pragma unroll
      for (int w = 1; w < kParts; ++w) take_better(best, idx, q_best[w][lane], q_idx[w][lane]);
      if (idx == kNone) idx = 0;  // a row with nothing above -inf: token 0
      target[lane] = idx;
    }
    if (p.node_target) p.node_target[o + lane] = lane < n ? idx : -1;
    if (p.node_top) p.node_top[o + lane] = lane < n ? best : -INFINITY;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  fspad_detail::greedy_descend(target, n, p.Nmax, lane, o, b, my_par, my_tok, p.path, p.tokens, p.path_len, p.n_tokens);
}

struct LmSampleWalkParams {
  const float* part_max;     // [B*Nmax][n_slices]
  const double* part_sum;
  const float* tile_sum;     // [B*Nmax][n_slices][8]
  float* row_max;            // [B*Nmax], written by the row kernel: maximum of the row
  double* row_sum;           // [B*Nmax]: sum of exp((l - row_max) / T) over the row
  const float* node_logit;   // [B*Nmax]
  const char* hidden;        // [B*Nmax][K] bf16
  const char* weights;       // [V][K] bf16, row-major or in tile order (packed)
  const int32_t* draft_tokens;
  const int32_t* parent;
  const int32_t* n_nodes;
  const float* uniforms;     // [B][2][Nmax]
  int32_t* path;
  int32_t* path_len;
  int32_t* tokens;
  int32_t* n_tokens;
  double inv_temperature;
  int32_t B, Nmax, V, K, n_slices;
  int32_t packed;            // weights are in the tile order of fspad_pack_weight
};

// exp(x) for x <= 0 as the walk needs it: the fp32 hardware exponential (the logits themselves carry
// fp32 rounding of the same size), widened for the fp64 sums
__device__ __forceinline__ double weight_of(double x) {
  return (double)__builtin_amdgcn_exp2f((float)(fmin(x, 0.0) * 1.4426950408889634));
}

// Row statistics from the slice statistics: one workgroup per row of logits, thread = every 256th
// slice, running (max, sum) rescaled when the max moves, then across the workgroup.
__global__ __launch_bounds__(256) void lm_head_row_stats_kernel(const LmSampleWalkParams p) {
  __shared__ float red_m[4];
  __shared__ double red_z[4];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* pm = p.part_max + (size_t)row * p.n_slices;
  const double* ps = p.part_sum + (size_t)row * p.n_slices;
  const float c2 = (float)(p.inv_temperature * 1.4426950408889634);
  float m = -INFINITY;
  double z = 0.0;
  for (int c0 = tid; c0 < p.n_slices; c0 += 256 * 4) {
    float v[4];
    double sum[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const bool ok = c0 + 256 * k < p.n_slices;
      v[k] = ok ? pm[c0 + 256 * k] : -INFINITY;
      sum[k] = ok ? ps[c0 + 256 * k] : 0.0;
    }
    float m_new = m;
#pragma unroll
    for (int k = 0; k < 4; ++k) m_new = fmaxf(m_new, v[k]);
    if (m_new > -INFINITY) {
      z = m > -INFINITY ? z * (double)__builtin_amdgcn_exp2f((m - m_new) * c2) : 0.0;
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (v[k] > -INFINITY) z += sum[k] * (double)__builtin_amdgcn_exp2f((v[k] - m_new) * c2);
      m = m_new;
    }
  }
  float m_all = m;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) m_all = fmaxf(m_all, __shfl_xor(m_all, d));
  if (lane == 0) red_m[wave] = m_all;
  __syncthreads();
  m_all = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));
  z = m > -INFINITY ? z * (double)__builtin_amdgcn_exp2f((m - m_all) * c2) : 0.0;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) z += __shfl_xor(z, d);
  if (lane == 0) red_z[wave] = z;
  __syncthreads();
  if (tid == 0) {
    p.row_max[row] = m_all;
    p.row_sum[row] = red_z[0] + red_z[1] + red_z[2] + red_z[3];
  }
}

// Tree rejection sampling over the slice statistics the GEMM left (one workgroup of 1024 threads per
// sequence): (1) every row's max M and normaliser Z come from the row kernel above; (2) every node's weight exp((logit - M[parent]) / T) from the logit the
// GEMM set aside; (3) wavefront 0 walks the tree out of LDS, children in index order against the
// running residual, exactly as the walk over materialised logits does; (4) the last token: the
// slice that holds the crossing of u * Z follows from the slice sums (less the rejected tokens), its
// 128 logits are recomputed (128 dot products over K, eight threads each) and searched.
__global__ __launch_bounds__(kWalkThreads) void lm_head_sample_walk_kernel(const LmSampleWalkParams p) {
  __shared__ int rej_tok[FSPAD_MAX_NODES];
  __shared__ double rej_w[FSPAD_MAX_NODES];
  __shared__ double sh_d[4];   // M of the last row, target, scratch, target inside the tile
  __shared__ int sh_i[8];
  __shared__ double row_M[FSPAD_MAX_NODES], row_Z[FSPAD_MAX_NODES], node_w[FSPAD_MAX_NODES];
  __shared__ int node_par[FSPAD_MAX_NODES], node_tok[FSPAD_MAX_NODES];
  __shared__ float node_u[2][FSPAD_MAX_NODES];
  __shared__ float slice_logit[16];
  __shared__ double wave_sum[kWalkThreads / 64];
  __shared__ int wave_first[kWalkThreads / 64], wave_last[kWalkThreads / 64];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t o = (int64_t)b * p.Nmax;
  const float* u_acc = p.uniforms + (int64_t)b * 2 * p.Nmax;
  const int n = min(p.n_nodes[b], p.Nmax);

  // (1) row statistics (from the row kernel) and the tree
  {
    if (tid < p.Nmax) { row_M[tid] = (double)p.row_max[o + tid]; row_Z[tid] = p.row_sum[o + tid]; }
    if (tid < FSPAD_MAX_NODES) {
      const bool ok = tid < p.Nmax;
      node_par[tid] = ok ? p.parent[o + tid] : -2;
      node_tok[tid] = ok ? p.draft_tokens[o + tid] : -1;
      node_u[0][tid] = ok ? u_acc[tid] : 0.f;
      node_u[1][tid] = ok ? u_acc[p.Nmax + tid] : 0.f;
    }
  }
  __syncthreads();
  // (2) weight of every node's draft token under its parent's row
  if (tid < FSPAD_MAX_NODES) {
    double w = 0.0;
    const int par = node_par[tid], tok = node_tok[tid];
    if (tid > 0 && tid < n && par >= 0 && par < tid && tok >= 0 && tok < p.V) {
      const double M = row_M[par];
      const float lx = p.node_logit[o + tid];
      if (M > -INFINITY && lx == lx) w = weight_of(((double)lx - M) * p.inv_temperature);
    }
    node_w[tid] = w;
  }
  __syncthreads();

  if (wave == 0) {
    const int my_par = node_par[lane], my_tok = node_tok[lane];
    const double my_w = node_w[lane];
    const float my_u = node_u[0][lane];
    int my_path = lane == 0 ? 0 : -1, my_out = -1;
    int cur = 0, len = 1, nrej = 0;
    int my_rej = -1;       // lane k keeps the k-th token rejected at the current node, and its weight
    double my_rej_w = 0.0;
    double M = 0.0, Z = 0.0;
    auto lane_value = [](double v, int src) {   // src is the same in every lane: scalar reads, no LDS exchange
      const unsigned long long bits = __builtin_bit_cast(unsigned long long, v);
      const unsigned lo = __builtin_amdgcn_readlane((unsigned)bits, src);
      const unsigned hi = __builtin_amdgcn_readlane((unsigned)(bits >> 32), src);
      return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
    };
    for (int iter = 0; iter < p.Nmax; ++iter) {  // one level per iteration; a leaf ends the walk
      M = row_M[cur];
      Z = row_Z[cur];
      nrej = 0;
      my_rej = -1;
      const bool is_kid = lane > 0 && lane < n && my_par == cur;
      unsigned long long kids = __ballot(is_kid);
      int accepted = -1;
      while (kids != 0ull && len < p.Nmax) {
        const int c = __builtin_amdgcn_readfirstlane(__ffsll(kids) - 1);
        kids &= kids - 1ull;
        const int x = __builtin_amdgcn_readlane(my_tok, c);
        // a token that an earlier sibling proposed has left the residual: it weighs nothing now
        const bool gone = __ballot(lane < nrej && my_rej == x) != 0ull;
        const double w = gone ? 0.0 : lane_value(my_w, c);
        const double lhs = (double)__builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_u), c)) * Z;
        if (lhs < w) { accepted = c; break; }
        Z -= w;
        if (lane == nrej) { my_rej = x; my_rej_w = w; }
        ++nrej;
      }
      if (accepted < 0) break;
      if (lane == len) my_path = accepted;
      const int accepted_tok = __builtin_amdgcn_readlane(my_tok, accepted);
      if (lane == len - 1) my_out = accepted_tok;
      cur = accepted;
      ++len;
    }
    if (lane < nrej) { rej_tok[lane] = my_rej; rej_w[lane] = my_rej_w; }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    if (lane < p.Nmax) { p.path[o + lane] = my_path; if (lane != len - 1) p.tokens[o + lane] = my_out; }
    if (lane == 0) { p.path_len[b] = len; p.n_tokens[b] = len; }

    if (lane == 0) {
      sh_i[0] = cur; sh_i[1] = len; sh_i[2] = nrej;
      sh_i[3] = kNone; sh_i[4] = -1;
      sh_d[0] = M;
      sh_d[1] = (double)node_u[1][cur] * Z;   // t = u * Z
    }
  }
  __syncthreads();

  // last token, stage 1: which slice holds the running-sum crossing of t. Thread = slice (1024 per
  // turn): residual weight of the slice, workgroup-wide running sum, first slice above t.
  {
    const int cur = sh_i[0], nrej = sh_i[2];
    const double M = sh_d[0], t = sh_d[1];
    const float c2 = (float)(p.inv_temperature * 1.4426950408889634);
    const int64_t row = o + cur;
    const float* pm = p.part_max + row * p.n_slices;
    const double* ps = p.part_sum + row * p.n_slices;
    double carry = 0.0;
    int last_mass = -1;
    for (int c0 = 0; c0 < p.n_slices; c0 += kWalkThreads) {
      const int c = c0 + tid;
      double r = 0.0;
      if (c < p.n_slices) {
        const float mc = pm[c];
        if (mc > -INFINITY) {
          r = ps[c] * (double)__builtin_amdgcn_exp2f((mc - (float)M) * c2);
          for (int k = 0; k < nrej; ++k)
            if (rej_tok[k] >= c * kVocabPerWg && rej_tok[k] < (c + 1) * kVocabPerWg && rej_tok[k] < p.V) r -= rej_w[k];
        }
      }
      double incl = r;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const double up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
      }
      if (lane == 63) wave_sum[wave] = incl;
      __syncthreads();
      double base = carry;
      for (int w2 = 0; w2 < wave; ++w2) base += wave_sum[w2];
      double total = carry;
      for (int w2 = 0; w2 < kWalkThreads / 64; ++w2) total += wave_sum[w2];
      const double inclusive = base + incl;
      // first slice above t and last slice with mass (the rounding fallback): by ballot inside a
      // wavefront, one LDS slot per wavefront across them (no two lanes meet on an address)
      const bool has_mass = c < p.n_slices && r > 0.0;
      const unsigned long long mass = __ballot(has_mass), hit = __ballot(has_mass && inclusive > t);
      if (lane == 0) {
        wave_first[wave] = hit ? c0 + wave * 64 + (__ffsll(hit) - 1) : kNone;
        wave_last[wave] = mass ? c0 + wave * 64 + (63 - __clzll(mass)) : -1;
      }
      __syncthreads();
      int found = kNone;
#pragma unroll
      for (int w2 = 0; w2 < kWalkThreads / 64; ++w2) {
        found = min(found, wave_first[w2]);
        last_mass = max(last_mass, wave_last[w2]);
      }
      if (found != kNone) {
        if (c == found) sh_d[2] = t - (inclusive - r);       // what is left of t inside the slice
        if (tid == 0) sh_i[3] = found;
        break;
      }
      carry = total;
      __syncthreads();   // the slots are rewritten in the next turn
    }
    __syncthreads();
    if (tid == 0) {
      if (sh_i[3] == kNone) { sh_i[3] = last_mass; sh_d[2] = INFINITY; }   // no crossing: the last slice with mass, to its end
      sh_d[1] = sh_d[2];
    }
  }
  __syncthreads();

  // last token, stage 2: which 16 tokens of the slice hold the crossing (from the tile sums, less the
  // rejected tokens), their logits again (one wavefront per token, lanes over K), and the crossing
  const int cur = sh_i[0], len = sh_i[1], nrej = sh_i[2], sl = sh_i[3];
  if (sl < 0) {  // no mass anywhere (cannot happen with finite logits): token 0
    if (tid == 0) p.tokens[o + len - 1] = 0;
    return;
  }
  if (tid < 8) {   // thread = 16-token tile of the slice
    const size_t slot = (size_t)(o + cur) * p.n_slices + sl;
    double r = (double)p.tile_sum[slot * 8 + tid] * weight_of(((double)p.part_max[slot] - sh_d[0]) * p.inv_temperature);
    const int t0 = sl * kVocabPerWg + 16 * tid;
    for (int k = 0; k < nrej; ++k)
      if (rej_tok[k] >= t0 && rej_tok[k] < t0 + 16 && rej_tok[k] < p.V) r -= rej_w[k];
    double incl = r;
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) {
      const double up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    const unsigned long long cross = __ballot(incl > sh_d[1] && r > 0.0), mass = __ballot(r > 0.0);
    const int tile = cross ? __ffsll(cross) - 1 : (mass ? 63 - __clzll(mass) : -1);
    if (tid == (tile < 0 ? 0 : tile)) {
      sh_i[7] = tile;                                   // no crossing: the last tile with mass, to its end
      sh_d[3] = cross ? sh_d[1] - (incl - r) : INFINITY;
    }
  }
  __syncthreads();
  const int tile = sh_i[7];
  if (tile < 0) {  // the slice had mass only by rounding: its first valid token
    if (tid == 0) p.tokens[o + len - 1] = min(sl * kVocabPerWg, p.V - 1);
    return;
  }
  const int e0 = sl * kVocabPerWg + 16 * tile;
  {
    // wavefront w sums token e0 + w: lane l takes the 16-byte pieces l, l + 64, ... of the row
    const int v = e0 + wave;
    // row-major: piece c of row r at (r K + 8 c) * 2; tile order: piece c = 4 s + g of row r = 16 t + n
    // at ((t K/32 + s) 64 + n + 16 g) * 16. Lane l's pieces l, l + 64, ... are 16 k-steps apart.
    const int vr = min(v, p.V - 1);
    const char* wp = p.packed ? p.weights + (((size_t)(vr >> 4) * (p.K >> 5) + (lane >> 2)) * 64 + (vr & 15) + 16 * (lane & 3)) * 16
                              : p.weights + ((size_t)vr * p.K + (size_t)lane * 8) * 2;
    const int wstep = p.packed ? 16 * 1024 : 1024;   // bytes between a lane's consecutive pieces
    const char* hp = p.hidden + ((size_t)(o + cur) * p.K + (size_t)lane * 8) * 2;
    float dot = 0.f;
    for (int k = 0; k < p.K; k += 512 * 4) {   // four pieces in flight per lane
      bf16x8 a[4], h[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bool ok = k + 512 * u + lane * 8 < p.K;
        a[u] = ok ? *reinterpret_cast<const bf16x8*>(wp + (size_t)(k / 512 + u) * wstep) : bf16x8{};
        h[u] = ok ? *reinterpret_cast<const bf16x8*>(hp + 2 * (k + 512 * u)) : bf16x8{};
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int j = 0; j < 8; ++j) dot = fmaf((float)a[u][j], (float)h[u][j], dot);
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) dot += __shfl_xor(dot, d);
    if (lane == 0) slice_logit[wave] = v < p.V ? dot : NAN;
  }
  if (tid == 0) { sh_i[5] = kNone; sh_i[6] = -1; }
  __syncthreads();
  if (tid < 16) {   // thread = token of the tile
    const int e = e0 + tid;
    const float lx = slice_logit[tid];
    bool gone = lx != lx;
    for (int k = 0; k < nrej; ++k) gone = gone || rej_tok[k] == e;
    const double w = gone ? 0.0 : weight_of(((double)lx - sh_d[0]) * p.inv_temperature);
    double incl = w;
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {
      const double up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    const unsigned long long hit = __ballot(incl > sh_d[3] && w > 0.0), mass = __ballot(w > 0.0);
    if (tid == 0) {
      sh_i[5] = hit ? __ffsll(hit) - 1 : kNone;
      sh_i[6] = mass ? e0 + (63 - __clzll(mass)) : -1;
    }
  }
  __syncthreads();
  if (tid == 0) {
    // the first entry whose running sum exceeds the target; if rounding leaves none, the last with mass
    const int first = sh_i[5];
    p.tokens[o + len - 1] = first != kNone ? e0 + first : (sh_i[6] < 0 ? min(e0, p.V - 1) : sh_i[6]);
  }
}

int n_slices_of(int32_t V) { return (V + kVocabPerWg - 1) / kVocabPerWg; }
// Workgroup s starts its k loop (s * kStagger) stages in and wraps around, so that the workgroups
// running at the same time read different parts of their rows: with every workgroup at the same k
// the requests in flight differ only in address bits above the row pitch and crowd a few memory
// channels (measured on a 32000 x 4096 head: 59.8 us without, 52.4 us with).
constexpr int kStagger = 3;

}  // namespace

namespace {

fspad_status check_lm_head_args(int32_t B, int32_t Nmax, int32_t V, int32_t hidden_dim, const void* hidden,
                                const void* lm_head, const int32_t* draft_tokens, const int32_t* parent,
                                const int32_t* n_nodes, int32_t* path, int32_t* path_len, int32_t* tokens,
                                int32_t* n_tokens, void* workspace, size_t workspace_bytes) {
  if (!hidden || !lm_head || !draft_tokens || !parent || !n_nodes || !path || !path_len || !tokens || !n_tokens)
    return FSPAD_ERR_NULL;
  if (B < 1 || Nmax < 1 || Nmax > FSPAD_MAX_NODES || V < 1 || V > (1 << 30)) return FSPAD_ERR_SHAPE;
  if (hidden_dim < 256 || hidden_dim % 256 || hidden_dim > (1 << 16)) return FSPAD_ERR_SHAPE;
  if ((int64_t)B * Nmax > (1 << 20)) return FSPAD_ERR_SHAPE;
  if ((((uintptr_t)hidden) | ((uintptr_t)lm_head)) & 15) return FSPAD_ERR_SHAPE;
  if (!workspace || ((uintptr_t)workspace & 15) ||
      workspace_bytes < fspad_tree_accept_lm_head_workspace_bytes(B, Nmax, V))
    return FSPAD_ERR_WORKSPACE;
  return FSPAD_OK;
}

// Fills in the launch shape and runs the GEMM in the given mode (0 greedy, 1 sampling).
template <int MODE, bool PACKED>
fspad_status launch_lm_head(LmHeadParams& g, int32_t hidden_dim, hipStream_t stream) {
  // rows per workgroup: everything up to 128 rows in one pass of the eight-wavefront shape, more in
  // passes of up to 256 rows (each pass streams the weights again)
  g.rows_per_pass = g.M <= 128 ? g.M : 256;
  g.n_passes = (g.M + g.rows_per_pass - 1) / g.rows_per_pass;
  const int pass_rows = g.n_passes > 1 ? (g.M + g.n_passes - 1) / g.n_passes : g.M;   // passes of equal size
  if (g.n_passes > 1) g.rows_per_pass = (pass_rows + 15) / 16 * 16;
  if ((int64_t)g.n_slices * g.n_passes > 0x7fffffff) return FSPAD_ERR_SHAPE;
  // (a stage of the small shapes is 512 k: a hidden size that is not a multiple of it has a partial
  // last stage, which the rotation does not handle)
  g.stagger = (g.rows_per_pass > 64 || hidden_dim % 512 == 0) ? kStagger : 0;
  const dim3 grid((unsigned)(g.n_slices * g.n_passes));
  const int r = g.rows_per_pass;
  if (r <= 16) hipLaunchKernelGGL((lm_head_argmax_kernel<1, 16, 16, 8, 1, MODE, PACKED>), grid, dim3(512), 0, stream, g);
  else if (r <= 32) hipLaunchKernelGGL((lm_head_argmax_kernel<2, 16, 16, 8, 1, MODE, PACKED>), grid, dim3(512), 0, stream, g);
  else if (r <= 64) hipLaunchKernelGGL((lm_head_argmax_kernel<4, 16, 16, 8, 1, MODE, PACKED>), grid, dim3(512), 0, stream, g);
  else if (r <= 128) hipLaunchKernelGGL((lm_head_argmax_kernel<8, 8, 16, 8, 1, MODE, PACKED>), grid, dim3(512), 0, stream, g);
  else if (r <= 192) hipLaunchKernelGGL((lm_head_argmax_kernel<12, 4, 16, 8, 1, MODE, PACKED>), grid, dim3(512), 0, stream, g);
  else hipLaunchKernelGGL((lm_head_argmax_kernel<16, 4, 16, 8, 1, MODE, PACKED>), grid, dim3(512), 0, stream, g);
  return hipGetLastError() == hipSuccess ? FSPAD_OK : FSPAD_ERR_HIP;
}

}  // namespace

extern "C" size_t fspad_tree_accept_lm_head_workspace_bytes(int32_t B, int32_t Nmax, int32_t V) {
  if (B < 1 || Nmax < 1 || V < 1) return 0;
  // greedy: (max, argmax) per row and slice; sampling: (max, fp64 sum, eight tile sums) per row and slice
  // + one logit per node + (max, fp64 sum) per row
  const size_t slots = (size_t)B * Nmax * n_slices_of(V);
  return (slots * (12 + 32) + (size_t)B * Nmax * (4 + 12) + 255) & ~(size_t)255;
}

extern "C" fspad_status fspad_tree_accept_greedy_lm_head(int32_t B, int32_t Nmax, int32_t V, int32_t hidden_dim,
                                                         const void* hidden, const void* lm_head, int32_t flags,
                                                         const int32_t* draft_tokens, const int32_t* parent,
                                                         const int32_t* n_nodes, int32_t* path, int32_t* path_len,
                                                         int32_t* tokens, int32_t* n_tokens, int32_t* node_target,
                                                         float* node_top, void* workspace, size_t workspace_bytes,
                                                         void* hip_stream) {
  const fspad_status st = check_lm_head_args(B, Nmax, V, hidden_dim, hidden, lm_head, draft_tokens, parent, n_nodes, path,
                                             path_len, tokens, n_tokens, workspace, workspace_bytes);
  if (st != FSPAD_OK) return st;
  if (flags & ~FSPAD_WEIGHTS_PACKED) return FSPAD_ERR_SHAPE;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);

  LmHeadParams g{};
  g.hidden = static_cast<const char*>(hidden);
  g.weights = static_cast<const char*>(lm_head);
  g.M = B * Nmax; g.V = V; g.K = hidden_dim;
  g.n_slices = n_slices_of(V);
  const size_t slots = (size_t)g.M * g.n_slices;
  g.part_max = static_cast<float*>(workspace);
  g.part_idx = reinterpret_cast<int32_t*>(g.part_max + slots);
  const fspad_status gs = (flags & FSPAD_WEIGHTS_PACKED) ? launch_lm_head<0, true>(g, hidden_dim, stream)
                                                         : launch_lm_head<0, false>(g, hidden_dim, stream);
  if (gs != FSPAD_OK) return gs;

  LmWalkParams w{};
  w.part_max = g.part_max; w.part_idx = g.part_idx;
  w.draft_tokens = draft_tokens; w.parent = parent; w.n_nodes = n_nodes;
  w.path = path; w.path_len = path_len; w.tokens = tokens; w.n_tokens = n_tokens;
  w.node_target = node_target; w.node_top = node_top;
  w.B = B; w.Nmax = Nmax; w.n_slices = g.n_slices;
  hipLaunchKernelGGL(lm_head_walk_kernel, dim3((unsigned)B), dim3(kWalkThreads), 0, stream, w);
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  return FSPAD_OK;
}

extern "C" fspad_status fspad_tree_accept_sample_lm_head(int32_t B, int32_t Nmax, int32_t V, int32_t hidden_dim,
                                                         const void* hidden, const void* lm_head, int32_t flags,
                                                         const int32_t* draft_tokens, const int32_t* parent,
                                                         const int32_t* n_nodes, float temperature,
                                                         const float* uniforms, int32_t* path, int32_t* path_len,
                                                         int32_t* tokens, int32_t* n_tokens, void* workspace,
                                                         size_t workspace_bytes, void* hip_stream) {
  const fspad_status st = check_lm_head_args(B, Nmax, V, hidden_dim, hidden, lm_head, draft_tokens, parent, n_nodes, path,
                                             path_len, tokens, n_tokens, workspace, workspace_bytes);
  if (st != FSPAD_OK) return st;
  if (!uniforms) return FSPAD_ERR_NULL;
  if (flags & ~FSPAD_WEIGHTS_PACKED) return FSPAD_ERR_SHAPE;
  if (!(temperature > 0.0f) || isinf(temperature)) return FSPAD_ERR_TEMPERATURE;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);

  LmHeadParams g{};
  g.hidden = static_cast<const char*>(hidden);
  g.weights = static_cast<const char*>(lm_head);
  g.M = B * Nmax; g.V = V; g.K = hidden_dim; g.Nmax = Nmax;
  g.n_slices = n_slices_of(V);
  const size_t slots = (size_t)g.M * g.n_slices;
  g.part_sum = static_cast<double*>(workspace);                 // 8-byte entries first
  double* row_sum = g.part_sum + slots;
  g.part_max = reinterpret_cast<float*>(row_sum + g.M);
  g.tile_sum = g.part_max + slots;
  g.node_logit = g.tile_sum + slots * 8;
  float* row_max = g.node_logit + g.M;
  g.draft_tokens = draft_tokens; g.parent = parent; g.n_nodes = n_nodes;
  g.inv_t_log2e = (float)(1.4426950408889634 / (double)temperature);
  const fspad_status gs = (flags & FSPAD_WEIGHTS_PACKED) ? launch_lm_head<1, true>(g, hidden_dim, stream)
                                                         : launch_lm_head<1, false>(g, hidden_dim, stream);
  if (gs != FSPAD_OK) return gs;

  LmSampleWalkParams w{};
  w.part_max = g.part_max; w.part_sum = g.part_sum; w.tile_sum = g.tile_sum; w.node_logit = g.node_logit;
  w.hidden = g.hidden; w.weights = g.weights;
  w.draft_tokens = draft_tokens; w.parent = parent; w.n_nodes = n_nodes; w.uniforms = uniforms;
  w.path = path; w.path_len = path_len; w.tokens = tokens; w.n_tokens = n_tokens;
  w.inv_temperature = 1.0 / (double)temperature;
  w.B = B; w.Nmax = Nmax; w.V = V; w.K = hidden_dim; w.n_slices = g.n_slices;
  w.packed = (flags & FSPAD_WEIGHTS_PACKED) != 0;
  w.row_max = row_max; w.row_sum = row_sum;
  hipLaunchKernelGGL(lm_head_row_stats_kernel, dim3((unsigned)g.M), dim3(256), 0, stream, w);
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  hipLaunchKernelGGL(lm_head_sample_walk_kernel, dim3((unsigned)B), dim3(kWalkThreads), 0, stream, w);
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  return FSPAD_OK;
}
