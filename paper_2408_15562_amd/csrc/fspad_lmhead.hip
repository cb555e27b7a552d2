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

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef const __attribute__((address_space(1))) void* GlobalPtr;
typedef __attribute__((address_space(3))) void* LdsPtr;

constexpr int kVocabPerWg = 128;                            // vocabulary rows per workgroup, in every shape below
constexpr int kNone = 0x7fffffff;
constexpr int kWalkThreads = 1024;

struct LmHeadParams {
  const char* hidden;   // [M][K] bf16
  const char* weights;  // [V][K] bf16
  float* part_max;      // [n_slices][M]
  int32_t* part_idx;    // [n_slices][M]
  int32_t M, V, K, n_slices, n_passes, rows_per_pass;
  int32_t stagger;      // stages by which consecutive workgroups are offset along k (0: all start at k = 0)
};

// (value, index) with "larger value, then lower index" order
__device__ __forceinline__ void take_better(float& v, int& i, float ov, int oi) {
  if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
}

// MT: 16-row tiles of hidden states per workgroup (rows of a pass <= 16 * MT).
// SPS: k-steps per LDS stage of hidden states (stage = 16*MT rows x 32*SPS k).
// kRing: weight operands (k-steps of 32) per vocabulary tile that a wavefront keeps requested.
// WAVES x VT = 8: wavefronts per workgroup x 16-row vocabulary tiles per wavefront. Eight
// wavefronts of one tile (two per SIMD) for up to 128 rows; for more, four wavefronts of two tiles
// (one per SIMD, the whole register file), which halves the LDS reads per product: with 256 rows an
// operand read of all of them for one weight tile would cost as much as its 16 products.
template <int MT, int SPS, int kRing, int WAVES, int VT>
__global__ __launch_bounds__(64 * WAVES, (WAVES == 8 ? 2 : 1)) void lm_head_argmax_kernel(const LmHeadParams p) {
  static_assert(WAVES * VT * 16 == kVocabPerWg, "workgroup shape");
  constexpr int kStageK = 32 * SPS;
  constexpr int kRowBytes = kStageK * 2;                        // 256, 512 or 1024
  constexpr int kStageBytes = MT * 16 * kRowBytes;
  constexpr int kChunksPerRow = kRowBytes / 16;                 // 16, 32 or 64
  constexpr int kRowsPerCopy = 1024 / kRowBytes;                // one copy instruction moves 1 KB
  constexpr int kCopiesPerWave = kStageBytes / 1024 / WAVES;
  static_assert(kCopiesPerWave >= 1 && kRing % SPS == 0 && kRing % 4 == 0, "stage shape");
  __shared__ __attribute__((aligned(16))) char xs[2 * kStageBytes];
  __shared__ float red_val[WAVES][MT * 16];
  __shared__ int red_idx[WAVES][MT * 16];

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, g = lane >> 4;
  const int slice = blockIdx.x / p.n_passes, pass = blockIdx.x - slice * p.n_passes;
  const int row0 = pass * p.rows_per_pass;
  const int v0 = slice * kVocabPerWg + wave * (16 * VT);
  const size_t row_bytes = (size_t)p.K * 2;
  const int n_steps = p.K >> 5;
  // workgroup `slice` walks k from stage `first_stage` on and wraps around
  const int first_step = p.stagger ? (int)(((unsigned)slice * (unsigned)p.stagger) % (unsigned)(n_steps / SPS)) * SPS : 0;

  // weight rows of this lane (rows past the vocabulary are clamped; their columns are never taken)
  const char* wrow[VT];
#pragma unroll
  for (int nv = 0; nv < VT; ++nv) wrow[nv] = p.weights + (size_t)min(v0 + 16 * nv + n, p.V - 1) * row_bytes + g * 16;

  // hidden-state copies of this wavefront: LDS slot s of row r receives the row's 16-byte chunk
  // s ^ (r & 15) of the stage's k range (chunks past the end of the row are clamped: never used)
  const char* xsrc[kCopiesPerWave];
  int xcol[kCopiesPerWave];
#pragma unroll
  for (int i = 0; i < kCopiesPerWave; ++i) {
    const int r = kRowsPerCopy * (wave * kCopiesPerWave + i) + lane / kChunksPerRow, s = lane % kChunksPerRow;
    xsrc[i] = p.hidden + (size_t)min(row0 + r, p.M - 1) * row_bytes;
    xcol[i] = s ^ (r & 15);
  }
  const int last_chunk = (p.K >> 3) - 1;
  // operand reads: lane (n, g) of tile t, k-step kk of the stage reads chunk 4*kk + g of row 16*t + n,
  // kept at slot (4*kk + g) ^ n = (4*kk) ^ (g ^ n)
  const unsigned xread = (unsigned)n * kRowBytes, xswz = (unsigned)(g ^ n) << 4;

  bf16x8 xr[kCopiesPerWave];
  auto fetch_x = [&](int stage_index) {
#pragma unroll
    for (int i = 0; i < kCopiesPerWave; ++i) {
      int stage = stage_index + first_step / SPS;
      stage -= stage * SPS >= n_steps ? n_steps / SPS : 0;
      const int chunk = min(stage * kChunksPerRow + xcol[i], last_chunk);
      xr[i] = *reinterpret_cast<const bf16x8*>(xsrc[i] + ((size_t)chunk << 4));
    }
  };
  auto store_x = [&](int stage_index) {
    char* dst = xs + (stage_index & 1) * kStageBytes + wave * kCopiesPerWave * 1024 + lane * 16;
#pragma unroll
    for (int i = 0; i < kCopiesPerWave; ++i) *reinterpret_cast<bf16x8*>(dst + i * 1024) = xr[i];
  };
  // workgroup barrier that orders LDS traffic only: the weight requests in flight stay in flight
  auto lds_barrier = [] {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  };
  // k-step ks of the weights: lane (n, g) holds k = 32*ks + 8*g .. +7 of its row (steps past the end
  // re-read the last one, so that every turn of the loop issues the same number of requests)
  auto load_w = [&](int nv, int ks) {
    int step = min(ks, n_steps - 1) + first_step;
    step -= step >= n_steps ? n_steps : 0;
    return *reinterpret_cast<const bf16x8*>(wrow[nv] + (size_t)step * 64);
  };

  f32x4 acc[MT][VT];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int nv = 0; nv < VT; ++nv) acc[t][nv] = f32x4{0.f, 0.f, 0.f, 0.f};

  // The weights are requested kRing k-steps ahead, every operand register being requested again as
  // soon as its products are issued. The hidden states of stage j+1 are requested into registers at
  // the top of stage j and written to the other LDS stage at its end (by then they have long
  // arrived, and the weight requests issued after them stay in flight); the barrier at the top of a
  // stage publishes every wavefront's share of it and retires the other one.
  bf16x8 w[VT][kRing];
  fetch_x(0);
#pragma unroll
  for (int i = 0; i < kRing; ++i)
#pragma unroll
    for (int nv = 0; nv < VT; ++nv) w[nv][i] = load_w(nv, i);
  store_x(0);
  const int n_stages = (n_steps + SPS - 1) / SPS;
  for (int ks0 = 0; ks0 < n_steps; ks0 += kRing) {
#pragma unroll
    for (int kk = 0; kk < kRing; ++kk) {
      const int ks = ks0 + kk;
      if (kk % 4 == 0 && ks >= n_steps) break;   // K is a multiple of 256 and the ring of 4: the end falls on a multiple of 4 steps
      if (kk % SPS == 0) {
        lds_barrier();
        if (ks / SPS + 1 < n_stages) fetch_x(ks / SPS + 1);
      }
      const char* base = xs + ((ks / SPS) & 1) * kStageBytes + xread + ((((unsigned)kk % SPS) << 6) ^ xswz);
      bf16x8 xf[MT];
#pragma unroll
      for (int t = 0; t < MT; ++t) xf[t] = *reinterpret_cast<const bf16x8*>(base + t * (16 * kRowBytes));
#pragma unroll
      for (int nv = 0; nv < VT; ++nv)
#pragma unroll
        for (int t = 0; t < MT; ++t)
          acc[t][nv] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[nv][kk], xf[t], acc[t][nv], 0, 0, 0);
#pragma unroll
      for (int nv = 0; nv < VT; ++nv) w[nv][kk] = load_w(nv, ks + kRing);
      if (kk % SPS == SPS - 1 && ks / SPS + 1 < n_stages) store_x(ks / SPS + 1);
    }
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

int n_slices_of(int32_t V) { return (V + kVocabPerWg - 1) / kVocabPerWg; }
// Workgroup s starts its k loop (s * g_stagger) stages in and wraps around, so that the workgroups
// running at the same time read different parts of their rows: with every workgroup at the same k
// the requests in flight differ only in address bits above the row pitch and crowd a few memory
// channels (measured on a 32000 x 4096 head: 59.8 us without, 52.4 us with).
int g_stagger = 3;

}  // namespace

// Experiment knob (not part of the declared interface): the k rotation between workgroups (0: none).
extern "C" void fspad_debug_set_lm_head_stagger(int32_t stages) { g_stagger = stages < 0 ? 0 : stages; }

extern "C" size_t fspad_tree_accept_lm_head_workspace_bytes(int32_t B, int32_t Nmax, int32_t V) {
  if (B < 1 || Nmax < 1 || V < 1) return 0;
  const size_t slots = (size_t)B * Nmax * n_slices_of(V);
  return (slots * 8 + 255) & ~(size_t)255;
}

extern "C" fspad_status fspad_tree_accept_greedy_lm_head(int32_t B, int32_t Nmax, int32_t V, int32_t hidden_dim,
                                                         const void* hidden, const void* lm_head,
                                                         const int32_t* draft_tokens, const int32_t* parent,
                                                         const int32_t* n_nodes, int32_t* path, int32_t* path_len,
                                                         int32_t* tokens, int32_t* n_tokens, int32_t* node_target,
                                                         float* node_top, void* workspace, size_t workspace_bytes,
                                                         void* hip_stream) {
  if (!hidden || !lm_head || !draft_tokens || !parent || !n_nodes || !path || !path_len || !tokens || !n_tokens)
    return FSPAD_ERR_NULL;
  if (B < 1 || Nmax < 1 || Nmax > FSPAD_MAX_NODES || V < 1 || V > (1 << 30)) return FSPAD_ERR_SHAPE;
  if (hidden_dim < 256 || hidden_dim % 256 || hidden_dim > (1 << 16)) return FSPAD_ERR_SHAPE;
  if ((int64_t)B * Nmax > (1 << 20)) return FSPAD_ERR_SHAPE;
  if ((((uintptr_t)hidden) | ((uintptr_t)lm_head)) & 15) return FSPAD_ERR_SHAPE;
  if (!workspace || ((uintptr_t)workspace & 15) ||
      workspace_bytes < fspad_tree_accept_lm_head_workspace_bytes(B, Nmax, V))
    return FSPAD_ERR_WORKSPACE;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);

  LmHeadParams g{};
  g.hidden = static_cast<const char*>(hidden);
  g.weights = static_cast<const char*>(lm_head);
  g.M = B * Nmax; g.V = V; g.K = hidden_dim;
  g.n_slices = n_slices_of(V);
  // rows per workgroup: everything up to 128 rows in one pass of the eight-wavefront shape, more in
  // passes of up to 256 rows of the four-wavefront shape (each pass streams the weights again)
  g.rows_per_pass = g.M <= 128 ? g.M : 256;
  g.n_passes = (g.M + g.rows_per_pass - 1) / g.rows_per_pass;
  const int pass_rows = g.n_passes > 1 ? (g.M + g.n_passes - 1) / g.n_passes : g.M;   // passes of equal size
  if (g.n_passes > 1) g.rows_per_pass = (pass_rows + 15) / 16 * 16;
  const size_t slots = (size_t)g.M * g.n_slices;
  g.part_max = static_cast<float*>(workspace);
  g.part_idx = reinterpret_cast<int32_t*>(g.part_max + slots);
  if ((int64_t)g.n_slices * g.n_passes > 0x7fffffff) return FSPAD_ERR_SHAPE;
  // (a stage of the small shapes is 512 k: a hidden size that is not a multiple of it has a partial
  // last stage, which the rotation does not handle)
  g.stagger = (g.rows_per_pass > 64 || hidden_dim % 512 == 0) ? g_stagger : 0;
  const dim3 grid((unsigned)(g.n_slices * g.n_passes));
  const int r = g.rows_per_pass;
  if (r <= 16) hipLaunchKernelGGL((lm_head_argmax_kernel<1, 16, 16, 8, 1>), grid, dim3(512), 0, stream, g);
  else if (r <= 32) hipLaunchKernelGGL((lm_head_argmax_kernel<2, 16, 16, 8, 1>), grid, dim3(512), 0, stream, g);
  else if (r <= 64) hipLaunchKernelGGL((lm_head_argmax_kernel<4, 16, 16, 8, 1>), grid, dim3(512), 0, stream, g);
  else if (r <= 128) hipLaunchKernelGGL((lm_head_argmax_kernel<8, 8, 16, 8, 1>), grid, dim3(512), 0, stream, g);
  else if (r <= 192) hipLaunchKernelGGL((lm_head_argmax_kernel<12, 4, 16, 4, 2>), grid, dim3(256), 0, stream, g);
  else hipLaunchKernelGGL((lm_head_argmax_kernel<16, 4, 8, 4, 2>), grid, dim3(256), 0, stream, g);
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;

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
