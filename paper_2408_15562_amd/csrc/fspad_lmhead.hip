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
// Workgroup = 128 vocabulary rows x up to 64 hidden-state rows x all of K; four wavefronts of 32
// vocabulary rows each. With `v_mfma_f32_16x16x32_bf16` and A = 16 weight rows, B = 16 hidden
// rows, both operands are "8 consecutive k per lane", i.e. plain 16-byte loads of row-major data:
// the weights go from HBM straight into registers (two chunks of 256 k in flight per wavefront),
// the hidden states are copied global -> LDS without registers (XOR-swizzled by 16-byte chunk so
// that a 16-row operand read touches 16 different bank groups), double-buffered, one barrier per
// 256 k. D[vocab][row] puts one hidden-state row per lane column, so the argmax over the
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

constexpr int kWaves = 4;
constexpr int kVocabTiles = 2;                              // 16-row weight tiles per wavefront
constexpr int kVocabPerWave = 16 * kVocabTiles;             // 32
constexpr int kVocabPerWg = kWaves * kVocabPerWave;         // 128
constexpr int kChunkK = 256;                                // k per LDS stage and register buffer
constexpr int kSteps = kChunkK / 32;                        // matrix-instruction k-steps per chunk
constexpr int kRowsPerPass = 64;                            // hidden-state rows one workgroup holds
constexpr int kNone = 0x7fffffff;
constexpr int kWalkThreads = 1024;

struct LmHeadParams {
  const char* hidden;   // [M][K] bf16
  const char* weights;  // [V][K] bf16
  float* part_max;      // [n_slices][M]
  int32_t* part_idx;    // [n_slices][M]
  int32_t M, V, K, n_slices, n_passes;
};

// (value, index) with "larger value, then lower index" order
__device__ __forceinline__ void take_better(float& v, int& i, float ov, int oi) {
  if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
}

// MT: 16-row tiles of hidden states per workgroup (rows of a pass <= 16 * MT)
template <int MT>
__global__ __launch_bounds__(64 * kWaves, 2) void lm_head_argmax_kernel(const LmHeadParams p) {
  constexpr int kStageBytes = MT * 16 * kChunkK * 2;          // MT * 8 KB
  constexpr int kCopiesPerWave = kStageBytes / 1024 / kWaves;  // 1 KB per copy instruction: 2 * MT
  __shared__ __attribute__((aligned(16))) char xs[2 * kStageBytes];
  __shared__ float red_val[kWaves][MT * 16];
  __shared__ int red_idx[kWaves][MT * 16];

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, g = lane >> 4;
  const int slice = blockIdx.x / p.n_passes, pass = blockIdx.x - slice * p.n_passes;
  const int row0 = pass * kRowsPerPass;
  const int v0 = slice * kVocabPerWg + wave * kVocabPerWave;
  const size_t row_bytes = (size_t)p.K * 2;

  // weight rows of this lane (rows past the vocabulary are clamped; their columns are never taken)
  const char* wrow[kVocabTiles];
#pragma unroll
  for (int nv = 0; nv < kVocabTiles; ++nv)
    wrow[nv] = p.weights + (size_t)min(v0 + nv * 16 + n, p.V - 1) * row_bytes + g * 16;

  // hidden-state copies of this wavefront: one instruction moves two rows of 512 bytes; LDS slot s
  // of row r receives the row's 16-byte chunk s ^ (r & 15)
  const char* xsrc[kCopiesPerWave];
#pragma unroll
  for (int i = 0; i < kCopiesPerWave; ++i) {
    const int r = 2 * (wave * kCopiesPerWave + i) + (lane >> 5), s = lane & 31;
    xsrc[i] = p.hidden + (size_t)min(row0 + r, p.M - 1) * row_bytes + ((s ^ (r & 15)) << 4);
  }
  // operand reads: lane (n, g) of tile t, k-step kk reads chunk 4*kk + g of row 16*t + n, kept at
  // slot (4*kk + g) ^ n = (4*kk) ^ (g ^ n)
  const unsigned xread = (unsigned)n * (kChunkK * 2), xswz = (unsigned)(g ^ n) << 4;

  auto copy_x = [&](int ck, int stage) {
#pragma unroll
    for (int i = 0; i < kCopiesPerWave; ++i)
      __builtin_amdgcn_global_load_lds((GlobalPtr)(xsrc[i] + (size_t)ck * (kChunkK * 2)),
                                       (LdsPtr)(xs + stage * kStageBytes + (wave * kCopiesPerWave + i) * 1024), 16, 0, 0);
  };
  auto load_w = [&](bf16x8 (&wr)[kVocabTiles][kSteps], int ck) {
#pragma unroll
    for (int nv = 0; nv < kVocabTiles; ++nv)
#pragma unroll
      for (int kk = 0; kk < kSteps; ++kk)
        wr[nv][kk] = *reinterpret_cast<const bf16x8*>(wrow[nv] + (size_t)ck * (kChunkK * 2) + kk * 64);
  };

  f32x4 acc[MT][kVocabTiles];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int nv = 0; nv < kVocabTiles; ++nv) acc[t][nv] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](const bf16x8 (&wr)[kVocabTiles][kSteps], int stage) {
    const char* base = xs + stage * kStageBytes + xread;
#pragma unroll
    for (int kk = 0; kk < kSteps; ++kk) {
      bf16x8 xf[MT];
#pragma unroll
      for (int t = 0; t < MT; ++t)
        xf[t] = *reinterpret_cast<const bf16x8*>(base + t * (16 * kChunkK * 2) + (((unsigned)kk << 6) ^ xswz));
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int nv = 0; nv < kVocabTiles; ++nv)
          acc[t][nv] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wr[nv][kk], xf[t], acc[t][nv], 0, 0, 0);
    }
  };

  // One turn: everything requested so far has landed (this chunk's hidden states and weights); the
  // barrier publishes every wavefront's share of the stage and retires the other stage, which the
  // next chunk's copy then overwrites while this chunk is being multiplied.
  const int n_chunks = p.K / kChunkK;
  bf16x8 w0[kVocabTiles][kSteps], w1[kVocabTiles][kSteps];
  copy_x(0, 0);
  load_w(w0, 0);
  for (int ck = 0; ck < n_chunks; ck += 2) {
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
    __syncthreads();
    if (ck + 1 < n_chunks) { copy_x(ck + 1, 1); load_w(w1, ck + 1); }
    compute(w0, 0);
    if (ck + 1 >= n_chunks) break;
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
    __syncthreads();
    if (ck + 2 < n_chunks) { copy_x(ck + 2, 0); load_w(w0, ck + 2); }
    compute(w1, 1);
  }

  // argmax over this wavefront's 32 vocabulary rows for each of its hidden-state rows (lane column n):
  // ascending vocabulary order inside the lane, then across the four lane groups
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    float best = -INFINITY;
    int idx = kNone;
#pragma unroll
    for (int nv = 0; nv < kVocabTiles; ++nv)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int v = v0 + nv * 16 + 4 * g + i;
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
  const int m = threadIdx.x;
  if (m < MT * 16 && row0 + m < p.M) {
    float best = red_val[0][m];
    int idx = red_idx[0][m];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) take_better(best, idx, red_val[w][m], red_idx[w][m]);
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
  {
    float best = -INFINITY;
    int idx = kNone;
    if (lane < n) {
      for (int c0 = part; c0 < p.n_slices; c0 += 8 * kParts) {
        float v[8];
        int ix[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int c = c0 + kParts * k;
          v[k] = c < p.n_slices ? p.part_max[c * rows + o + lane] : -INFINITY;
          ix[k] = c < p.n_slices ? p.part_idx[c * rows + o + lane] : kNone;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) take_better(best, idx, v[k], ix[k]);
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
  fspad_detail::greedy_descend(target, n, p.Nmax, lane, o, b, p.parent, p.draft_tokens, p.path, p.tokens, p.path_len,
                               p.n_tokens);
}

int n_slices_of(int32_t V) { return (V + kVocabPerWg - 1) / kVocabPerWg; }

}  // namespace

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
  if (hidden_dim < kChunkK || hidden_dim % kChunkK || hidden_dim > (1 << 16)) return FSPAD_ERR_SHAPE;
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
  g.n_passes = (g.M + kRowsPerPass - 1) / kRowsPerPass;
  const size_t slots = (size_t)g.M * g.n_slices;
  g.part_max = static_cast<float*>(workspace);
  g.part_idx = reinterpret_cast<int32_t*>(g.part_max + slots);
  if ((int64_t)g.n_slices * g.n_passes > 0x7fffffff) return FSPAD_ERR_SHAPE;
  const dim3 grid((unsigned)(g.n_slices * g.n_passes)), block(64 * kWaves);
  const int rows_per_pass = g.n_passes > 1 ? kRowsPerPass : g.M;
  if (rows_per_pass <= 16) hipLaunchKernelGGL(lm_head_argmax_kernel<1>, grid, block, 0, stream, g);
  else if (rows_per_pass <= 32) hipLaunchKernelGGL(lm_head_argmax_kernel<2>, grid, block, 0, stream, g);
  else hipLaunchKernelGGL(lm_head_argmax_kernel<4>, grid, block, 0, stream, g);
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
