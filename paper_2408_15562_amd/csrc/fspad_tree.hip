// Dynamic draft tree from its candidates (arXiv 2408.15562, Preliminaries, last paragraph:
// per-step top-k, joint probabilities from the dependencies, one more top-k over all tokens;
// then the tokens are organised into a tree and the attention mask derived from it).
// One workgroup per sequence, everything in LDS: at most 1024 candidates, a few microseconds.
//   1. joint scores, level by level (a candidate is scored once its parent is)
//   2. rank of every candidate = number of candidates that beat it (score, then index)
//   3. kept = rank < n_keep-1, closed under "parent kept" (level by level again)
//   4. node index = number of kept candidates before it; parents, tokens, ancestor words
#include "fspad.h"

#include <hip/hip_runtime.h>
#include <math.h>

namespace {

constexpr int kThreads = 256;
constexpr int kPerThread = FSPAD_MAX_CANDIDATES / kThreads;

struct BuildParams {
  const int32_t* cand_parent;
  const int32_t* cand_token;
  const float* cand_logp;
  const int32_t* n_cand;
  int32_t* parent;
  int32_t* tokens;
  int32_t* n_nodes;
  uint64_t* anc_mask;
  int32_t* node_cand;
  int32_t M, Nmax, n_keep;
};

__global__ __launch_bounds__(kThreads) void tree_build_kernel(const BuildParams p) {
  __shared__ __attribute__((aligned(16))) float joint[FSPAD_MAX_CANDIDATES];
  __shared__ int16_t par[FSPAD_MAX_CANDIDATES];     // -1 root, -2 unreachable
  __shared__ int16_t node_of[FSPAD_MAX_CANDIDATES];  // node index of a kept candidate, else -1
  __shared__ uint8_t state[FSPAD_MAX_CANDIDATES];    // pass 1: scored; pass 2: 1 kept, 0 dropped, 2 undecided
  __shared__ int16_t node_par[FSPAD_MAX_NODES];
  __shared__ int wave_count[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int m = p.n_cand[b];
  m = m < 1 ? 1 : (m > p.M ? p.M : m);
  const int32_t* cp = p.cand_parent + (size_t)b * p.M;
  const float* lp = p.cand_logp + (size_t)b * p.M;

  // candidate c lives in thread c / kPerThread (contiguous runs, so that counts of kept
  // candidates before c are a thread-local count plus an exclusive scan over threads)
  float my_lp[kPerThread];
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    const int c = tid * kPerThread + k;
    my_lp[k] = 0.f;
    if (c < m) {
      const int pc = cp[c];
      par[c] = c == 0 ? (int16_t)-1 : ((pc >= 0 && pc < c) ? (int16_t)pc : (int16_t)-2);
      const float v = lp[c];
      my_lp[k] = (v != v) ? -INFINITY : v;
      state[c] = c == 0 ? 1 : 0;
      if (c == 0) joint[0] = 0.f;
    } else {
      joint[c] = -INFINITY;   // padding: never beats a candidate (its index is larger as well)
    }
  }
  __syncthreads();

  // 1. joint scores: a candidate is scored in the round after its parent was
  for (;;) {
    bool progressed = false;
    uint8_t newly[kPerThread];
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
      const int c = tid * kPerThread + k;
      newly[k] = 0;
      if (c > 0 && c < m && !state[c] && par[c] >= 0 && state[par[c]]) {
        joint[c] = joint[par[c]] + my_lp[k];
        newly[k] = 1;
        progressed = true;
      }
    }
    __syncthreads();   // all reads of state[] of this round are done
#pragma unroll
    for (int k = 0; k < kPerThread; ++k)
      if (newly[k]) state[tid * kPerThread + k] = 1;
    if (!__syncthreads_or(progressed)) break;
  }
  // candidates that were never reached (bad parent index somewhere above them) cannot be kept
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    const int c = tid * kPerThread + k;
    if (c < m && !state[c]) { joint[c] = -INFINITY; par[c] = -2; }
  }
  __syncthreads();

  // 2. rank among the non-root candidates: higher joint first, then lower index
  int rank[kPerThread];
  float mine[kPerThread];
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    const int c = tid * kPerThread + k;
    rank[k] = 0;
    mine[k] = c < m ? joint[c] : 0.f;
  }
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  const f32x4* joint4 = reinterpret_cast<const f32x4*>(joint);
#pragma unroll 4
  for (int j4 = 0; j4 < (m + 3) / 4; ++j4) {
    const f32x4 o = joint4[j4];   // same address in all lanes: one broadcast read of four scores
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int k = 0; k < kPerThread; ++k) {
        const int c = tid * kPerThread + k;
        // bitwise on purpose: with || and && every comparison becomes a branch
        rank[k] += (int)(o[e] > mine[k]) | ((int)(o[e] == mine[k]) & (int)(4 * j4 + e < c));
      }
  }
  // the root (score 0, index 0) is not a competitor: take its count out again
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    const int c = tid * kPerThread + k;
    rank[k] -= (int)(0.f > mine[k]) | ((int)(0.f == mine[k]) & (int)(0 < c));
  }
  __syncthreads();   // state[] is reused below
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    const int c = tid * kPerThread + k;
    if (c < m) state[c] = c == 0 ? 1 : ((rank[k] < p.n_keep - 1 && par[c] != -2) ? 2 : 0);
  }
  __syncthreads();

  // 3. closure: an undecided candidate is kept once its parent is, dropped once its parent is
  for (;;) {
    bool progressed = false;
    uint8_t decided[kPerThread];
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
      const int c = tid * kPerThread + k;
      decided[k] = 2;
      if (c < m && state[c] == 2 && state[par[c]] != 2) {
        decided[k] = state[par[c]];
        progressed = true;
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kPerThread; ++k)
      if (decided[k] != 2) state[tid * kPerThread + k] = decided[k];
    if (!__syncthreads_or(progressed)) break;
  }

  // 4. node index = kept candidates before it
  int local = 0;
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    const int c = tid * kPerThread + k;
    local += (c < m && state[c] == 1) ? 1 : 0;
  }
  int incl = local;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int v = __shfl_up(incl, off);
    if (lane >= off) incl += v;
  }
  if (lane == 63) wave_count[wave] = incl;
  __syncthreads();
  int before = incl - local;
  for (int w2 = 0; w2 < wave; ++w2) before += wave_count[w2];
  const int total = wave_count[0] + wave_count[1] + wave_count[2] + wave_count[3];
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    const int c = tid * kPerThread + k;
    if (c < m) {
      const bool kept = state[c] == 1;
      node_of[c] = kept ? (int16_t)before : (int16_t)-1;
      before += kept ? 1 : 0;
    }
  }
  __syncthreads();
  int32_t* out_par = p.parent + (size_t)b * p.Nmax;
  int32_t* out_tok = p.tokens + (size_t)b * p.Nmax;
  int32_t* out_cand = p.node_cand + (size_t)b * p.Nmax;
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    const int c = tid * kPerThread + k;
    if (c < m && node_of[c] >= 0) {   // total <= n_keep <= Nmax
      const int i = node_of[c];
      const int pi = c == 0 ? -1 : node_of[par[c]];
      node_par[i] = (int16_t)pi;
      out_par[i] = pi;
      out_tok[i] = p.cand_token[(size_t)b * p.M + c];
      out_cand[i] = c;
    }
  }
  __syncthreads();
  if (tid < p.Nmax) {
    uint64_t word = 0;
    if (tid < total) {
      for (int a = tid; a >= 0; a = node_par[a]) word |= 1ull << a;   // parents have smaller indices: it ends
    } else {
      out_par[tid] = -1; out_tok[tid] = -1; out_cand[tid] = -1;
    }
    p.anc_mask[(size_t)b * p.Nmax + tid] = word;
  }
  if (tid == 0) p.n_nodes[b] = total;
}

}  // namespace

extern "C" fspad_status fspad_tree_build(int32_t B, int32_t M, int32_t Nmax, const int32_t* cand_parent,
                                         const int32_t* cand_token, const float* cand_logp,
                                         const int32_t* n_cand, int32_t n_keep, int32_t* parent,
                                         int32_t* draft_tokens, int32_t* n_nodes, uint64_t* anc_mask,
                                         int32_t* node_cand, void* hip_stream) {
  if (!cand_parent || !cand_token || !cand_logp || !n_cand || !parent || !draft_tokens || !n_nodes || !anc_mask ||
      !node_cand)
    return FSPAD_ERR_NULL;
  if (B < 1 || M < 1 || M > FSPAD_MAX_CANDIDATES || Nmax < 1 || Nmax > FSPAD_MAX_NODES || n_keep < 1 || n_keep > Nmax)
    return FSPAD_ERR_SHAPE;
  BuildParams prm{cand_parent, cand_token, cand_logp, n_cand, parent, draft_tokens, n_nodes, anc_mask, node_cand,
                  M, Nmax, n_keep};
  hipLaunchKernelGGL(tree_build_kernel, dim3((unsigned)B), dim3(kThreads), 0, reinterpret_cast<hipStream_t>(hip_stream), prm);
  return hipGetLastError() == hipSuccess ? FSPAD_OK : FSPAD_ERR_HIP;
}
