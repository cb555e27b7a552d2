// Dynamic draft tree from its candidates (arXiv 2408.15562, Preliminaries, last paragraph:
// per-step top-k, joint probabilities from the dependencies, one more top-k over all tokens;
// then the tokens are organised into a tree and the attention mask derived from it).
// One workgroup per sequence, everything in LDS: at most 1024 candidates, a few microseconds.
// Candidate c belongs to thread c % 256 (row c / 256 of that thread).
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
  __shared__ int16_t node_of[FSPAD_MAX_CANDIDATES];  // node index of a kept candidate, else -1
  __shared__ uint8_t state[FSPAD_MAX_CANDIDATES];    // pass 1: scored; pass 2: 1 kept, 0 dropped, 2 undecided
  __shared__ int16_t node_par[FSPAD_MAX_NODES];
  __shared__ int wave_count[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int m = p.n_cand[b];
  m = m < 1 ? 1 : (m > p.M ? p.M : m);
  const int rows = (m + kThreads - 1) / kThreads;   // candidate c = k*256 + tid belongs to row k of thread tid
  const int32_t* cp = p.cand_parent + (size_t)b * p.M;
  const float* lp = p.cand_logp + (size_t)b * p.M;

  // per-candidate values stay in registers; LDS holds what other threads look up
  float my_lp[kPerThread];
  int my_par[kPerThread];       // -1 root, -2 unreachable / no candidate
  bool pending[kPerThread];
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    const int c = k * kThreads + tid;
    my_lp[k] = 0.f;
    my_par[k] = -2;
    pending[k] = false;
    if (c < m) {
      const int pc = cp[c];
      const float v = lp[c];
      my_par[k] = c == 0 ? -1 : ((pc >= 0 && pc < c) ? pc : -2);
      my_lp[k] = (v != v) ? -INFINITY : v;
      pending[k] = my_par[k] >= 0;
      state[c] = c == 0 ? 1 : 0;
      joint[c] = c == 0 ? 0.f : -INFINITY;   // a candidate that is never reached keeps -infinity
    } else {
      joint[c] = -INFINITY;   // padding: never beats a candidate (its index is larger as well)
    }
  }
  __syncthreads();

  // 1. joint scores: a candidate is scored in the round after its parent was
  for (;;) {
    bool progressed = false;
    bool newly[kPerThread];
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
      newly[k] = false;
      if (k < rows && pending[k] && state[my_par[k]]) {
        joint[k * kThreads + tid] = joint[my_par[k]] + my_lp[k];
        newly[k] = true;
        pending[k] = false;
        progressed = true;
      }
    }
    __syncthreads();   // all reads of state[] of this round are done
#pragma unroll
    for (int k = 0; k < kPerThread; ++k)
      if (newly[k]) state[k * kThreads + tid] = 1;
    if (!__syncthreads_or(progressed)) break;
  }
  // candidates that were never reached (bad parent index somewhere above them) cannot be kept
#pragma unroll
  for (int k = 0; k < kPerThread; ++k)
    if (pending[k]) my_par[k] = -2;

  // 2. rank among the non-root candidates: higher joint first, then lower index
  int rank[kPerThread];
  float mine[kPerThread];
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    rank[k] = 0;
    mine[k] = joint[k * kThreads + tid];
  }
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  const f32x4* joint4 = reinterpret_cast<const f32x4*>(joint);
  for (int j16 = 0; j16 < (m + 15) / 16; ++j16) {   // the padding up to 1024 entries is -infinity
    f32x4 o[4];   // same addresses in all lanes: four broadcast reads, issued together
#pragma unroll
    for (int u = 0; u < 4; ++u) o[u] = joint4[4 * j16 + u];
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
      if (k >= rows) continue;    // uniform: rows past the last candidate cost nothing
      const int c = k * kThreads + tid;
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)   // bitwise on purpose: with || and && every comparison becomes a branch
          rank[k] += (int)(o[u][e] > mine[k]) | ((int)(o[u][e] == mine[k]) & (int)(16 * j16 + 4 * u + e < c));
    }
  }
  __syncthreads();   // state[] is reused below
  // the root (score 0, index 0) is not a competitor: its count is taken out again
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    const int c = k * kThreads + tid;
    rank[k] -= (int)(0.f > mine[k]) | ((int)(0.f == mine[k]) & (int)(0 < c));
    pending[k] = false;
    if (c < m) {
      const bool top = c > 0 && rank[k] < p.n_keep - 1 && my_par[k] >= 0;
      state[c] = c == 0 ? 1 : (top ? 2 : 0);
      pending[k] = top;
    }
  }
  __syncthreads();

  // 3. closure: an undecided candidate is kept once its parent is, dropped once its parent is
  for (;;) {
    bool progressed = false;
    uint8_t decided[kPerThread];
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
      decided[k] = 2;
      if (k < rows && pending[k]) {
        const uint8_t ps = state[my_par[k]];
        if (ps != 2) { decided[k] = ps; pending[k] = false; progressed = true; }
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kPerThread; ++k)
      if (decided[k] != 2) state[k * kThreads + tid] = decided[k];
    if (!__syncthreads_or(progressed)) break;
  }

  // 4. node index = kept candidates before it, one row of 256 candidates after the other
  int base = 0;
  int my_node[kPerThread];
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    my_node[k] = -1;
    if (k >= rows) continue;
    const int c = k * kThreads + tid;
    const int kept = (c < m && state[c] == 1) ? 1 : 0;
    int incl = kept;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int v = __shfl_up(incl, off);
      if (lane >= off) incl += v;
    }
    if (lane == 63) wave_count[wave] = incl;
    __syncthreads();
    int before = base + incl - kept;
    for (int w2 = 0; w2 < wave; ++w2) before += wave_count[w2];
    base += wave_count[0] + wave_count[1] + wave_count[2] + wave_count[3];
    if (kept) my_node[k] = before;
    if (c < m) node_of[c] = (int16_t)my_node[k];
    __syncthreads();   // wave_count is reused by the next row; node_of is read below
  }
  const int total = base;   // <= n_keep <= Nmax
  int32_t* out_par = p.parent + (size_t)b * p.Nmax;
  int32_t* out_tok = p.tokens + (size_t)b * p.Nmax;
  int32_t* out_cand = p.node_cand + (size_t)b * p.Nmax;
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    if (my_node[k] >= 0) {
      const int c = k * kThreads + tid, i = my_node[k];
      const int pi = c == 0 ? -1 : node_of[my_par[k]];
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
