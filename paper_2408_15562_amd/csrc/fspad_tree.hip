// Dynamic draft tree from its candidates (arXiv 2408.15562, Preliminaries, last paragraph:
// per-step top-k, joint probabilities from the dependencies, one more top-k over all tokens;
// then the tokens are organised into a tree and the attention mask derived from it).
// One workgroup per sequence, one thread per candidate (256, 512 or 1024 threads), everything in
// LDS: at most 1024 candidates, a few microseconds.
//   1. joint scores, level by level (a candidate is scored once its parent is)
//   2. rank of every candidate = number of candidates that beat it (score, then index): each
//      candidate becomes one 64-bit word (order-preserving score bits, complemented index), so
//      that "beats" is one unsigned comparison against broadcast LDS reads
//   3. kept = rank < n_keep-1, closed under "parent kept" (level by level again)
//   4. node index = number of kept candidates before it; parents, tokens, ancestor words
#include "fspad.h"

#include <hip/hip_runtime.h>
#include <math.h>

namespace {

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

// float -> unsigned with the same order (-0 ranks with +0)
__device__ __forceinline__ unsigned ordered_bits(float x) {
  const unsigned u = __float_as_uint(x + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <int THREADS>
__global__ __launch_bounds__(THREADS) void tree_build_kernel(const BuildParams p) {
  constexpr int kWavesPerWg = THREADS / 64;
  typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
  __shared__ float joint[THREADS];
  __shared__ __attribute__((aligned(16))) unsigned long long keys[THREADS];   // 0: not a competitor
  __shared__ int16_t node_of[THREADS];   // node index of a kept candidate, else -1
  __shared__ uint8_t state[THREADS];     // pass 1: scored; pass 2: 1 kept, 0 dropped, 2 undecided
  __shared__ int16_t node_par[FSPAD_MAX_NODES];
  __shared__ int wave_count[kWavesPerWg];
  const int b = blockIdx.x, c = threadIdx.x, lane = c & 63, wave = c >> 6;   // candidate c belongs to thread c
  int m = p.n_cand[b];
  m = m < 1 ? 1 : (m > p.M ? p.M : m);
  m = m > THREADS ? THREADS : m;
  const int32_t* cp = p.cand_parent + (size_t)b * p.M;
  const float* lp = p.cand_logp + (size_t)b * p.M;

  float my_lp = 0.f;
  int my_par = -2;          // -1 root, -2 unreachable / no candidate
  bool pending = false;
  if (c < m) {
    const int pc = cp[c];
    const float v = lp[c];
    my_par = c == 0 ? -1 : ((pc >= 0 && pc < c) ? pc : -2);
    my_lp = (v != v) ? -INFINITY : v;
    pending = my_par >= 0;
    state[c] = c == 0 ? 1 : 0;
    joint[c] = c == 0 ? 0.f : -INFINITY;   // a candidate that is never reached keeps -infinity
  }
  __syncthreads();

  // 1. joint scores: a candidate is scored in the round after its parent was
  for (;;) {
    const bool newly = pending && state[my_par];
    if (newly) {
      joint[c] = joint[my_par] + my_lp;
      pending = false;
    }
    __syncthreads();   // all reads of state[] of this round are done
    if (newly) state[c] = 1;
    if (!__syncthreads_or(newly)) break;
  }
  // candidates that were never reached (bad parent index somewhere above them) cannot be kept
  if (pending) my_par = -2;

  // 2. rank among the non-root candidates: higher joint first, then lower index
  const unsigned long long mine =
      (c > 0 && c < m) ? (((unsigned long long)ordered_bits(joint[c]) << 32) | (0xffffffffu - (unsigned)c)) : 0ull;
  keys[c] = mine;
  __syncthreads();
  int rank = 0;
  const u32x4* keys2 = reinterpret_cast<const u32x4*>(keys);   // two words per read
  for (int j8 = 0; j8 < (m + 7) / 8; ++j8) {   // entries from m on are 0
    u32x4 o[4];   // same addresses in all lanes: four broadcast reads, issued together
#pragma unroll
    for (int u = 0; u < 4; ++u) o[u] = keys2[4 * j8 + u];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const unsigned long long k0 = ((unsigned long long)o[u][1] << 32) | o[u][0];
      const unsigned long long k1 = ((unsigned long long)o[u][3] << 32) | o[u][2];
      rank += (int)(k0 > mine) + (int)(k1 > mine);
    }
  }
  pending = false;
  __syncthreads();   // state[] is reused below
  if (c < m) {
    const bool top = c > 0 && rank < p.n_keep - 1 && my_par >= 0;
    state[c] = c == 0 ? 1 : (top ? 2 : 0);
    pending = top;
  }
  __syncthreads();

  // 3. closure: an undecided candidate is kept once its parent is, dropped once its parent is
  for (;;) {
    uint8_t decided = 2;
    if (pending) {
      const uint8_t ps = state[my_par];
      if (ps != 2) { decided = ps; pending = false; }
    }
    __syncthreads();
    if (decided != 2) state[c] = decided;
    if (!__syncthreads_or(decided != 2)) break;
  }

  // 4. node index = kept candidates before it
  const int kept = (c < m && state[c] == 1) ? 1 : 0;
  int incl = kept;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int v = __shfl_up(incl, off);
    if (lane >= off) incl += v;
  }
  if (lane == 63) wave_count[wave] = incl;
  __syncthreads();
  int before = incl - kept, total = 0;   // total <= n_keep <= Nmax
#pragma unroll
  for (int w2 = 0; w2 < kWavesPerWg; ++w2) {
    before += w2 < wave ? wave_count[w2] : 0;
    total += wave_count[w2];
  }
  const int my_node = kept ? before : -1;
  if (c < m) node_of[c] = (int16_t)my_node;
  __syncthreads();
  int32_t* out_par = p.parent + (size_t)b * p.Nmax;
  int32_t* out_tok = p.tokens + (size_t)b * p.Nmax;
  int32_t* out_cand = p.node_cand + (size_t)b * p.Nmax;
  if (my_node >= 0) {
    const int pi = c == 0 ? -1 : node_of[my_par];
    node_par[my_node] = (int16_t)pi;
    out_par[my_node] = pi;
    out_tok[my_node] = p.cand_token[(size_t)b * p.M + c];
    out_cand[my_node] = c;
  }
  __syncthreads();
  if (c < p.Nmax) {
    uint64_t word = 0;
    if (c < total) {
      for (int a = c; a >= 0; a = node_par[a]) word |= 1ull << a;   // parents have smaller indices: it ends
    } else {
      out_par[c] = -1; out_tok[c] = -1; out_cand[c] = -1;
    }
    p.anc_mask[(size_t)b * p.Nmax + c] = word;
  }
  if (c == 0) p.n_nodes[b] = total;
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
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  if (M <= 256) hipLaunchKernelGGL(tree_build_kernel<256>, dim3((unsigned)B), dim3(256), 0, stream, prm);
  else if (M <= 512) hipLaunchKernelGGL(tree_build_kernel<512>, dim3((unsigned)B), dim3(512), 0, stream, prm);
  else hipLaunchKernelGGL(tree_build_kernel<1024>, dim3((unsigned)B), dim3(1024), 0, stream, prm);
  return hipGetLastError() == hipSuccess ? FSPAD_OK : FSPAD_ERR_HIP;
}
