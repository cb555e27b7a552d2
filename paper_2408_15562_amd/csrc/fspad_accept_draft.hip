// Tree acceptance for drafts that were sampled from a draft distribution q (arXiv 2408.15562,
// Introduction: the draft-then-verify scheme of speculative sampling that keeps the target's output
// distribution), in its multi-candidate form: at a node with target distribution p and draft
// distribution q the children are tested in sibling order,
//
//     accept x  <=>  u q(x) < p(x);      reject x:  p <- max(p - q, 0) / sum,  q(x) <- 0, q <- q / sum
//
// and when none is accepted the step's last token is drawn from what p has become. gfx950 (CDNA4) only.
//
// One workgroup of 1024 threads per sequence walks the tree; the two distributions of the current
// node live unnormalised in the workspace (fp64, 2 V entries per sequence) with their scale factors
// in registers, so that a rejection is one pass over them. Every decision is taken in fp64; all
// threads take it from the same values, so the control flow stays uniform without an exchange.
// The walk visits one row pair per accepted level: the cost is a few passes over 2 V entries per
// level, not a pass over all B N V logits.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "exp_nonpos.h"
#include "fspad.h"

namespace {

using fspad_detail::exp_nonpos;

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;

struct DraftAcceptParams {
  const float* logits;        // [B][Nmax][row_stride]
  const float* draft_logits;  // same layout
  int64_t row_stride;
  const int32_t* draft_tokens;
  const int32_t* parent;
  const int32_t* n_nodes;
  const float* uniforms;      // [B][2][Nmax]
  int32_t* path;
  int32_t* path_len;
  int32_t* tokens;
  int32_t* n_tokens;
  double* work;               // [B][2][V]: unnormalised p and q of the current node
  double inv_temperature;
  int32_t B, Nmax, V;
};

__device__ __forceinline__ double wg_sum(double v, double* sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  __syncthreads();                  // sh may still be read from the previous reduction
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  double s = 0.0;
#pragma unroll
  for (int i = 0; i < kWaves; ++i) s += sh[i];   // the same order in every thread
  return s;
}

__device__ __forceinline__ float wg_max(float v, float* sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  float m = sh[0];
#pragma unroll
  for (int i = 1; i < kWaves; ++i) m = fmaxf(m, sh[i]);
  return m;
}

__global__ __launch_bounds__(kThreads) void accept_sample_draft_kernel(const DraftAcceptParams p) {
  __shared__ double sh_d[kWaves];
  __shared__ float sh_f[kWaves];
  __shared__ double scan_incl[kThreads];
  __shared__ int sh_tok, sh_last;
  const int b = blockIdx.x, tid = threadIdx.x;
  const int64_t o = (int64_t)b * p.Nmax;
  const int n = p.n_nodes[b];
  const float* u_acc = p.uniforms + (int64_t)b * 2 * p.Nmax;
  const float* u_draw = u_acc + p.Nmax;
  double* wp = p.work + (int64_t)b * 2 * p.V;
  double* wq = wp + p.V;
  const int V = p.V;

  for (int i = tid; i < p.Nmax; i += kThreads) { p.path[o + i] = i == 0 ? 0 : -1; p.tokens[o + i] = -1; }

  int cur = 0, len = 1;
  for (;;) {
    // the node's two distributions, unnormalised: w = exp((l - max) / T), scale = 1 / sum
    const float* lrow = p.logits + (o + cur) * p.row_stride;
    const float* qrow = p.draft_logits + (o + cur) * p.row_stride;
    float mp = -INFINITY, mq = -INFINITY;
    for (int v = tid; v < V; v += kThreads) {
      const float a = lrow[v], c = qrow[v];
      if (a == a) mp = fmaxf(mp, a);
      if (c == c) mq = fmaxf(mq, c);
    }
    mp = wg_max(mp, sh_f);
    mq = wg_max(mq, sh_f);
    double zp = 0.0, zq = 0.0;
    for (int v = tid; v < V; v += kThreads) {
      const float a = lrow[v], c = qrow[v];
      const double ea = (a == a && mp > -INFINITY) ? exp_nonpos(((double)a - (double)mp) * p.inv_temperature) : 0.0;
      const double ec = (c == c && mq > -INFINITY) ? exp_nonpos(((double)c - (double)mq) * p.inv_temperature) : 0.0;
      wp[v] = ea; wq[v] = ec;
      zp += ea; zq += ec;
    }
    zp = wg_sum(zp, sh_d);
    zq = wg_sum(zq, sh_d);
    double sp = zp > 0.0 ? 1.0 / zp : 0.0, sq = zq > 0.0 ? 1.0 / zq : 0.0;   // p(v) = wp[v] * sp, q(v) = wq[v] * sq
    __syncthreads();                                                           // wp / wq are visible to every thread

    int next = -1;
    for (int c = cur + 1; c < n && len < p.Nmax; ++c) {
      if (p.parent[o + c] != cur) continue;
      const int x = p.draft_tokens[o + c];
      const bool valid = x >= 0 && x < V;
      const double px = valid ? wp[x] * sp : 0.0, qx = valid ? wq[x] * sq : 0.0;
      if ((double)u_acc[c] * qx < px) { next = c; break; }
      // rejected: p <- max(p - q, 0), renormalised; q loses x and is renormalised
      __syncthreads();                       // every thread has read wp[x], wq[x]
      double z = 0.0;
      for (int v = tid; v < V; v += kThreads) {
        const double r = fmax(wp[v] * sp - wq[v] * sq, 0.0);
        z += r;
      }
      z = wg_sum(z, sh_d);
      if (z > 0.0) {
        for (int v = tid; v < V; v += kThreads) wp[v] = fmax(wp[v] * sp - wq[v] * sq, 0.0);
        sp = 1.0 / z;
      }
      __syncthreads();                       // every thread is done with the old wq[x]
      if (valid && tid == 0) wq[x] = 0.0;
      __syncthreads();
      // what q keeps once x is gone, summed again from the entries (a difference of the old sum and
      // wq[x] would cancel when the drafter was nearly certain of x)
      double s = 0.0;
      for (int v = tid; v < V; v += kThreads) s += wq[v];
      s = wg_sum(s, sh_d);
      sq = s > 0.0 ? 1.0 / s : sq;
      __syncthreads();
    }
    if (next >= 0) {
      if (tid == 0) { p.tokens[o + len - 1] = p.draft_tokens[o + next]; p.path[o + len] = next; }
      ++len;
      cur = next;
      __syncthreads();                       // the next node overwrites wp / wq
      continue;
    }

    // no child accepted: inverse-CDF draw from the current p. Thread k owns the contiguous entries
    // [k * per, (k + 1) * per); the target is u times the sum formed in the same order as the scan.
    const int per = (V + kThreads - 1) / kThreads;
    const int v0 = tid * per, v1 = min(V, v0 + per);
    double mine = 0.0;
    for (int v = v0; v < v1; ++v) mine += wp[v];
    scan_incl[tid] = mine;
    __syncthreads();
    for (int off = 1; off < kThreads; off <<= 1) {   // Hillis-Steele inclusive scan
      const double add = tid >= off ? scan_incl[tid - off] : 0.0;
      __syncthreads();
      scan_incl[tid] += add;
      __syncthreads();
    }
    const double total = scan_incl[kThreads - 1];
    const double t = (double)u_draw[cur] * total;
    if (tid == 0) { sh_tok = -1; sh_last = kThreads; }
    __syncthreads();
    // the scanned sums chain from 0 to the total, so some segment brackets t; they are formed in
    // different orders and need not be monotone to the last bit: the first bracketing segment counts
    const double before = tid > 0 ? scan_incl[tid - 1] : 0.0;
    if (before <= t && t < scan_incl[tid]) atomicMin(&sh_last, tid);
    __syncthreads();
    if (tid == sh_last) {
      double run = before;
      int tok = -1;
      for (int v = v0; v < v1; ++v) {
        run += wp[v];
        if (run > t) { tok = v; break; }
      }
      if (tok < 0)   // the segment's own sum said "here" but its running sum fell short: its last entry with mass
        for (int v = v1 - 1; v >= v0; --v)
          if (wp[v] > 0.0) { tok = v; break; }
      sh_tok = tok;
    }
    __syncthreads();
    if (sh_tok < 0) {   // rounding left no crossing: the last entry with mass (0 if none)
      int last = -1;
      for (int v = v1 - 1; v >= v0; --v)
        if (wp[v] > 0.0) { last = v; break; }
      if (tid == 0) sh_last = -1;
      __syncthreads();
      if (last >= 0) atomicMax(&sh_last, last);   // the highest such entry over the workgroup
      __syncthreads();
      if (tid == 0) sh_tok = sh_last < 0 ? 0 : sh_last;
      __syncthreads();
    }
    if (tid == 0) {
      p.tokens[o + len - 1] = sh_tok;
      p.path_len[b] = len;
      p.n_tokens[b] = len;
    }
    return;
  }
}

}  // namespace

extern "C" size_t fspad_tree_accept_sample_draft_workspace_bytes(int32_t B, int32_t Nmax, int32_t V) {
  if (B < 1 || Nmax < 1 || V < 1) return 0;
  return ((size_t)B * 2 * (size_t)V * 8 + 255) & ~(size_t)255;
}

extern "C" fspad_status fspad_tree_accept_sample_draft(int32_t B, int32_t Nmax, int32_t V, const float* logits,
                                                       const float* draft_logits, int64_t row_stride,
                                                       const int32_t* draft_tokens, const int32_t* parent,
                                                       const int32_t* n_nodes, float temperature, const float* uniforms,
                                                       int32_t* path, int32_t* path_len, int32_t* tokens,
                                                       int32_t* n_tokens, void* workspace, size_t workspace_bytes,
                                                       void* hip_stream) {
  if (!logits || !draft_logits || !draft_tokens || !parent || !n_nodes || !uniforms || !path || !path_len || !tokens ||
      !n_tokens)
    return FSPAD_ERR_NULL;
  if (B < 1 || Nmax < 1 || Nmax > FSPAD_MAX_NODES || V < 1 || row_stride < V) return FSPAD_ERR_SHAPE;
  if (!(temperature > 0.0f) || temperature > 3.0e38f) return FSPAD_ERR_TEMPERATURE;
  if (!workspace || ((uintptr_t)workspace & 15) ||
      workspace_bytes < fspad_tree_accept_sample_draft_workspace_bytes(B, Nmax, V))
    return FSPAD_ERR_WORKSPACE;
  DraftAcceptParams p{};
  p.logits = logits; p.draft_logits = draft_logits; p.row_stride = row_stride;
  p.draft_tokens = draft_tokens; p.parent = parent; p.n_nodes = n_nodes; p.uniforms = uniforms;
  p.path = path; p.path_len = path_len; p.tokens = tokens; p.n_tokens = n_tokens;
  p.work = static_cast<double*>(workspace);
  p.inv_temperature = 1.0 / (double)temperature;
  p.B = B; p.Nmax = Nmax; p.V = V;
  hipLaunchKernelGGL(accept_sample_draft_kernel, dim3((unsigned)B), dim3(kThreads), 0,
                     reinterpret_cast<hipStream_t>(hip_stream), p);
  return hipGetLastError() == hipSuccess ? FSPAD_OK : FSPAD_ERR_HIP;
}
