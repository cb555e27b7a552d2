// Lossless acceptance over the per-node logits of a verified draft tree
// (arXiv 2408.15562, Preliminaries, validation phase: strict comparison of the
// tree with the target's results, a differing token dropped with all its
// descendants; Experiments "Settings": temperature 0 and 1, acceptance not
// relaxed). gfx950 (CDNA4) only.
//
// Two kernels per call. The first streams the [B*N, V] fp32 logits once, 16 bytes
// per lane, one workgroup per (row, chunk of 1024..8192 entries), and leaves per-chunk
// statistics: (max, first index of max) for greedy, (max, fp64 sum of
// exp((l-max)/T)) for sampling. The second, one workgroup per sequence, merges the
// chunk statistics of every row at once, walks the tree with wavefront ballots
// out of LDS and, for sampling, draws the last token by an inverse-CDF search that
// descends chunk -> thread segment -> element.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <atomic>
#include <stdint.h>

#include <mutex>

#include "fspad.h"
#include "exp_nonpos.h"
#include "greedy_walk.h"

namespace {

using fspad_detail::exp_nonpos;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kThreads = 256;
constexpr int kMinChunk = 1024;           // logits per workgroup of the streaming kernel: 1024 .. 8192,
constexpr int kMaxChunk = 8192;           // chosen per call so that small problems still fill the chip
constexpr int kMaxPerThread = kMaxChunk / kThreads;  // 32
constexpr int kNone = 0x7fffffff;

struct AcceptParams {
  const float* logits;
  int64_t row_stride;
  const int32_t* draft_tokens;
  const int32_t* parent;
  const int32_t* n_nodes;
  const float* uniforms;
  int32_t* path;
  int32_t* path_len;
  int32_t* tokens;
  int32_t* n_tokens;
  float* part_max;     // [rows][chunks]
  int32_t* part_idx;   // greedy  [rows][chunks]
  double* part_sum;    // sampling [rows][chunks]
  double inv_temperature;
  int32_t B, Nmax, V, n_chunks;
  int32_t chunk;       // logits per (row, chunk) workgroup: 256 * PT
  uint32_t* clear_words;   // words this launch sets to zero for the kernel behind it (may be null)
  int32_t clear_count;
  // a second logit array of the same shape for the same launch (grid.z = 2; sampling statistics only), or null
  const float* logits2;
  float* part_max2;
  double* part_sum2;
};

// Inclusive running sum over the 64 lanes of a wavefront, lane order, with data-parallel-primitive moves
// (no LDS round trips): four shifts inside each row of 16 lanes (a lane without a source adds 0), then the
// last lane of row 0 / 2 onto rows 1 / 3 and lane 31 onto rows 2 and 3.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_take(double v) {
  const unsigned long long bits = __builtin_bit_cast(unsigned long long, v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(unsigned)bits, CTRL, ROW_MASK, 0xf, true);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(unsigned)(bits >> 32), CTRL, ROW_MASK, 0xf, true);
  return __builtin_bit_cast(double, ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo);
}
__device__ __forceinline__ double wave_running_sum(double v) {
  v += dpp_take<0x111, 0xf>(v);   // row_shr:1
  v += dpp_take<0x112, 0xf>(v);   // row_shr:2
  v += dpp_take<0x114, 0xf>(v);   // row_shr:4
  v += dpp_take<0x118, 0xf>(v);   // row_shr:8
  v += dpp_take<0x142, 0xa>(v);   // row_bcast:15 onto rows 1 and 3
  v += dpp_take<0x143, 0xc>(v);   // row_bcast:31 onto rows 2 and 3
  return v;
}

__device__ __forceinline__ float clean(float x) { return (x != x) ? -INFINITY : x; }  // NaN ranks lowest

// (value, index) with "larger value, then lower index" order
__device__ __forceinline__ void take_better(float& v, int& i, float ov, int oi) {
  if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
}

// ------------------------------------------------------------------------------------------------
// Streaming pass. MODE 0: greedy (max, argmax). MODE 1: sampling (max, sum of exp).
// VEC: rows are 16-byte aligned so that float4 loads are legal.
template <int MODE, bool VEC, int PT>
__global__ __launch_bounds__(kThreads) void accept_rows_kernel(const AcceptParams p) {
  constexpr int kChunk = kThreads * PT;
  constexpr int kPerThread = PT;
  __shared__ float sh_max[4];
  __shared__ int sh_idx[4];
  __shared__ double sh_sum[4];
  const int row = blockIdx.y, chunk = blockIdx.x;
  const int b = row / p.Nmax, node = row - b * p.Nmax;
  if (row == 0 && chunk == 0)
    for (int i = threadIdx.x; i < p.clear_count; i += kThreads) p.clear_words[i] = 0u;
  if (node >= p.n_nodes[b]) return;  // rows of unused tree slots are never read
  const bool second = blockIdx.z != 0;
  const float* rp = (second ? p.logits2 : p.logits) + (int64_t)row * p.row_stride;
  float* const part_max = second ? p.part_max2 : p.part_max;
  double* const part_sum = second ? p.part_sum2 : p.part_sum;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int base = chunk * kChunk;

  float x[kPerThread];
#pragma unroll
  for (int k = 0; k < kPerThread / 4; ++k) {
    const int e0 = base + (k * kThreads + tid) * 4;
    if (VEC && e0 + 3 < p.V) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(rp + e0);
      x[4 * k] = clean(v[0]); x[4 * k + 1] = clean(v[1]); x[4 * k + 2] = clean(v[2]); x[4 * k + 3] = clean(v[3]);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) x[4 * k + j] = (e0 + j < p.V) ? clean(rp[e0 + j]) : -INFINITY;
    }
  }

  const int64_t slot = (int64_t)row * p.n_chunks + chunk;
  if (MODE == 1) {
    // sampling: each thread sums exp((x - its own max)/T) over its entries as soon as they arrive
    // (fp64, no waiting for the rest of the workgroup); the threads' (max, sum) pairs are then merged
    // into the chunk's: sum_c = sum_t sum_t * exp((max_t - max_c)/T).
    float mt = x[0];
#pragma unroll
    for (int k = 1; k < kPerThread; ++k) mt = fmaxf(mt, x[k]);
    double st = 0.0;
    if (mt > -INFINITY) {
      const double mtd = (double)mt;
#pragma unroll
      for (int k = 0; k < kPerThread; ++k) st += exp_nonpos(((double)x[k] - mtd) * p.inv_temperature);
    }
    float mw = mt;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mw = fmaxf(mw, __shfl_xor(mw, off));
    if (lane == 0) sh_max[wave] = mw;
    __syncthreads();
    const float mc = fmaxf(fmaxf(sh_max[0], sh_max[1]), fmaxf(sh_max[2], sh_max[3]));
    double sum = mt > -INFINITY ? st * exp_nonpos(((double)mt - (double)mc) * p.inv_temperature) : 0.0;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) sh_sum[wave] = sum;
    __syncthreads();
    if (tid == 0) {
      part_max[slot] = mc;
      part_sum[slot] = (sh_sum[0] + sh_sum[1]) + (sh_sum[2] + sh_sum[3]);
    }
    return;
  }

  float best = -INFINITY;
  int idx = kNone;
#pragma unroll
  for (int k = 0; k < kPerThread / 4; ++k)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (x[4 * k + j] > best) { best = x[4 * k + j]; idx = base + (k * kThreads + tid) * 4 + j; }

  // workgroup (max, index): wavefront butterflies, then 4 partials through LDS
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float ov = __shfl_xor(best, off);
    const int oi = __shfl_xor(idx, off);
    take_better(best, idx, ov, oi);
  }
  if (lane == 0) { sh_max[wave] = best; sh_idx[wave] = idx; }
  __syncthreads();
  best = sh_max[0]; idx = sh_idx[0];
#pragma unroll
  for (int w = 1; w < 4; ++w) take_better(best, idx, sh_max[w], sh_idx[w]);
  if (tid == 0) { part_max[slot] = best; p.part_idx[slot] = idx; }
}

// ------------------------------------------------------------------------------------------------
// Greedy: merge chunk argmaxes per node, then wavefront 0 descends while a child carries the
// target's token.
__global__ __launch_bounds__(kThreads) void accept_greedy_walk_kernel(const AcceptParams p) {
  __shared__ int amax[FSPAD_MAX_NODES];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = p.n_nodes[b];
  const int64_t o = (int64_t)b * p.Nmax;
  // the tree itself does not depend on the logits: wavefront 0 asks for it before anything else
  int my_par = -2, my_tok = -1;
  if (wave == 0 && lane < n) {
    my_par = p.parent[o + lane];
    my_tok = p.draft_tokens[o + lane];
  }
  // thread (node = lane, quarter = wave) scans every 4th chunk entry of its node, eight loads in
  // flight at a time; the four quarters of a node meet in LDS (no lane exchange needed)
  __shared__ float q_best[4][FSPAD_MAX_NODES];
  __shared__ int q_idx[4][FSPAD_MAX_NODES];
  {
    float best = -INFINITY;
    int idx = kNone;
    if (lane < n) {
      const int64_t slot0 = (o + lane) * p.n_chunks;
      for (int c0 = wave; c0 < p.n_chunks; c0 += 32) {
        float v[8];
        int ix[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int c = c0 + 4 * k;
          v[k] = c < p.n_chunks ? p.part_max[slot0 + c] : -INFINITY;
          ix[k] = c < p.n_chunks ? p.part_idx[slot0 + c] : kNone;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) take_better(best, idx, v[k], ix[k]);
      }
    }
    q_best[wave][lane] = best;
    q_idx[wave][lane] = idx;
  }
  __syncthreads();
  if (wave == 0 && lane < n) {
    float best = q_best[0][lane];
    int idx = q_idx[0][lane];
#pragma unroll
    for (int w = 1; w < 4; ++w) take_better(best, idx, q_best[w][lane], q_idx[w][lane]);
    amax[lane] = idx == kNone ? 0 : idx;  // a row with nothing above -inf: token 0
  }
  __syncthreads();
  if (wave != 0) return;
  fspad_detail::greedy_descend(amax, n, p.Nmax, lane, o, b, my_par, my_tok, p.path, p.tokens, p.path_len, p.n_tokens);
}

// ------------------------------------------------------------------------------------------------
// The sampling walk runs with 1024 threads: its code runs once per call, so what it costs is the
// longest chain of dependent fp64 instructions in any one thread and the number of instruction lines
// fetched (cold at every launch), and both shrink when the same arithmetic is spread over more lanes.
constexpr int kWalkThreads = 1024;
constexpr int kWalkWaves = kWalkThreads / 64;

// Last step of the sampling pass: the workgroup draws the token at which the running sum of the
// residual weights of one chunk crosses `target`. Thread k owns E consecutive entries; their
// weights are formed once and stay in registers, so the thread that owns the crossing finds it
// without touching memory again. If rounding leaves no crossing, the last entry with mass is taken.
struct DrawArgs {
  const float* rp;          // the row
  int first, V;             // first entry of the chunk, vocabulary size
  double M, target, inv_temperature;
  const int* rej_tok;       // tokens rejected at this node: zero weight
  int nrej;
  double* scan_part;        // LDS scratch: kWalkWaves doubles
  int* sh_wave;             // LDS scratch: 2 * kWalkWaves ints
  int32_t* out;
  bool vec;                 // rows are 16-byte aligned
};

template <int E>
__device__ __forceinline__ void draw_in_chunk(const DrawArgs& a) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int e0 = a.first + tid * E;
  float lx[E];
  if constexpr (E % 4 == 0) {
#pragma unroll
    for (int k = 0; k < E / 4; ++k) {
      const int e = e0 + 4 * k;
      if (a.vec && e + 3 < a.V) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(a.rp + e);
        lx[4 * k] = v[0]; lx[4 * k + 1] = v[1]; lx[4 * k + 2] = v[2]; lx[4 * k + 3] = v[3];
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) lx[4 * k + j] = (e + j < a.V) ? a.rp[e + j] : NAN;
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < E; ++j) lx[j] = (e0 + j < a.V) ? a.rp[e0 + j] : NAN;
  }
  unsigned gone = 0u;   // bit j: entry e0 + j was rejected at this node and has left the residual
  for (int k = 0; k < a.nrej; ++k) {
    const unsigned r = (unsigned)(a.rej_tok[k] - e0);
    if (r < (unsigned)E) gone |= 1u << r;
  }
  double w[E];
  double local = 0.0;
  int last_here = -1;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    double wj = 0.0;
    if (lx[j] == lx[j] && !((gone >> j) & 1u))   // not NaN (entries past the vocabulary were loaded as NaN)
      wj = exp_nonpos(((double)lx[j] - a.M) * a.inv_temperature);
    w[j] = wj;
    local += wj;
    if (wj > 0.0) last_here = e0 + j;
  }
  const double incl = wave_running_sum(local);
  if (lane == 63) a.scan_part[wave] = incl;
  __syncthreads();
  double wave_base = 0.0;   // the wavefronts before this one, in order (every partial is read: the loads go out together)
#pragma unroll
  for (int v = 0; v < kWalkWaves; ++v) {
    const double part = a.scan_part[v];
    if (v < wave) wave_base += part;
  }
  // the owner is the first thread whose inclusive running sum exceeds the target: first lane of a
  // wavefront by ballot, first wavefront through LDS (one slot each: no two lanes meet on an address)
  const double inclusive = wave_base + incl;
  const unsigned long long hits = __ballot(inclusive > a.target && local > 0.0);
  int last_wave = last_here;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) last_wave = max(last_wave, __shfl_xor(last_wave, off));
  if (lane == 0) {
    a.sh_wave[wave] = hits ? wave * 64 + (__ffsll(hits) - 1) : kNone;
    a.sh_wave[kWalkWaves + wave] = last_wave;
  }
  __syncthreads();
  int owner = kNone, last_any = -1;
#pragma unroll
  for (int v = 0; v < kWalkWaves; ++v) {
    owner = min(owner, a.sh_wave[v]);
    last_any = max(last_any, a.sh_wave[kWalkWaves + v]);
  }
  if (owner == kNone) {  // rounding left no crossing: the last entry with mass
    if (tid == 0) *a.out = last_any < 0 ? 0 : last_any;
    return;
  }
  if (tid == owner) {
    double run = inclusive - local;
    int pick = last_here;  // if rounding hides the crossing inside the segment: its last entry with mass
    bool done = false;
#pragma unroll
    for (int j = 0; j < E; ++j) {
      run += w[j];
      if (!done && run > a.target) { pick = e0 + j; done = true; }
    }
    *a.out = pick;
  }
}

// Sampling. Everything the walk can need is fetched up front, in parallel, so that the walk itself
// touches no memory: (1) the chunk statistics of every row are merged into the row's max M and
// normaliser Z (four threads per row); (2) every node fetches the weight of its own draft token
// under its parent's distribution (one gather for the whole tree; a token that an earlier sibling
// already proposed weighs nothing, because it has left the residual by the time it is tested);
// (3) wavefront 0 walks the tree out of LDS, testing the children of the current node in index
// order against the running residual; (4) the workgroup draws the last token.
__global__ __launch_bounds__(kWalkThreads) void accept_sample_walk_kernel(const AcceptParams p) {
  __shared__ int rej_tok[FSPAD_MAX_NODES];
  __shared__ double rej_w[FSPAD_MAX_NODES];
  __shared__ double sh_d[8];
  __shared__ int sh_i[8];
  __shared__ double scan_part[kWalkWaves];
  __shared__ int sh_wave[2 * kWalkWaves];
  __shared__ double row_M[FSPAD_MAX_NODES], row_Z[FSPAD_MAX_NODES], node_w[FSPAD_MAX_NODES];
  __shared__ int node_par[FSPAD_MAX_NODES], node_tok[FSPAD_MAX_NODES];
  __shared__ float node_u[2][FSPAD_MAX_NODES];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t o = (int64_t)b * p.Nmax;
  const float* u_acc = p.uniforms + (int64_t)b * 2 * p.Nmax;

  // (1) row statistics: thread (row = tid / 16, part = tid % 16) takes every 16th chunk of its row,
  // two chunks in flight at a time, keeping a running (max, sum); the sixteen parts of a row are then
  // merged with lane exchanges. Nothing here waits for the tree size: rows past it hold unused numbers.
  const int n_raw = p.n_nodes[b];
  {
    const int row = tid >> 4, q = tid & 15;
    const bool in_range = row < p.Nmax;
    const float* pm = p.part_max + (o + (in_range ? row : 0)) * p.n_chunks;
    const double* ps = p.part_sum + (o + (in_range ? row : 0)) * p.n_chunks;
    float m_run = -INFINITY;
    double z_run = 0.0;
    for (int c0 = q; c0 < p.n_chunks; c0 += 32) {
      float m_c[2];
      double s_c[2];
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int c = c0 + 16 * k;
        const bool ok = in_range && c < p.n_chunks;
        m_c[k] = ok ? pm[c] : -INFINITY;
        s_c[k] = ok ? ps[c] : 0.0;
      }
      const float m_new = fmaxf(m_run, fmaxf(m_c[0], m_c[1]));
      if (m_new > -INFINITY) {
        double z = m_run > -INFINITY ? z_run * exp_nonpos(((double)m_run - (double)m_new) * p.inv_temperature) : 0.0;
#pragma unroll
        for (int k = 0; k < 2; ++k)
          if (m_c[k] > -INFINITY) z += s_c[k] * exp_nonpos(((double)m_c[k] - (double)m_new) * p.inv_temperature);
        z_run = z;
        m_run = m_new;
      }
    }
    float mx = m_run;
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    double z = m_run > -INFINITY ? z_run * exp_nonpos(((double)m_run - (double)mx) * p.inv_temperature) : 0.0;
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) z += __shfl_xor(z, off);
    if (in_range && q == 0) { row_M[row] = (double)mx; row_Z[row] = z; }
    if (tid < FSPAD_MAX_NODES) {
      const bool ok = tid < p.Nmax;
      node_par[tid] = ok ? p.parent[o + tid] : -2;
      node_tok[tid] = ok ? p.draft_tokens[o + tid] : -1;
      node_u[0][tid] = ok ? u_acc[tid] : 0.f;
      node_u[1][tid] = ok ? u_acc[p.Nmax + tid] : 0.f;
    }
  }
  const int n = n_raw;
  __syncthreads();
  // (2) weight of every node's draft token under its parent's row
  if (tid < FSPAD_MAX_NODES) {
    double w = 0.0;
    const int par = node_par[tid], tok = node_tok[tid];
    if (tid > 0 && tid < n && par >= 0 && par < tid && tok >= 0 && tok < p.V) {
      const double M = row_M[par];
      if (M > -INFINITY) {
        const float lx = p.logits[(o + par) * p.row_stride + tok];
        if (lx == lx) w = exp_nonpos(((double)lx - M) * p.inv_temperature);
      }
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
    __builtin_amdgcn_wave_barrier();
    if (lane < p.Nmax) { p.path[o + lane] = my_path; if (lane != len - 1) p.tokens[o + lane] = my_out; }
    if (lane == 0) {
      p.path_len[b] = len; p.n_tokens[b] = len;
      sh_i[0] = cur; sh_i[1] = len; sh_i[2] = nrej;
      sh_d[0] = M; sh_d[1] = Z;
    }

    // bonus, stage 1: which chunk holds the running-sum crossing of t = u * Z
    const double t = (double)node_u[1][cur] * Z;
    const int64_t row = o + cur;
    const float* pm = p.part_max + row * p.n_chunks;
    const double* ps = p.part_sum + row * p.n_chunks;
    double carry = 0.0, before = 0.0;
    int found = -1, last_pos = -1;
    for (int c0 = 0; c0 < p.n_chunks && found < 0; c0 += 64) {
      const int c = c0 + lane;
      double r = 0.0;
      if (c < p.n_chunks && pm[c] > -INFINITY) {
        r = ps[c] * exp_nonpos(((double)pm[c] - M) * p.inv_temperature);
        for (int k = 0; k < nrej; ++k)
          if (rej_tok[k] >= c * p.chunk && rej_tok[k] < (c + 1) * p.chunk && rej_tok[k] < p.V) r -= rej_w[k];
      }
      const double incl = wave_running_sum(r);
      const unsigned long long pos = __ballot(r > 0.0);
      if (pos) last_pos = c0 + 63 - __clzll(pos);
      const unsigned long long hit = __ballot(c < p.n_chunks && carry + incl > t);
      if (hit) {
        const int first = __ffsll(hit) - 1;
        found = c0 + first;
        before = carry + __shfl(incl - r, first);
      } else {
        carry += __shfl(incl, 63);
      }
    }
    if (lane == 0) {
      // rounding fallback: the last chunk that still has mass, searched to its end
      sh_i[3] = found >= 0 ? found : last_pos;
      sh_i[4] = found >= 0;
      sh_d[2] = found >= 0 ? t - before : INFINITY;
    }
  }
  __syncthreads();

  // bonus, stage 2: inside the chunk, thread k owns chunk/1024 consecutive entries
  const int cur = sh_i[0], len = sh_i[1], nrej = sh_i[2], chunk = sh_i[3];
  if (chunk < 0) {  // no mass anywhere (cannot happen with finite logits): token 0
    if (tid == 0) p.tokens[o + len - 1] = 0;
    return;
  }
  DrawArgs a;
  a.rp = p.logits + (o + cur) * p.row_stride;
  a.first = chunk * p.chunk;
  a.V = p.V;
  a.M = sh_d[0];
  a.target = sh_d[2];
  a.inv_temperature = p.inv_temperature;
  a.rej_tok = rej_tok;
  a.nrej = nrej;
  a.scan_part = scan_part;
  a.sh_wave = sh_wave;
  a.out = p.tokens + o + len - 1;
  a.vec = (((uintptr_t)p.logits) & 15) == 0 && (p.row_stride % 4) == 0;
  switch (p.chunk / kWalkThreads) {
    case 1: draw_in_chunk<1>(a); break;
    case 2: draw_in_chunk<2>(a); break;
    case 4: draw_in_chunk<4>(a); break;
    default: draw_in_chunk<8>(a); break;
  }
}

// Largest chunk that still gives about a thousand workgroups (rows x chunks), so that a few rows of
// a small vocabulary are spread over the whole chip.
constexpr int kTargetWorkgroups = 1024;
int pick_chunk(int32_t B, int32_t Nmax, int32_t V) {
  int chunk = kMaxChunk;
  while (chunk > kMinChunk && (int64_t)B * Nmax * ((V + chunk - 1) / chunk) < kTargetWorkgroups) chunk >>= 1;
  return chunk;
}

fspad_status check_accept_args(int32_t B, int32_t Nmax, int32_t V, const float* logits, int64_t row_stride,
                               const int32_t* draft_tokens, const int32_t* parent, const int32_t* n_nodes,
                               int32_t* path, int32_t* path_len, int32_t* tokens, int32_t* n_tokens,
                               void* workspace, size_t workspace_bytes) {
  if (!logits || !draft_tokens || !parent || !n_nodes || !path || !path_len || !tokens || !n_tokens) return FSPAD_ERR_NULL;
  if (B < 1 || Nmax < 1 || Nmax > FSPAD_MAX_NODES || V < 1 || V > (1 << 30) || row_stride < V) return FSPAD_ERR_SHAPE;
  if ((int64_t)B * Nmax > 65535) return FSPAD_ERR_SHAPE;  // grid.y
  if (((uintptr_t)logits) & 3) return FSPAD_ERR_SHAPE;
  if (!workspace || ((uintptr_t)workspace & 15) || workspace_bytes < fspad_tree_accept_workspace_bytes(B, Nmax, V))
    return FSPAD_ERR_WORKSPACE;
  return FSPAD_OK;
}

void fill_params(AcceptParams& p, int32_t B, int32_t Nmax, int32_t V, const float* logits, int64_t row_stride,
                 const int32_t* draft_tokens, const int32_t* parent, const int32_t* n_nodes, int32_t* path,
                 int32_t* path_len, int32_t* tokens, int32_t* n_tokens, void* workspace) {
  p.logits = logits; p.row_stride = row_stride; p.draft_tokens = draft_tokens; p.parent = parent;
  p.n_nodes = n_nodes; p.path = path; p.path_len = path_len; p.tokens = tokens; p.n_tokens = n_tokens;
  p.B = B; p.Nmax = Nmax; p.V = V;
  p.chunk = pick_chunk(B, Nmax, V);
  p.n_chunks = (V + p.chunk - 1) / p.chunk;
  const size_t slots = (size_t)B * Nmax * p.n_chunks;
  p.part_sum = reinterpret_cast<double*>(workspace);                 // 8-byte entries first
  p.part_max = reinterpret_cast<float*>(p.part_sum + slots);
  p.part_idx = reinterpret_cast<int32_t*>(p.part_max + slots);
  p.uniforms = nullptr;
  p.inv_temperature = 1.0;
}

bool rows_vectorisable(const float* logits, int64_t row_stride) {
  return (((uintptr_t)logits) & 15) == 0 && (row_stride % 4) == 0;
}

template <int MODE>
void launch_rows(const AcceptParams& p, bool vec, hipStream_t stream) {
  const dim3 grid((unsigned)p.n_chunks, (unsigned)(p.B * p.Nmax), p.logits2 ? 2u : 1u);
#define FSPAD_ROWS(PT)                                                                                         \
  do {                                                                                                           \
    if (vec) hipLaunchKernelGGL((accept_rows_kernel<MODE, true, PT>), grid, dim3(kThreads), 0, stream, p);      \
    else hipLaunchKernelGGL((accept_rows_kernel<MODE, false, PT>), grid, dim3(kThreads), 0, stream, p);         \
  } while (0)
  switch (p.chunk / kThreads) {
    case 4: FSPAD_ROWS(4); break;
    case 8: FSPAD_ROWS(8); break;
    case 16: FSPAD_ROWS(16); break;
    default: FSPAD_ROWS(32); break;
  }
#undef FSPAD_ROWS
}

// ------------------------------------------------------------------------------------------------
// Acceptance for drafts that were sampled from a draft distribution q (Introduction: the
// draft-then-verify scheme of speculative sampling), in its multi-candidate form: at a node with
// target distribution p and draft distribution q the children are tested in sibling order,
//     accept x  <=>  u q(x) < p(x);      reject x:  p <- max(p - q, 0) / sum,  q(x) <- 0, q <- q / sum
// and when none is accepted the step's last token is drawn from what p has become.
//
// The streaming pass above leaves the chunk statistics of both logit arrays; one workgroup of 1024
// threads per sequence then walks the tree. Every decision is taken in fp64; all threads take it
// from the same values, so the control flow stays uniform without an exchange. A rejection or the
// draw needs the node's two whole rows: they are then written out unnormalised (fp64, 2 V entries
// per sequence) with their scale factors in registers, and every further rejection is one pass.
constexpr int kDraftThreads = 1024;
constexpr int kDraftWaves = kDraftThreads / 64;

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
  double* work;               // [B][3][V]: unnormalised p, a spare for the next p, and q of the current node
  const float* part_max_p;    // [B*Nmax][n_chunks] chunk statistics of logits (accept_rows_kernel<1>)
  const double* part_sum_p;
  const float* part_max_q;    // the same of draft_logits
  const double* part_sum_q;
  double inv_temperature;
  int32_t B, Nmax, V, n_chunks;
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
  for (int i = 0; i < kDraftWaves; ++i) s += sh[i];   // the same order in every thread
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
  for (int i = 1; i < kDraftWaves; ++i) m = fmaxf(m, sh[i]);
  return m;
}

__global__ __launch_bounds__(kDraftThreads) void accept_sample_draft_kernel(const DraftAcceptParams p) {
  __shared__ double sh_d[kDraftWaves];
  __shared__ float sh_f[kDraftWaves];
  __shared__ int sh_tok, sh_last;
  const int b = blockIdx.x, tid = threadIdx.x;
  const int64_t o = (int64_t)b * p.Nmax;
  const int n = p.n_nodes[b];
  const float* u_acc = p.uniforms + (int64_t)b * 2 * p.Nmax;
  const float* u_draw = u_acc + p.Nmax;
  double* wp = p.work + (int64_t)b * 3 * p.V;   // unnormalised p of the current node
  double* wp_spare = wp + p.V;                  // where a rejection writes the next p
  double* wq = wp + 2 * p.V;                    // unnormalised q
  const int V = p.V;

  for (int i = tid; i < p.Nmax; i += kDraftThreads) { p.path[o + i] = i == 0 ? 0 : -1; p.tokens[o + i] = -1; }

  int cur = 0, len = 1;
  for (;;) {
    // row statistics of the node from the chunk statistics of the streaming pass: p(v) = exp((l[v] - mp) / T) / zp
    const float* lrow = p.logits + (o + cur) * p.row_stride;
    const float* qrow = p.draft_logits + (o + cur) * p.row_stride;
    float mp = -INFINITY, mq = -INFINITY;
    for (int c = tid; c < p.n_chunks; c += kDraftThreads) {
      mp = fmaxf(mp, p.part_max_p[(o + cur) * p.n_chunks + c]);
      mq = fmaxf(mq, p.part_max_q[(o + cur) * p.n_chunks + c]);
    }
    mp = wg_max(mp, sh_f);
    mq = wg_max(mq, sh_f);
    double zp = 0.0, zq = 0.0;
    for (int c = tid; c < p.n_chunks; c += kDraftThreads) {
      const float cp = p.part_max_p[(o + cur) * p.n_chunks + c], cq = p.part_max_q[(o + cur) * p.n_chunks + c];
      if (cp > -INFINITY) zp += p.part_sum_p[(o + cur) * p.n_chunks + c] * exp_nonpos(((double)cp - (double)mp) * p.inv_temperature);
      if (cq > -INFINITY) zq += p.part_sum_q[(o + cur) * p.n_chunks + c] * exp_nonpos(((double)cq - (double)mq) * p.inv_temperature);
    }
    zp = wg_sum(zp, sh_d);
    zq = wg_sum(zq, sh_d);
    double sp = zp > 0.0 ? 1.0 / zp : 0.0, sq = zq > 0.0 ? 1.0 / zq : 0.0;
    // The unnormalised weights of the whole rows are written out only when a rejection or the draw
    // needs them: a node whose first child is accepted costs two logits.
    bool filled = false;
    auto weight_p = [&](int v) {
      const float a = lrow[v];
      return (a == a && mp > -INFINITY) ? exp_nonpos(((double)a - (double)mp) * p.inv_temperature) : 0.0;
    };
    auto weight_q = [&](int v) {
      const float c = qrow[v];
      return (c == c && mq > -INFINITY) ? exp_nonpos(((double)c - (double)mq) * p.inv_temperature) : 0.0;
    };
    auto fill_p = [&]() {   // p alone, for a draw at a node without a rejection: p(v) = wp[v] * sp
      __syncthreads();
      for (int v = tid; v < V; v += kDraftThreads) wp[v] = weight_p(v);
      __syncthreads();
    };

    int next = -1;
    for (int c = cur + 1; c < n && len < p.Nmax; ++c) {
      if (p.parent[o + c] != cur) continue;
      const int x = p.draft_tokens[o + c];
      const bool valid = x >= 0 && x < V;
      double px = 0.0, qx = 0.0;
      if (valid && filled) {
        px = wp[x] * sp; qx = wq[x] * sq;
      } else if (valid) {
        const float a = lrow[x], d = qrow[x];
        px = (a == a && mp > -INFINITY) ? exp_nonpos(((double)a - (double)mp) * p.inv_temperature) * sp : 0.0;
        qx = (d == d && mq > -INFINITY) ? exp_nonpos(((double)d - (double)mq) * p.inv_temperature) * sq : 0.0;
      }
      if ((double)u_acc[c] * qx < px) { next = c; break; }
      // rejected: p <- max(p - q, 0), renormalised; q loses x and is renormalised
      if (!filled) {
        // the first rejection at this node: the rows are formed and the rejection applied in the same pass
        __syncthreads();
        double z = 0.0, s = 0.0;
        for (int v = tid; v < V; v += kDraftThreads) {
          const double qv = weight_q(v);
          const double r = fmax(weight_p(v) * sp - qv * sq, 0.0);
          const double keep = (valid && v == x) ? 0.0 : qv;
          wp[v] = r;
          wq[v] = keep;
          z += r;
          s += keep;
        }
        z = wg_sum(z, sh_d);
        s = wg_sum(s, sh_d);
        if (z > 0.0) {
          sp = 1.0 / z;
        } else {                               // p = q exactly: p is kept
          for (int v = tid; v < V; v += kDraftThreads) wp[v] = weight_p(v);
        }
        sq = s > 0.0 ? 1.0 / s : sq;
        filled = true;
        __syncthreads();
        continue;
      }
      // One pass (a workgroup streams its rows at the rate of one compute unit, so passes are what a
      // rejection costs): the residual goes to the spare buffer while its sum forms, and what q keeps
      // once x is gone is summed from the entries alongside (a difference of the old sum and wq[x]
      // would cancel when the drafter was nearly certain of x).
      __syncthreads();                       // every thread has read wp[x], wq[x]
      double z = 0.0, s = 0.0;
      for (int v = tid; v < V; v += kDraftThreads) {
        const double qv = wq[v];
        const double r = fmax(wp[v] * sp - qv * sq, 0.0);
        wp_spare[v] = r;
        z += r;
        s += (valid && v == x) ? 0.0 : qv;
      }
      z = wg_sum(z, sh_d);
      s = wg_sum(s, sh_d);                   // (its barriers: every thread is done with the old wq[x])
      if (z > 0.0) {                         // else p = q exactly: p is kept
        double* const tmp = wp; wp = wp_spare; wp_spare = tmp;
        sp = 1.0 / z;
      }
      if (valid && tid == 0) wq[x] = 0.0;
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

    if (!filled) fill_p();
    // no child accepted: inverse-CDF draw from the current p. Wavefront w owns the contiguous range
    // [w * per_wave, (w + 1) * per_wave) and walks it in chunks of 64 consecutive entries (one per
    // lane: the loads are contiguous), summing chunk totals in chunk order; the same chunk totals, in
    // the same order, locate the crossing afterwards.
    const int lane = tid & 63, wave = tid >> 6;
    const int per_wave = (V + kDraftThreads - 1) / kDraftThreads * 64;
    const int w0 = wave * per_wave, w1 = min(V, w0 + per_wave);
    auto chunk_total = [&](double x) {
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
      return x;
    };
    double mine = 0.0;
    for (int c0 = w0; c0 < w1; c0 += 64) mine += chunk_total(c0 + lane < w1 ? wp[c0 + lane] : 0.0);
    __syncthreads();                  // sh_d may still be read from the last reduction
    if (lane == 0) sh_d[wave] = mine;
    if (tid == 0) sh_tok = -1;
    __syncthreads();
    double total = 0.0, before = 0.0;
    for (int w = 0; w < kDraftWaves; ++w) {
      if (w == wave) before = total;
      total += sh_d[w];
    }
    const double t = (double)u_draw[cur] * total;
    // the first wavefront whose range brackets t (the same arithmetic in every thread)
    int owner = -1;
    {
      double run = 0.0;
      for (int w = 0; w < kDraftWaves && owner < 0; ++w) {
        run += sh_d[w];
        if (run > t) owner = w;
      }
    }
    if (wave == owner) {
      double run = before;
      int tok = -1;
      for (int c0 = w0; c0 < w1 && tok < 0; c0 += 64) {
        const double x = c0 + lane < w1 ? wp[c0 + lane] : 0.0;
        const double tot = chunk_total(x);
        if (run + tot > t) {
          double incl = x;            // running sum inside the chunk, lane order
#pragma unroll
          for (int off = 1; off < 64; off <<= 1) {
            const double up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
          }
          const unsigned long long hit = __ballot(run + incl > t && x > 0.0);
          const unsigned long long mass = __ballot(x > 0.0);
          // (the chunk's total and its lane-order running sum are formed in different orders: if the
          // running sum falls short by rounding, the chunk's last entry with mass)
          tok = c0 + (hit ? __ffsll(hit) - 1 : 63 - __clzll(mass));
        }
        run += tot;
      }
      if (tok < 0) {   // the range's total said "here", its chunk-by-chunk sum fell short: its last entry with mass
        int last = -1;
        for (int c0 = w0; c0 < w1; c0 += 64)
          if (c0 + lane < w1 && wp[c0 + lane] > 0.0) last = c0 + lane;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) last = max(last, __shfl_xor(last, off));
        tok = last;
      }
      if (lane == 0) sh_tok = tok;
    }
    __syncthreads();
    if (sh_tok < 0) {   // no mass at all, or rounding left no crossing: the last entry with mass (0 if none)
      int last = -1;
      for (int c0 = w0; c0 < w1; c0 += 64)
        if (c0 + lane < w1 && wp[c0 + lane] > 0.0) last = c0 + lane;
      if (tid == 0) sh_last = -1;
      __syncthreads();
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) last = max(last, __shfl_xor(last, off));
      if (lane == 0 && last >= 0) atomicMax(&sh_last, last);   // the highest such entry over the workgroup (one lane a wavefront)
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


// ------------------------------------------------------------------------------------------------
// The same acceptance spread over the chip. With one workgroup per sequence every rejection is a
// pass over two rows of V fp64 entries at the rate of one compute unit. Here G workgroups share a
// sequence: each thread keeps E consecutive entries of the unnormalised p and q of the current node
// in registers, a rejection is arithmetic on registers plus one barrier across the G workgroups
// (partial sums and the two entries the next test needs go through memory), and the draw is located
// from the workgroups' totals. Every workgroup takes every decision from the same published numbers,
// summed in the same order, so the control flow is the same in all of them.
//
// The barrier counts arrivals in a word that the streaming pass of the same call has set to zero;
// the kernel is launched as a cooperative grid (all workgroups resident). A wait is bounded all the
// same: a workgroup that sees no progress for kSpinLimit polls raises the sequence's failure word,
// reports path_len = n_tokens = -1 and leaves, and so does every other workgroup at its next wait.
constexpr int kGridThreads = 256;
constexpr int kGridWaves = kGridThreads / 64;
constexpr int kGridMaxWgs = 64;          // workgroups per sequence, at most
constexpr unsigned kSpinLimit = 1u << 20;

struct DraftGridParams {
  const float* logits;
  const float* draft_logits;
  int64_t row_stride;
  const int32_t* draft_tokens;
  const int32_t* parent;
  const int32_t* n_nodes;
  const float* uniforms;
  int32_t* path;
  int32_t* path_len;
  int32_t* tokens;
  int32_t* n_tokens;
  const float* part_max_p;
  const double* part_sum_p;
  const float* part_max_q;
  const double* part_sum_q;
  uint32_t* sync;      // [B][2]: arrivals, failure word
  double* slots;       // [B][2][G][4]: per round parity and workgroup: sum of the new p, of what q keeps, of the old p
  double* pubs;        // [B][2][4]: the next test's entry of the new p, of the old p, of q
  double* row_stats;   // [2][B*Nmax][2]: (max, sum of exponentials) of every row of logits, then of draft_logits
  double inv_temperature;
  int32_t B, Nmax, V, n_chunks, G;
};

__device__ __forceinline__ double grid_wg_sum(double v, double* sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  __syncthreads();                  // sh may still be read from the previous reduction
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

// K sums over the workgroup at once: running sums inside the wavefronts (no LDS), the four totals of each
// through LDS, one barrier. `sh` holds two sets of K x 4 doubles used in turn, so that a wavefront that
// runs ahead into the next call writes the other set.
template <int K>
__device__ __forceinline__ void grid_wg_sums(double (&v)[K], double* sh, int& flip) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  double* const buf = sh + flip * (K * kGridWaves);
  flip ^= 1;
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const double run = wave_running_sum(v[k]);
    if (lane == 63) buf[k * kGridWaves + wave] = run;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < K; ++k)
    v[k] = (buf[k * kGridWaves] + buf[k * kGridWaves + 1]) + (buf[k * kGridWaves + 2] + buf[k * kGridWaves + 3]);
}

__device__ __forceinline__ float grid_wg_max(float v, float* sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
}

// All G workgroups of a sequence meet; what each wrote before is visible to all after. False: the wait ran out.
__device__ __forceinline__ bool grid_barrier(uint32_t* sync, unsigned target, int* sh_ok) {
  __syncthreads();
  if (threadIdx.x == 0) {
    __threadfence();
    __hip_atomic_fetch_add(&sync[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned polls = 0;
    int ok = 1;
    while (__hip_atomic_load(&sync[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
      if (__hip_atomic_load(&sync[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u || ++polls > kSpinLimit) {
        __hip_atomic_store(&sync[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ok = 0;
        break;
      }
      __builtin_amdgcn_s_sleep(4);
    }
    __threadfence();
    *sh_ok = ok;
  }
  __syncthreads();
  return *sh_ok != 0;
}

// Row statistics of both logit arrays from the chunk statistics of the streaming pass, for every row at once
// (one workgroup per row and array): the walk then finds a node's (max, sum) ready instead of merging them,
// node after node, on its critical path.
__global__ __launch_bounds__(kGridThreads) void accept_row_merge_kernel(const DraftGridParams p) {
  __shared__ double sh_sums[2 * kGridWaves];
  __shared__ float sh_f[kGridWaves];
  const int row = blockIdx.x, arr = blockIdx.y, tid = threadIdx.x;
  const int b = row / p.Nmax, node = row - b * p.Nmax;
  if (node >= p.n_nodes[b]) return;   // rows of unused tree slots have no chunk statistics
  const float* pm = (arr ? p.part_max_q : p.part_max_p) + (int64_t)row * p.n_chunks;
  const double* ps = (arr ? p.part_sum_q : p.part_sum_p) + (int64_t)row * p.n_chunks;
  float m = -INFINITY;
  for (int c = tid; c < p.n_chunks; c += kGridThreads) m = fmaxf(m, pm[c]);
  m = grid_wg_max(m, sh_f);
  double z[1] = {0.0};
  for (int c = tid; c < p.n_chunks; c += kGridThreads) {
    const float mc = pm[c];
    if (mc > -INFINITY) z[0] += ps[c] * exp_nonpos(((double)mc - (double)m) * p.inv_temperature);
  }
  int flip = 0;
  grid_wg_sums<1>(z, sh_sums, flip);
  if (tid == 0) {
    double* out = p.row_stats + ((int64_t)arr * p.B * p.Nmax + row) * 2;
    out[0] = (double)m;
    out[1] = z[0];
  }
}

template <int E>
__global__ __launch_bounds__(kGridThreads) void accept_sample_draft_grid_kernel(const DraftGridParams p) {
  __shared__ double sh_d[kGridWaves];
  __shared__ double sh_sums[2 * 3 * kGridWaves];
  __shared__ float sh_f[kGridWaves];
  __shared__ int sh_ok;
  __shared__ int sh_w[2 * kGridWaves];
  __shared__ double sh_tot[2];
  int flip = 0;
  const int g = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int G = p.G, V = p.V;
  const int64_t o = (int64_t)b * p.Nmax;
  const int n = min(p.n_nodes[b], p.Nmax);
  const float* u_acc = p.uniforms + (int64_t)b * 2 * p.Nmax;
  const float* u_draw = u_acc + p.Nmax;
  uint32_t* sync = p.sync + 2 * b;
  double* slots = p.slots + (int64_t)b * 2 * G * 4;
  double* pubs = p.pubs + (int64_t)b * 2 * 4;
  const int e0 = (g * kGridThreads + tid) * E;   // this thread's E consecutive entries

  if (g == 0)
    for (int i = tid; i < p.Nmax; i += kGridThreads) { p.path[o + i] = i == 0 ? 0 : -1; p.tokens[o + i] = -1; }
  // the tree and the uniforms go to LDS once: the walk reads them in loops
  __shared__ int t_par[FSPAD_MAX_NODES], t_tok[FSPAD_MAX_NODES];
  __shared__ float t_ua[FSPAD_MAX_NODES], t_ud[FSPAD_MAX_NODES];
  __shared__ double t_stats[2][FSPAD_MAX_NODES][2];   // (max, sum) of every row of this sequence: logits, draft logits
  for (int i = tid; i < 4 * p.Nmax; i += kGridThreads) {
    const int arr = i / (2 * p.Nmax), rest = i - arr * 2 * p.Nmax;
    t_stats[arr][rest >> 1][rest & 1] = p.row_stats[((int64_t)arr * p.B * p.Nmax + o) * 2 + rest];
  }
  if (tid < FSPAD_MAX_NODES) {
    const bool ok = tid < p.Nmax;
    t_par[tid] = ok ? p.parent[o + tid] : -2;
    t_tok[tid] = ok ? p.draft_tokens[o + tid] : -1;
    t_ua[tid] = ok ? u_acc[tid] : 0.f;
    t_ud[tid] = ok ? u_draw[tid] : 0.f;
  }
  __syncthreads();

  double rp[E], rq[E];   // unnormalised p and q of the current node, once a rejection or the draw has formed them
  unsigned round = 0;
  auto meet = [&]() {
    ++round;
    if (grid_barrier(sync, round * (unsigned)G, &sh_ok)) return true;
    if (tid == 0) { p.path_len[b] = -1; p.n_tokens[b] = -1; }
    return false;
  };

  int cur = 0, len = 1;
  for (;;) {
    const float* lrow = p.logits + (o + cur) * p.row_stride;
    const float* qrow = p.draft_logits + (o + cur) * p.row_stride;
    // (rows of nodes beyond the tree are never walked: their entries hold no statistics)
    const double mp = t_stats[0][cur][0], zp = t_stats[0][cur][1], mq = t_stats[1][cur][0], zq = t_stats[1][cur][1];
    double sp = zp > 0.0 ? 1.0 / zp : 0.0, sq = zq > 0.0 ? 1.0 / zq : 0.0;
    auto weight_p = [&](int v) {
      const float a = lrow[v];
      return (a == a && mp > -INFINITY) ? exp_nonpos(((double)a - (double)mp) * p.inv_temperature) : 0.0;
    };
    auto weight_q = [&](int v) {
      const float c = qrow[v];
      return (c == c && mq > -INFINITY) ? exp_nonpos(((double)c - (double)mq) * p.inv_temperature) : 0.0;
    };

    bool filled = false;
    int total_at = 2;             // which slot entry holds the workgroups' totals of the p in the registers
    double pub_p = 0.0, pub_q = 0.0;   // the entries of p and q for the child under test, once filled
    int next = -1;
    for (int c = cur + 1; c < n && len < p.Nmax; ++c) {
      if (t_par[c] != cur) continue;
      const int x = t_tok[c];
      const bool valid = x >= 0 && x < V;
      double px = 0.0, qx = 0.0;
      if (valid && filled) {
        px = pub_p * sp; qx = pub_q * sq;
      } else if (valid) {
        const float a = lrow[x], d = qrow[x];
        px = (a == a && mp > -INFINITY) ? exp_nonpos(((double)a - (double)mp) * p.inv_temperature) * sp : 0.0;
        qx = (d == d && mq > -INFINITY) ? exp_nonpos(((double)d - (double)mq) * p.inv_temperature) * sq : 0.0;
      }
      if ((double)t_ua[c] * qx < px) { next = c; break; }
      // rejected: p <- max(p - q, 0), renormalised; q loses x and is renormalised. The sibling tested
      // next (if any) needs its entries of the new p and q: their owner publishes them in the same round.
      int x2 = -1;
      for (int c2 = c + 1; c2 < n; ++c2)
        if (t_par[c2] == cur) { x2 = t_tok[c2]; break; }
      const unsigned buf = (round + 1u) & 1u;
      double rn[E];
      double z = 0.0, s = 0.0, told = 0.0;
#pragma unroll
      for (int j = 0; j < E; ++j) {
        const int v = e0 + j;
        double qv, pold, r;
        if (!filled) {
          qv = v < V ? weight_q(v) : 0.0;
          pold = v < V ? weight_p(v) : 0.0;
        } else {
          qv = rq[j];
          pold = rp[j];
        }
        r = fmax(pold * sp - qv * sq, 0.0);
        const double keep = (valid && v == x) ? 0.0 : qv;
        rn[j] = r; rp[j] = pold; rq[j] = keep;
        z += r; s += keep; told += pold;
        if (v == x2 && v < V) { pubs[buf * 4 + 0] = r; pubs[buf * 4 + 1] = pold; pubs[buf * 4 + 2] = keep; }
      }
      {
        double three[3] = {z, s, told};
        grid_wg_sums<3>(three, sh_sums, flip);
        z = three[0]; s = three[1]; told = three[2];
      }
      if (tid == 0) {
        double* mine = slots + ((int64_t)buf * G + g) * 4;
        mine[0] = z; mine[1] = s; mine[2] = told;
      }
      if (!meet()) return;
      // (every load of the round goes out before the first is used: one trip to memory, not three)
      const double* sl = slots + (int64_t)(round & 1u) * G * 4;
      const double part_z = tid < G ? sl[tid * 4] : 0.0, part_s = tid < G ? sl[tid * 4 + 1] : 0.0;
      const double pub_new = pubs[(round & 1u) * 4], pub_old = pubs[(round & 1u) * 4 + 1], pub_keep = pubs[(round & 1u) * 4 + 2];
      double both[2] = {part_z, part_s};
      grid_wg_sums<2>(both, sh_sums, flip);
      const double Z = both[0], S = both[1];
      const bool moved = Z > 0.0;            // else p = q exactly: p is kept
      if (moved) {
#pragma unroll
        for (int j = 0; j < E; ++j) rp[j] = rn[j];
        sp = 1.0 / Z;
      }
      total_at = moved ? 0 : 2;
      sq = S > 0.0 ? 1.0 / S : sq;
      filled = true;
      pub_p = moved ? pub_new : pub_old;
      pub_q = pub_keep;
    }
    if (next >= 0) {
      if (g == 0 && tid == 0) { p.tokens[o + len - 1] = t_tok[next]; p.path[o + len] = next; }
      ++len;
      cur = next;
      continue;
    }

    // no child accepted: inverse-CDF draw from the current p, located from the workgroups' totals
    if (!filled) {
      double told = 0.0;
#pragma unroll
      for (int j = 0; j < E; ++j) {
        rp[j] = e0 + j < V ? weight_p(e0 + j) : 0.0;
        told += rp[j];
      }
      told = grid_wg_sum(told, sh_d);
      if (tid == 0) slots[((int64_t)((round + 1u) & 1u) * G + g) * 4 + 2] = told;
      if (!meet()) return;
      total_at = 2;
    }
    // wavefront 0, one lane per workgroup (G <= 64): running sum of the totals, first workgroup above t
    static_assert(kGridMaxWgs <= 64, "one lane per workgroup");
    if (wave == 0) {
      const double mine = lane < G ? slots[((int64_t)(round & 1u) * G + lane) * 4 + total_at] : 0.0;
      const double incl = wave_running_sum(mine);
      const double total = __shfl(incl, 63);
      const double t = (double)t_ud[cur] * total;
      const unsigned long long mass = __ballot(mine > 0.0), hit = __ballot(mine > 0.0 && incl > t);
      const int first = hit ? __ffsll(hit) - 1 : (mass ? 63 - __clzll(mass) : -1);
      // (no crossing by rounding: the last workgroup with mass, to its last entry with mass)
      const double left = hit ? t - (__shfl(incl, first < 0 ? 0 : first) - __shfl(mine, first < 0 ? 0 : first)) : INFINITY;
      if (lane == 0) { sh_w[0] = first; sh_tot[0] = left; }
    }
    __syncthreads();
    const int owner = sh_w[0];
    const double target = sh_tot[0];
    __syncthreads();   // sh_w is written again below
    if (owner < 0) {                                            // no mass at all: token 0
      if (g == 0 && tid == 0) { p.tokens[o + len - 1] = 0; p.path_len[b] = len; p.n_tokens[b] = len; }
      return;
    }
    if (g != owner) return;
    double local = 0.0;
    int last_here = -1;
#pragma unroll
    for (int j = 0; j < E; ++j) {
      local += rp[j];
      if (rp[j] > 0.0) last_here = e0 + j;
    }
    const double incl = wave_running_sum(local);
    __syncthreads();
    if (lane == 63) sh_d[wave] = incl;
    __syncthreads();
    double wave_base = 0.0;
#pragma unroll
    for (int w = 0; w < kGridWaves; ++w) {
      const double part = sh_d[w];
      if (w < wave) wave_base += part;
    }
    const double inclusive = wave_base + incl;
    const unsigned long long hits = __ballot(inclusive > target && local > 0.0);
    int last_wave = last_here;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) last_wave = max(last_wave, __shfl_xor(last_wave, off));
    if (lane == 0) {
      sh_w[wave] = hits ? wave * 64 + (__ffsll(hits) - 1) : kNone;
      sh_w[kGridWaves + wave] = last_wave;
    }
    __syncthreads();
    int first_thread = kNone, last_any = -1;
#pragma unroll
    for (int w = 0; w < kGridWaves; ++w) {
      first_thread = min(first_thread, sh_w[w]);
      last_any = max(last_any, sh_w[kGridWaves + w]);
    }
    if (first_thread == kNone) {
      if (tid == 0) { p.tokens[o + len - 1] = last_any < 0 ? 0 : last_any; p.path_len[b] = len; p.n_tokens[b] = len; }
      return;
    }
    if (tid == first_thread) {
      double run = inclusive - local;
      int pick = last_here;
      bool done = false;
#pragma unroll
      for (int j = 0; j < E; ++j) {
        run += rp[j];
        if (!done && run > target && rp[j] > 0.0) { pick = e0 + j; done = true; }
      }
      p.tokens[o + len - 1] = pick;
      p.path_len[b] = len;
      p.n_tokens[b] = len;
    }
    return;
  }
}

struct GridPlan { int G, E; size_t slots_at, pubs_at, stats_at; };
// E = 0: the chip-wide form does not apply (too many sequences, a vocabulary beyond 64 x 256 x 32 entries or too
// small to hold the exchange area in the workspace's row buffers, or no cooperative launch on this device).
GridPlan plan_draft_grid(int32_t B, int32_t Nmax, int32_t V) {
  GridPlan pl{0, 0, 0, 0, 0};
  if (B > 256) return pl;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    (void)hipGetLastError();
    return pl;
  }
  static std::atomic<int> coop_known[64];   // 0: not asked yet, 1: no, 2: yes (asked once per device)
  int known = coop_known[dev].load(std::memory_order_relaxed);
  if (known == 0) {
    int coop = 0;
    if (hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess) {
      (void)hipGetLastError();
      coop = 0;
    }
    known = coop ? 2 : 1;
    coop_known[dev].store(known, std::memory_order_relaxed);
  }
  if (known != 2) return pl;
  const int max_g = std::min(kGridMaxWgs, 256 / B);
  const int64_t per = ((int64_t)V + (int64_t)max_g * kGridThreads - 1) / ((int64_t)max_g * kGridThreads);
  const int E = per <= 4 ? 4 : per <= 8 ? 8 : per <= 16 ? 16 : per <= 32 ? 32 : 0;
  if (E == 0) return pl;
  const int G = (int)(((int64_t)V + (int64_t)kGridThreads * E - 1) / ((int64_t)kGridThreads * E));
  const size_t slots_at = ((size_t)B * 2 * sizeof(uint32_t) + 255) & ~(size_t)255;
  const size_t pubs_at = slots_at + (size_t)B * 2 * G * 4 * sizeof(double);
  const size_t stats_at = pubs_at + (size_t)B * 2 * 4 * sizeof(double);
  const size_t end = stats_at + (size_t)2 * B * Nmax * 2 * sizeof(double);
  if (end > (size_t)B * 3 * (size_t)V * 8) return pl;
  pl.G = G; pl.E = E; pl.slots_at = slots_at; pl.pubs_at = pubs_at; pl.stats_at = stats_at;
  return pl;
}

}  // namespace

extern "C" size_t fspad_tree_accept_workspace_bytes(int32_t B, int32_t Nmax, int32_t V) {
  if (B < 1 || Nmax < 1 || V < 1) return 0;
  const size_t slots = (size_t)B * Nmax * ((V + kMinChunk - 1) / kMinChunk);  // room for the finest split
  return (slots * 16 + 255) & ~(size_t)255;
}

extern "C" fspad_status fspad_tree_accept_greedy(int32_t B, int32_t Nmax, int32_t V, const float* logits,
                                                 int64_t row_stride, const int32_t* draft_tokens,
                                                 const int32_t* parent, const int32_t* n_nodes, int32_t* path,
                                                 int32_t* path_len, int32_t* tokens, int32_t* n_tokens,
                                                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  const fspad_status st = check_accept_args(B, Nmax, V, logits, row_stride, draft_tokens, parent, n_nodes, path,
                                            path_len, tokens, n_tokens, workspace, workspace_bytes);
  if (st != FSPAD_OK) return st;
  AcceptParams p{};
  fill_params(p, B, Nmax, V, logits, row_stride, draft_tokens, parent, n_nodes, path, path_len, tokens, n_tokens, workspace);
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  launch_rows<0>(p, rows_vectorisable(logits, row_stride), stream);
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  hipLaunchKernelGGL(accept_greedy_walk_kernel, dim3((unsigned)B), dim3(kThreads), 0, stream, p);
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  return FSPAD_OK;
}

// ------------------------------------------------------------------------------------------------
// The greedy acceptance for callers that cannot allocate: the chunk statistics live in a fixed
// device array of the library image. In host code the array's name is only a handle: its device
// address is looked up once per device (with that device current) and kept; the kernels get that
// address exactly as they get a caller's workspace.
namespace {
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[FSPAD_STATIC_SCRATCH_BYTES];
namespace {
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, nullptr until looked up

// Device address of the static array on the current device, or nullptr.
void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" fspad_status fspad_tree_accept_greedy_static(int32_t B, int32_t Nmax, int32_t V, const float* logits,
                                                        int64_t row_stride, const int32_t* draft_tokens,
                                                        const int32_t* parent, const int32_t* n_nodes, int32_t* path,
                                                        int32_t* path_len, int32_t* tokens, int32_t* n_tokens,
                                                        void* hip_stream) {
  if (!logits || !draft_tokens || !parent || !n_nodes || !path || !path_len || !tokens || !n_tokens) return FSPAD_ERR_NULL;
  if (B < 1 || Nmax < 1 || Nmax > FSPAD_MAX_NODES || V < 1 || V > (1 << 30)) return FSPAD_ERR_SHAPE;
  const size_t need = fspad_tree_accept_workspace_bytes(B, Nmax, V);
  if (need == 0 || need > FSPAD_STATIC_SCRATCH_BYTES) return FSPAD_ERR_WORKSPACE;  // beyond the fixed array
  void* ptr = static_scratch();
  if (!ptr) return FSPAD_ERR_HIP;
  // every slot the walk reads is written by the row pass of the same call: nothing to clear
  return fspad_tree_accept_greedy(B, Nmax, V, logits, row_stride, draft_tokens, parent, n_nodes, path, path_len, tokens,
                                  n_tokens, ptr, FSPAD_STATIC_SCRATCH_BYTES, hip_stream);
}

extern "C" fspad_status fspad_tree_accept_sample(int32_t B, int32_t Nmax, int32_t V, const float* logits,
                                                 int64_t row_stride, const int32_t* draft_tokens,
                                                 const int32_t* parent, const int32_t* n_nodes, float temperature,
                                                 const float* uniforms, int32_t* path, int32_t* path_len,
                                                 int32_t* tokens, int32_t* n_tokens, void* workspace,
                                                 size_t workspace_bytes, void* hip_stream) {
  if (!(temperature > 0.0f) || temperature > 3.0e38f) return FSPAD_ERR_TEMPERATURE;
  if (!uniforms) return FSPAD_ERR_NULL;
  const fspad_status st = check_accept_args(B, Nmax, V, logits, row_stride, draft_tokens, parent, n_nodes, path,
                                            path_len, tokens, n_tokens, workspace, workspace_bytes);
  if (st != FSPAD_OK) return st;
  AcceptParams p{};
  fill_params(p, B, Nmax, V, logits, row_stride, draft_tokens, parent, n_nodes, path, path_len, tokens, n_tokens, workspace);
  p.uniforms = uniforms;
  p.inv_temperature = 1.0 / (double)temperature;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  launch_rows<1>(p, rows_vectorisable(logits, row_stride), stream);
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  hipLaunchKernelGGL(accept_sample_walk_kernel, dim3((unsigned)B), dim3(kWalkThreads), 0, stream, p);
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  return FSPAD_OK;
}

extern "C" size_t fspad_tree_accept_sample_draft_workspace_bytes(int32_t B, int32_t Nmax, int32_t V) {
  if (B < 1 || Nmax < 1 || V < 1) return 0;
  // chunk statistics of both logit arrays, then 3 V fp64 entries per sequence
  return 2 * fspad_tree_accept_workspace_bytes(B, Nmax, V) + (((size_t)B * 3 * (size_t)V * 8 + 255) & ~(size_t)255);
}

extern "C" fspad_status fspad_tree_accept_sample_draft(int32_t B, int32_t Nmax, int32_t V, const float* logits,
                                                       const float* draft_logits, int64_t row_stride,
                                                       const int32_t* draft_tokens, const int32_t* parent,
                                                       const int32_t* n_nodes, float temperature, const float* uniforms,
                                                       int32_t* path, int32_t* path_len, int32_t* tokens,
                                                       int32_t* n_tokens, void* workspace, size_t workspace_bytes,
                                                       void* hip_stream) {
  if (!draft_logits || !uniforms) return FSPAD_ERR_NULL;
  if (((uintptr_t)draft_logits) & 3) return FSPAD_ERR_SHAPE;
  const size_t need = fspad_tree_accept_sample_draft_workspace_bytes(B, Nmax, V);
  const fspad_status st = check_accept_args(B, Nmax, V, logits, row_stride, draft_tokens, parent, n_nodes, path, path_len,
                                            tokens, n_tokens, workspace, workspace_bytes >= need ? workspace_bytes : 0);
  if (st != FSPAD_OK) return st;
  if (!(temperature > 0.0f) || temperature > 3.0e38f) return FSPAD_ERR_TEMPERATURE;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const size_t region = fspad_tree_accept_workspace_bytes(B, Nmax, V);
  char* ws = static_cast<char*>(workspace);
  AcceptParams pa{}, pb{};
  fill_params(pa, B, Nmax, V, logits, row_stride, draft_tokens, parent, n_nodes, path, path_len, tokens, n_tokens, ws);
  fill_params(pb, B, Nmax, V, draft_logits, row_stride, draft_tokens, parent, n_nodes, path, path_len, tokens, n_tokens,
              ws + region);
  pa.inv_temperature = pb.inv_temperature = 1.0 / (double)temperature;
  // Chip-wide form: G workgroups a sequence, E entries a thread, if the shape allows it and the device
  // runs cooperative grids; else one workgroup a sequence.
  const GridPlan plan = plan_draft_grid(B, Nmax, V);
  char* const work = ws + 2 * region;
  if (plan.E != 0) {
    pb.clear_words = reinterpret_cast<uint32_t*>(work);
    pb.clear_count = 2 * B;
  }
  // one streaming launch over both logit arrays (grid.z picks the array)
  AcceptParams both = pa;
  both.logits2 = draft_logits; both.part_max2 = pb.part_max; both.part_sum2 = pb.part_sum;
  both.clear_words = pb.clear_words; both.clear_count = pb.clear_count;
  launch_rows<1>(both, rows_vectorisable(logits, row_stride) && rows_vectorisable(draft_logits, row_stride), stream);
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  if (plan.E != 0) {
    DraftGridParams gp{};
    gp.logits = logits; gp.draft_logits = draft_logits; gp.row_stride = row_stride;
    gp.draft_tokens = draft_tokens; gp.parent = parent; gp.n_nodes = n_nodes; gp.uniforms = uniforms;
    gp.path = path; gp.path_len = path_len; gp.tokens = tokens; gp.n_tokens = n_tokens;
    gp.part_max_p = pa.part_max; gp.part_sum_p = pa.part_sum; gp.part_max_q = pb.part_max; gp.part_sum_q = pb.part_sum;
    gp.sync = reinterpret_cast<uint32_t*>(work);
    gp.slots = reinterpret_cast<double*>(work + plan.slots_at);
    gp.pubs = reinterpret_cast<double*>(work + plan.pubs_at);
    gp.row_stats = reinterpret_cast<double*>(work + plan.stats_at);
    gp.inv_temperature = pa.inv_temperature;
    gp.B = B; gp.Nmax = Nmax; gp.V = V; gp.n_chunks = pa.n_chunks; gp.G = plan.G;
    hipLaunchKernelGGL(accept_row_merge_kernel, dim3((unsigned)(B * Nmax), 2u), dim3(kGridThreads), 0, stream, gp);
    if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
    void* args[] = {&gp};
    const dim3 grid((unsigned)plan.G, (unsigned)B), block(kGridThreads);
    hipError_t err = hipErrorInvalidValue;
    switch (plan.E) {
      case 4: err = hipLaunchCooperativeKernel(reinterpret_cast<const void*>(&accept_sample_draft_grid_kernel<4>), grid, block, args, 0, stream); break;
      case 8: err = hipLaunchCooperativeKernel(reinterpret_cast<const void*>(&accept_sample_draft_grid_kernel<8>), grid, block, args, 0, stream); break;
      case 16: err = hipLaunchCooperativeKernel(reinterpret_cast<const void*>(&accept_sample_draft_grid_kernel<16>), grid, block, args, 0, stream); break;
      case 32: err = hipLaunchCooperativeKernel(reinterpret_cast<const void*>(&accept_sample_draft_grid_kernel<32>), grid, block, args, 0, stream); break;
    }
    if (err == hipSuccess) return FSPAD_OK;
    (void)hipGetLastError();   // the launch was refused (a capture in progress, say): the one-workgroup form below
  }
  DraftAcceptParams p{};
  p.logits = logits; p.draft_logits = draft_logits; p.row_stride = row_stride;
  p.draft_tokens = draft_tokens; p.parent = parent; p.n_nodes = n_nodes; p.uniforms = uniforms;
  p.path = path; p.path_len = path_len; p.tokens = tokens; p.n_tokens = n_tokens;
  p.work = reinterpret_cast<double*>(ws + 2 * region);
  p.part_max_p = pa.part_max; p.part_sum_p = pa.part_sum; p.part_max_q = pb.part_max; p.part_sum_q = pb.part_sum;
  p.inv_temperature = pa.inv_temperature;
  p.B = B; p.Nmax = Nmax; p.V = V; p.n_chunks = pa.n_chunks;
  hipLaunchKernelGGL(accept_sample_draft_kernel, dim3((unsigned)B), dim3(kDraftThreads), 0, stream, p);
  return hipGetLastError() == hipSuccess ? FSPAD_OK : FSPAD_ERR_HIP;
}
