// Top-k cut of a draft step's output (arXiv 2408.15562, Preliminaries, last paragraph: the output
// of every draft step is cut to its k most probable tokens; their probabilities feed the joint
// scores from which the tree is chosen). Per row of logits: the k largest entries, best first
// (equal logits: lower token first; NaN counts as -infinity), and their log-softmax values.
// gfx950 (CDNA4) only.
//
// Two kernels. The first, one workgroup per (chunk of 1024..8192 logits, row), reads its chunk once
// (16 bytes per lane), keeps it in registers as order-preserving integer keys, and leaves the
// chunk's maximum, its sum of exponentials and its own k best entries. The second, one workgroup
// per row, picks the k best of the chunks' candidates and turns them into log-probabilities.
// "k best" is k rounds of a workgroup-wide maximum over packed (key, ~token) words: a thread
// re-scans its registers only when it owned the winner.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "fspad.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMinChunk = 1024, kMaxChunk = 8192;
constexpr int kMergePerThread = 8;   // candidates per thread of the merge kernel: 2048 in all

struct TopkParams {
  const float* logits;
  int64_t row_stride;
  int32_t* tokens;        // [rows][k]
  float* logp;            // [rows][k]
  unsigned long long* cand;  // [rows][n_chunks][k] packed (key << 32 | ~token), 0 = none
  float* chunk_max;       // [rows][n_chunks]
  double* chunk_sum;      // [rows][n_chunks]  sum of exp(l - chunk_max)
  int32_t rows, V, k, n_chunks, chunk;
};

// float -> unsigned key with the same order; NaN ranks with -infinity, -0 with +0; key 0 is
// reserved for "no entry" (smaller than the key of -infinity)
__device__ __forceinline__ unsigned key_of(float x) {
  x = (x != x) ? -INFINITY : x + 0.0f;
  const unsigned u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float value_of(unsigned key) {
  return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}
__device__ __forceinline__ unsigned long long pack(unsigned key, int token) {
  return ((unsigned long long)key << 32) | (unsigned)(0xffffffffu - (unsigned)token);
}
__device__ __forceinline__ int token_of(unsigned long long w) { return (int)(0xffffffffu - (unsigned)w); }

// One step of a maximum over lanes with a data-parallel-primitive lane pattern (no LDS round trip)
template <int CTRL>
__device__ __forceinline__ unsigned long long dpp_max_u64(unsigned long long x) {
  const int lo = (int)(unsigned)x, hi = (int)(unsigned)(x >> 32);
  const unsigned olo = (unsigned)__builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xf, 0xf, false);
  const unsigned ohi = (unsigned)__builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xf, 0xf, false);
  const unsigned long long o = ((unsigned long long)ohi << 32) | olo;
  return o > x ? o : x;
}

// Maximum over the 64 lanes, the same value in every lane: neighbours, pairs, mirrored halves of
// eight and of sixteen lanes (after which a row of 16 agrees), then the four rows through scalars.
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long x) {
  x = dpp_max_u64<0xB1>(x);    // quad_perm [1,0,3,2]
  x = dpp_max_u64<0x4E>(x);    // quad_perm [2,3,0,1]
  x = dpp_max_u64<0x141>(x);   // row_half_mirror
  x = dpp_max_u64<0x140>(x);   // row_mirror
  unsigned long long m = 0ull;
#pragma unroll
  for (int row = 0; row < 4; ++row) {
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)x, 16 * row);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(x >> 32), 16 * row);
    const unsigned long long o = ((unsigned long long)hi << 32) | lo;
    m = o > m ? o : m;
  }
  return m;
}

// Workgroup-wide maximum of one word per thread; every thread gets it. `slots` is 2 x 4 words of
// LDS, alternated by `round`, so that one barrier per call is enough.
__device__ __forceinline__ unsigned long long block_max_u64(unsigned long long x, unsigned long long* slots, int round) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  x = wave_max_u64(x);
  unsigned long long* s = slots + (round & 1) * 4;
  if (lane == 0) s[wave] = x;
  __syncthreads();
  unsigned long long m = s[0];
#pragma unroll
  for (int w = 1; w < kThreads / 64; ++w) m = s[w] > m ? s[w] : m;
  return m;
}

// PT entries per thread, entry j*4+i of thread t is logit chunk0 + (j*256 + t)*4 + i.
// VEC: rows are 16-byte aligned so that float4 loads are legal.
template <int PT, bool VEC>
__global__ __launch_bounds__(kThreads) void topk_chunk_kernel(const TopkParams p) {
  __shared__ unsigned long long slots[8];
  __shared__ double red_d[kThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = blockIdx.x, row = blockIdx.y;
  const int chunk0 = c * p.chunk;
  const float* src = p.logits + (size_t)row * p.row_stride;

  unsigned key[PT];
#pragma unroll
  for (int j = 0; j < PT / 4; ++j) {
    const int e = chunk0 + (j * kThreads + tid) * 4;
    float v[4];
    if (VEC && e + 3 < p.V) {
      const float4 x = *reinterpret_cast<const float4*>(src + e);
      v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = e + i < p.V ? src[e + i] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) key[j * 4 + i] = e + i < p.V ? key_of(v[i]) : 0u;
  }
  auto token_at = [&](int q) { return chunk0 + ((q >> 2) * kThreads + tid) * 4 + (q & 3); };
  auto local_best = [&] {
    unsigned long long best = 0ull;
#pragma unroll
    for (int q = 0; q < PT; ++q) {
      const unsigned long long w = key[q] ? pack(key[q], token_at(q)) : 0ull;
      best = w > best ? w : best;
    }
    return best;
  };

  // chunk maximum and sum of exponentials (entries past the row end and -infinity add nothing)
  unsigned long long mine = local_best();
  const unsigned long long top = block_max_u64(mine, slots, 1);
  const float cmax = top ? value_of((unsigned)(top >> 32)) : -INFINITY;
  float sum = 0.f;
  if (cmax > -INFINITY) {
#pragma unroll
    for (int q = 0; q < PT; ++q)
      if (key[q]) sum += __expf(value_of(key[q]) - cmax);
  }
  double dsum = sum;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) dsum += __shfl_xor(dsum, d);
  if (lane == 0) red_d[wave] = dsum;

  // k rounds: the workgroup's best entry goes out, its owner strikes it and re-scans
  unsigned long long* out = p.cand + ((size_t)row * p.n_chunks + c) * p.k;
  for (int r = 0; r < p.k; ++r) {
    const unsigned long long win = block_max_u64(mine, slots, r);
    if (tid == 0) out[r] = win;
    if (win != 0ull && win == mine) {
      const int tok = token_of(win);
#pragma unroll
      for (int q = 0; q < PT; ++q)
        if (token_at(q) == tok) key[q] = 0u;
      mine = local_best();
    }
  }
  __syncthreads();
  if (tid == 0) {
    p.chunk_max[(size_t)row * p.n_chunks + c] = cmax;
    p.chunk_sum[(size_t)row * p.n_chunks + c] = red_d[0] + red_d[1] + red_d[2] + red_d[3];
  }
}

__global__ __launch_bounds__(kThreads) void topk_merge_kernel(const TopkParams p) {
  __shared__ unsigned long long slots[8];
  __shared__ double red_d[kThreads / 64];
  __shared__ float red_m[kThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.x;
  const int n_cand = p.n_chunks * p.k;
  const unsigned long long* cand = p.cand + (size_t)row * n_cand;

  unsigned long long mine[kMergePerThread];
#pragma unroll
  for (int q = 0; q < kMergePerThread; ++q) {
    const int i = q * kThreads + tid;
    mine[q] = i < n_cand ? cand[i] : 0ull;
  }
  // row maximum and normaliser from the chunk statistics
  float m = -INFINITY;
  for (int c = tid; c < p.n_chunks; c += kThreads) m = fmaxf(m, p.chunk_max[(size_t)row * p.n_chunks + c]);
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) m = fmaxf(m, __shfl_xor(m, d));
  if (lane == 0) red_m[wave] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));
  double z = 0.0;
  if (m > -INFINITY) {
    for (int c = tid; c < p.n_chunks; c += kThreads) {
      const float cm = p.chunk_max[(size_t)row * p.n_chunks + c];
      if (cm > -INFINITY) z += p.chunk_sum[(size_t)row * p.n_chunks + c] * exp((double)cm - (double)m);
    }
  }
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) z += __shfl_xor(z, d);
  if (lane == 0) red_d[wave] = z;
  __syncthreads();
  z = red_d[0] + red_d[1] + red_d[2] + red_d[3];
  const double lse = (double)m + log(z);

  auto local_best = [&] {
    unsigned long long best = 0ull;
#pragma unroll
    for (int q = 0; q < kMergePerThread; ++q) best = mine[q] > best ? mine[q] : best;
    return best;
  };
  unsigned long long best = local_best();
  for (int r = 0; r < p.k; ++r) {
    const unsigned long long win = block_max_u64(best, slots, r);
    if (tid == 0) {
      // k <= V and every chunk hands in its own k best: a winner exists in every round
      p.tokens[(size_t)row * p.k + r] = win ? token_of(win) : 0;
      const float v = win ? value_of((unsigned)(win >> 32)) : -INFINITY;
      p.logp[(size_t)row * p.k + r] = (m > -INFINITY && v > -INFINITY) ? (float)((double)v - lse) : -INFINITY;
    }
    if (win != 0ull && win == best) {
#pragma unroll
      for (int q = 0; q < kMergePerThread; ++q)
        if (mine[q] == win) mine[q] = 0ull;
      best = local_best();
    }
  }
}

// Largest chunk that still gives a few hundred workgroups, and few enough chunks for the merge kernel
int pick_chunk(int32_t rows, int32_t V, int32_t k) {
  int chunk = kMaxChunk;
  while (chunk > kMinChunk && (int64_t)rows * ((V + chunk - 1) / chunk) < 512) chunk >>= 1;
  while (chunk < kMaxChunk && (int64_t)((V + chunk - 1) / chunk) * k > kMergePerThread * kThreads) chunk <<= 1;
  return chunk;
}

}  // namespace

extern "C" size_t fspad_draft_topk_workspace_bytes(int32_t rows, int32_t V, int32_t k) {
  if (rows < 1 || V < 1 || k < 1 || k > FSPAD_MAX_TOPK) return 0;
  const size_t chunks = (size_t)rows * ((V + kMinChunk - 1) / kMinChunk);   // room for the finest split
  return ((chunks * (8 * (size_t)k + 4 + 8)) + 255 + 16) & ~(size_t)255;
}

extern "C" fspad_status fspad_draft_topk(int32_t rows, int32_t V, int32_t k, const float* logits, int64_t row_stride,
                                         int32_t* tokens, float* logp, void* workspace, size_t workspace_bytes,
                                         void* hip_stream) {
  if (!logits || !tokens || !logp) return FSPAD_ERR_NULL;
  if (rows < 1 || rows > 65535 || V < 1 || V > (1 << 30) || row_stride < V) return FSPAD_ERR_SHAPE;
  if (k < 1 || k > FSPAD_MAX_TOPK || k > V) return FSPAD_ERR_SHAPE;
  if (((uintptr_t)logits) & 3) return FSPAD_ERR_SHAPE;
  if (!workspace || ((uintptr_t)workspace & 15) || workspace_bytes < fspad_draft_topk_workspace_bytes(rows, V, k))
    return FSPAD_ERR_WORKSPACE;
  TopkParams p{};
  p.logits = logits; p.row_stride = row_stride; p.tokens = tokens; p.logp = logp;
  p.rows = rows; p.V = V; p.k = k;
  p.chunk = pick_chunk(rows, V, k);
  p.n_chunks = (V + p.chunk - 1) / p.chunk;
  if ((int64_t)p.n_chunks * k > kMergePerThread * kThreads) return FSPAD_ERR_SHAPE;   // V > 8192 * 2048 / k
  const size_t chunks = (size_t)rows * p.n_chunks;
  p.cand = static_cast<unsigned long long*>(workspace);                       // 8-byte entries first
  p.chunk_sum = reinterpret_cast<double*>(p.cand + chunks * k);
  p.chunk_max = reinterpret_cast<float*>(p.chunk_sum + chunks);
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const bool vec = (((uintptr_t)logits) & 15) == 0 && (row_stride % 4) == 0;
  const dim3 grid((unsigned)p.n_chunks, (unsigned)rows);
#define FSPAD_TOPK(PT)                                                                                  \
  do {                                                                                                    \
    if (vec) hipLaunchKernelGGL((topk_chunk_kernel<PT, true>), grid, dim3(kThreads), 0, stream, p);      \
    else hipLaunchKernelGGL((topk_chunk_kernel<PT, false>), grid, dim3(kThreads), 0, stream, p);         \
  } while (0)
  switch (p.chunk / kThreads) {
    case 4: FSPAD_TOPK(4); break;
    case 8: FSPAD_TOPK(8); break;
    case 16: FSPAD_TOPK(16); break;
    default: FSPAD_TOPK(32); break;
  }
#undef FSPAD_TOPK
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  hipLaunchKernelGGL(topk_merge_kernel, dim3((unsigned)rows), dim3(kThreads), 0, stream, p);
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  return FSPAD_OK;
}
