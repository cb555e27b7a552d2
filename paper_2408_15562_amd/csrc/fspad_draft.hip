// Draft-side forward of the draft model (arXiv 2408.15562, Methodology). gfx950 (CDNA4) only.
//
// 1. The Feature Sampler ("Feature Sampling": an Up Projector for the feature f, a Gate Projector
//    for the token embedding e, SiLU on the lifted embedding, element-wise product with the lifted
//    feature, a Down Projector back to the hidden size, and the feature path's residual connection):
//
//        eta = W_down (SiLU(W_gate e) * (W_up f)) + f
//
// 2. The draft model itself (first paragraph of Methodology: a Transformer Decoder Layer; "Partial
//    Alignment Distillation": the output dimension of its MLP is doubled and both halves share one
//    residual connection, giving the features f~ and f): RMSNorm, fused q / k / v projection with
//    rotary encoding, tree attention over the draft's own cache (the attention entry point of this
//    library), output projection and residual, RMSNorm, gated MLP whose down projection is 2 Hd wide.
//
// Both work on the few rows of one draft step (sequences x tree nodes), so every projection is a
// skinny GEMM bound by streaming its weights once (3 x Hd x I bf16 = 270 MB for the Feature
// Sampler of a 4096 / 11008 model, 494 MB for the decoder layer); they share the streaming core of
// the LM head. A projector has too few 128-row slices of its weight matrix to fill the chip (86 for
// the up / gate projectors, 32 for a 4096-wide output), so every slice is also cut along k:
// workgroup (slice, split) leaves an fp32 partial tile, and a small element-wise kernel sums the
// splits in a fixed order (no atomics: the result is the same from run to run) and applies what
// follows the projector -- SiLU and the product for up / gate, the residual for down and for the
// output projection, the rotary encoding for q / k / v.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "fspad.h"
#include "stream_gemm.h"

namespace {

using fspad_detail::bf16x8;
using fspad_detail::f32x4;
using fspad_detail::StreamGemm;

constexpr int kWaves = 8;            // wavefronts per workgroup, 16 weight rows each (with 4, twice the
                                     // workgroups: 166 against 158 us for the decoder layer at 4096 / 11008)
constexpr int kSliceRows = 128;      // weight rows per workgroup
constexpr int kChunkK = 256;         // k is cut in multiples of this
constexpr int kMaxRows = 128;        // rows of X per call

struct PartialGemmParams {
  const char* x[2];        // [rows][K] bf16, one per problem (up / gate share a launch)
  const char* w[2];        // [N][K] bf16
  float* part;             // [problem][split][rows][N] fp32
  int32_t rows, N, K;
  int32_t n_slices, n_splits, chunks_per_split;
  int32_t stagger;         // stages by which consecutive slices are offset along k (0: none)
  int32_t packed;          // w is in the tile order of fspad_pack_weight
};

// Workgroup (slice, split) of problem blockIdx.y: X[rows, k range] . W[slice rows, k range]^T
template <int MT, int SPS, bool PACKED = false>
__global__ __launch_bounds__(64 * kWaves, 2) void partial_gemm_kernel(const PartialGemmParams p) {
  typedef StreamGemm<MT, SPS, 16, kWaves, 1, PACKED> G;
  __shared__ __attribute__((aligned(16))) char xs[2 * G::kStageBytes];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, g = lane >> 4;
  const int slice = blockIdx.x / p.n_splits, split = blockIdx.x - slice * p.n_splits, prob = blockIdx.y;
  const int n_chunks = p.K / kChunkK;
  const int chunk0 = split * p.chunks_per_split;
  const int chunks = min(p.chunks_per_split, n_chunks - chunk0);
  const int v0 = slice * kSliceRows + wave * 16;
  const size_t k_off = (size_t)chunk0 * kChunkK * 2;

  f32x4 acc[MT][1];
#pragma unroll
  for (int t = 0; t < MT; ++t) acc[t][0] = f32x4{0.f, 0.f, 0.f, 0.f};
  // consecutive slices start their k range p.stagger stages apart and wrap around: workgroups that
  // run at the same time then read different parts of their rows, instead of crowding the few
  // memory channels that one k offset of rows a power-of-two pitch apart maps to
  const int n_steps = chunks * (kChunkK / 32);
  const int n_stages = n_steps / SPS;
  const int first_step = (p.stagger && n_steps % SPS == 0) ? (int)(((unsigned)slice * (unsigned)p.stagger) % (unsigned)n_stages) * SPS : 0;
  G::run(xs, p.x[prob] + k_off, p.w[prob] + (PACKED ? k_off * 16 : k_off), (size_t)p.K * 2, p.rows, p.N, 0, v0, n_steps, first_step, acc);

  // lane (n, g) holds columns v0 + 4g .. +3 of row 16t + n
  float* out = p.part + ((size_t)prob * p.n_splits + split) * p.rows * p.N;
  const int c0 = v0 + 4 * g;
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int r = 16 * t + n;
    if (r < p.rows && c0 < p.N) *reinterpret_cast<f32x4*>(out + (size_t)r * p.N + c0) = acc[t][0];   // N is a multiple of 4
  }
}

struct CombineParams {
  const float* part;       // [problem][split][rows][N]
  const char* f;           // residual input [rows][N] bf16 (MODE 1)
  char* out;               // [rows][N] bf16 (MODE 2: [rows][N/2], columns below N/2)
  char* out2;              // MODE 2: [rows][N/2], columns from N/2 on
  int32_t rows, N, n_splits, residual;
};

// MODE 0: out = SiLU(sum of the gate partials) * (sum of the up partials). MODE 1: out = sum of the
// partials (+ f). MODE 2: the N columns are two halves that go to two arrays, each half added to the
// same residual f [rows][N/2]. Four columns per thread.
template <int MODE>
__global__ __launch_bounds__(256) void combine_kernel(const CombineParams p) {
  typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
  const size_t quads = (size_t)p.rows * p.N / 4;
  const size_t q = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= quads) return;
  const size_t plane = (size_t)p.rows * p.N;
  f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < p.n_splits; ++s) {
    a += *reinterpret_cast<const f32x4*>(p.part + (size_t)s * plane + 4 * q);
    if (MODE == 0) b += *reinterpret_cast<const f32x4*>(p.part + ((size_t)p.n_splits + s) * plane + 4 * q);
  }
  bf16x4 o;
  if (MODE == 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = (__bf16)(b[i] / (1.0f + __expf(-b[i])) * a[i]);   // a: up, b: gate
  } else if (MODE == 1) {
    if (p.residual) {
      const bf16x4 r = *reinterpret_cast<const bf16x4*>(p.f + 8 * q);
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] += (float)r[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = (__bf16)a[i];
  } else {
    const int half_n = p.N / 2;
    const int row = (int)(4 * q / (size_t)p.N), col = (int)(4 * q - (size_t)row * p.N);
    const bool second = col >= half_n;
    const size_t at = ((size_t)row * half_n + (second ? col - half_n : col)) * 2;   // bytes
    const bf16x4 r = *reinterpret_cast<const bf16x4*>(p.f + at);
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = (__bf16)(a[i] + (float)r[i]);
    *reinterpret_cast<bf16x4*>((second ? p.out2 : p.out) + at) = o;
    return;
  }
  *reinterpret_cast<bf16x4*>(p.out + 8 * q) = o;
}

// RMSNorm of one row per workgroup: out = x / sqrt(mean(x^2) + eps) * gain, fp32 arithmetic, one
// rounding to bf16. Hd is a multiple of 8.
struct RmsNormParams {
  const char* x;           // [rows][Hd] bf16
  const char* gain;        // [Hd] bf16
  char* out;               // [rows][Hd] bf16
  int32_t Hd;
  float eps;
};
__global__ __launch_bounds__(256) void rms_norm_kernel(const RmsNormParams p) {
  __shared__ float wave_sum[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const char* xr = p.x + (size_t)blockIdx.x * p.Hd * 2;
  const int n_vec = p.Hd / 8;
  float ss = 0.f;
  for (int v = tid; v < n_vec; v += 256) {
    const bf16x8 xv = *reinterpret_cast<const bf16x8*>(xr + 16 * v);
#pragma unroll
    for (int i = 0; i < 8; ++i) { const float t = (float)xv[i]; ss += t * t; }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if (lane == 0) wave_sum[wave] = ss;
  __syncthreads();
  const float total = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
  const float inv = 1.0f / sqrtf(total / (float)p.Hd + p.eps);
  char* outr = p.out + (size_t)blockIdx.x * p.Hd * 2;
  for (int v = tid; v < n_vec; v += 256) {
    const bf16x8 xv = *reinterpret_cast<const bf16x8*>(xr + 16 * v);
    const bf16x8 gv = *reinterpret_cast<const bf16x8*>(p.gain + 16 * v);
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (__bf16)((float)xv[i] * inv * (float)gv[i]);
    *reinterpret_cast<bf16x8*>(outr + 16 * v) = o;
  }
}

// Output projection's epilogue and the normalisation that follows it, one row per workgroup:
// h = sum of the partials + residual (rounded to bf16, written), then out = rmsnorm(h) of the rounded
// values, as rms_norm_kernel would compute it from h. Every thread re-reads only what it wrote. 1024
// threads: with the few rows of a draft step the row's loads must all be in flight at once.
struct CombineNormParams {
  const float* part;       // [split][rows][Hd]
  const char* residual;    // [rows][Hd] bf16
  const char* gain;        // [Hd] bf16
  char* h;                 // [rows][Hd] bf16
  char* out;               // [rows][Hd] bf16
  int32_t rows, Hd, n_splits;
  float eps;
};
__global__ __launch_bounds__(1024) void combine_norm_kernel(const CombineNormParams p) {
  typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
  __shared__ float wave_sum[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const size_t row_at = (size_t)blockIdx.x * p.Hd, plane = (size_t)p.rows * p.Hd;
  const int n_quads = p.Hd / 4;
  float ss = 0.f;
  for (int q = tid; q < n_quads; q += 1024) {
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < p.n_splits; ++s) a += *reinterpret_cast<const f32x4*>(p.part + (size_t)s * plane + row_at + 4 * q);
    const bf16x4 r = *reinterpret_cast<const bf16x4*>(p.residual + (row_at + 4 * q) * 2);
    bf16x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[i] = (__bf16)(a[i] + (float)r[i]);
      const float t = (float)o[i];
      ss += t * t;
    }
    *reinterpret_cast<bf16x4*>(p.h + (row_at + 4 * q) * 2) = o;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if (lane == 0) wave_sum[wave] = ss;
  __syncthreads();
  float total = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) total += wave_sum[i];
  const float inv = 1.0f / sqrtf(total / (float)p.Hd + p.eps);
  for (int q = tid; q < n_quads; q += 1024) {
    const bf16x4 hv = *reinterpret_cast<const bf16x4*>(p.h + (row_at + 4 * q) * 2);
    const bf16x4 gv = *reinterpret_cast<const bf16x4*>(p.gain + 8 * q);
    bf16x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = (__bf16)((float)hv[i] * inv * (float)gv[i]);
    *reinterpret_cast<bf16x4*>(p.out + (row_at + 4 * q) * 2) = o;
  }
}

// Sum of the q / k / v projection's partials, rotary encoding of the query and key heads, scatter
// into the attention's layouts. A thread owns four columns of the first half of one head of one
// row and the four partner columns of the second half: entry i of the first half and entry i of
// the second half turn by position * theta^(-2i/D). Angles and their sine / cosine are formed in
// fp64 (a position of some thousands times a frequency rounded to fp32 would already be off by
// more than the result's bf16 rounding).
struct QkvRopeParams {
  const float* part;       // [split][rows][(Hq + 2 Hkv) D]
  const int32_t* positions;  // [rows]
  char* q;                 // [rows][Hq][D] bf16
  char* k;                 // [rows][Hkv][D] bf16
  char* v;                 // [rows][Hkv][D] bf16
  int32_t rows, Hq, Hkv, D, n_splits;
  double neg_log2_theta_2_over_d;   // -2 log2(theta) / D
};
__global__ __launch_bounds__(256) void qkv_rope_kernel(const QkvRopeParams p) {
  typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
  const int quads_per_head = p.D / 8, heads = p.Hq + 2 * p.Hkv;
  const size_t total = (size_t)p.rows * heads * quads_per_head;
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= total) return;
  const int j = (int)(t % quads_per_head);
  const int head = (int)((t / quads_per_head) % heads);
  const int row = (int)(t / ((size_t)quads_per_head * heads));
  const int N = heads * p.D, half = p.D / 2;
  const size_t plane = (size_t)p.rows * N;
  const size_t at = (size_t)row * N + (size_t)head * p.D + 4 * j;
  f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < p.n_splits; ++s) {
    a += *reinterpret_cast<const f32x4*>(p.part + (size_t)s * plane + at);
    b += *reinterpret_cast<const f32x4*>(p.part + (size_t)s * plane + at + half);
  }
  char* dst;
  if (head < p.Hq) dst = p.q + ((size_t)row * p.Hq + head) * p.D * 2;
  else if (head < p.Hq + p.Hkv) dst = p.k + ((size_t)row * p.Hkv + (head - p.Hq)) * p.D * 2;
  else dst = p.v + ((size_t)row * p.Hkv + (head - p.Hq - p.Hkv)) * p.D * 2;
  bf16x4 oa, ob;
  if (head < p.Hq + p.Hkv) {
    const double pos = (double)p.positions[row];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const double ang = pos * exp2((double)(4 * j + i) * p.neg_log2_theta_2_over_d);
      double sn, cs;
      sincos(ang, &sn, &cs);
      const float c = (float)cs, s = (float)sn;
      oa[i] = (__bf16)(a[i] * c - b[i] * s);
      ob[i] = (__bf16)(b[i] * c + a[i] * s);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) { oa[i] = (__bf16)a[i]; ob[i] = (__bf16)b[i]; }
  }
  *reinterpret_cast<bf16x4*>(dst + 8 * j) = oa;
  *reinterpret_cast<bf16x4*>(dst + 8 * j + 2 * half) = ob;
}

// splits of a projector with n_slices slices and n_chunks k-chunks: as few as give a workgroup to
// about two thirds of the compute units (measured at 4096 / 11008 and 4096 / 14336: 76 and 93 us
// with this target, 83 and 95 us with one workgroup per unit, 84 and 97 us with two: a workgroup
// that streams few chunks is mostly set-up, and every split adds a partial tile to write and read
// back), never less than two chunks per split
constexpr int kTargetWorkgroups = 180;
void plan_splits(int n_slices, int n_chunks, int problems, int& n_splits, int& chunks_per_split) {
  int want = (2 * kTargetWorkgroups + n_slices * problems) / (2 * n_slices * problems);   // rounded to nearest
  if (want < 1) want = 1;
  chunks_per_split = (n_chunks + want - 1) / want;
  if (chunks_per_split < 2) chunks_per_split = n_chunks < 2 ? n_chunks : 2;
  n_splits = (n_chunks + chunks_per_split - 1) / chunks_per_split;
}

// measured at 4096 / 11008, 4 rows: Feature Sampler 78.4 us without the rotation, 72.1 / 72.4 / 71.5 us with
// 1 / 3 / 5 stages between consecutive slices; decoder layer 164.5 against 158.5 / 158.3 / 158.8 us
constexpr int kStagger = 3;
void launch_partial(PartialGemmParams g, int problems, hipStream_t stream) {
  g.stagger = kStagger;
  const dim3 grid((unsigned)(g.n_slices * g.n_splits), (unsigned)problems);
  if (g.packed) {
    if (g.rows <= 16) hipLaunchKernelGGL((partial_gemm_kernel<1, 16, true>), grid, dim3(512), 0, stream, g);
    else if (g.rows <= 32) hipLaunchKernelGGL((partial_gemm_kernel<2, 16, true>), grid, dim3(512), 0, stream, g);
    else if (g.rows <= 64) hipLaunchKernelGGL((partial_gemm_kernel<4, 16, true>), grid, dim3(512), 0, stream, g);
    else hipLaunchKernelGGL((partial_gemm_kernel<8, 8, true>), grid, dim3(512), 0, stream, g);
    return;
  }
  if (g.rows <= 16) hipLaunchKernelGGL((partial_gemm_kernel<1, 16>), grid, dim3(512), 0, stream, g);
  else if (g.rows <= 32) hipLaunchKernelGGL((partial_gemm_kernel<2, 16>), grid, dim3(512), 0, stream, g);
  else if (g.rows <= 64) hipLaunchKernelGGL((partial_gemm_kernel<4, 16>), grid, dim3(512), 0, stream, g);
  else hipLaunchKernelGGL((partial_gemm_kernel<8, 8>), grid, dim3(512), 0, stream, g);
}

struct Plan {
  int slices_up, splits_up, cps_up, slices_down, splits_down, cps_down;
  size_t part_floats, s_bytes;
};
Plan make_plan(int rows, int Hd, int I) {
  Plan pl{};
  pl.slices_up = (I + kSliceRows - 1) / kSliceRows;
  plan_splits(pl.slices_up, Hd / kChunkK, 2, pl.splits_up, pl.cps_up);
  pl.slices_down = (Hd + kSliceRows - 1) / kSliceRows;
  plan_splits(pl.slices_down, I / kChunkK, 1, pl.splits_down, pl.cps_down);
  const size_t up = (size_t)2 * pl.splits_up * rows * I, down = (size_t)pl.splits_down * rows * Hd;
  pl.part_floats = up > down ? up : down;
  pl.s_bytes = ((size_t)rows * I * 2 + 255) & ~(size_t)255;
  return pl;
}

}  // namespace

extern "C" size_t fspad_feature_sampler_workspace_bytes(int32_t rows, int32_t hidden_dim, int32_t intermediate_dim) {
  if (rows < 1 || rows > kMaxRows || hidden_dim < kChunkK || hidden_dim % kChunkK || intermediate_dim < kChunkK ||
      intermediate_dim % kChunkK)
    return 0;
  const Plan pl = make_plan(rows, hidden_dim, intermediate_dim);
  return pl.s_bytes + ((pl.part_floats * 4 + 255) & ~(size_t)255);
}

extern "C" fspad_status fspad_feature_sampler(int32_t rows, int32_t hidden_dim, int32_t intermediate_dim, const void* f,
                                              const void* e, const void* w_up, const void* w_gate, const void* w_down,
                                              int32_t flags, void* eta, void* workspace, size_t workspace_bytes,
                                              void* hip_stream) {
  if (flags & ~(FSPAD_SAMPLER_RESIDUAL | FSPAD_WEIGHTS_PACKED)) return FSPAD_ERR_SHAPE;
  const int residual = flags & FSPAD_SAMPLER_RESIDUAL, packed = (flags & FSPAD_WEIGHTS_PACKED) != 0;
  if (!f || !e || !w_up || !w_gate || !w_down || !eta) return FSPAD_ERR_NULL;
  if (rows < 1 || rows > kMaxRows) return FSPAD_ERR_SHAPE;
  if (hidden_dim < kChunkK || hidden_dim % kChunkK || hidden_dim > (1 << 16)) return FSPAD_ERR_SHAPE;
  if (intermediate_dim < kChunkK || intermediate_dim % kChunkK || intermediate_dim > (1 << 18)) return FSPAD_ERR_SHAPE;
  if ((((uintptr_t)f) | ((uintptr_t)e) | ((uintptr_t)w_up) | ((uintptr_t)w_gate) | ((uintptr_t)w_down) | ((uintptr_t)eta)) & 15)
    return FSPAD_ERR_SHAPE;
  if (!workspace || ((uintptr_t)workspace & 15) ||
      workspace_bytes < fspad_feature_sampler_workspace_bytes(rows, hidden_dim, intermediate_dim))
    return FSPAD_ERR_WORKSPACE;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const Plan pl = make_plan(rows, hidden_dim, intermediate_dim);
  char* s_buf = static_cast<char*>(workspace);                       // SiLU(gate) * up, [rows][I] bf16
  float* part = reinterpret_cast<float*>(s_buf + pl.s_bytes);

  // up and gate projectors, one launch
  PartialGemmParams g{};
  g.x[0] = static_cast<const char*>(f); g.x[1] = static_cast<const char*>(e);
  g.w[0] = static_cast<const char*>(w_up); g.w[1] = static_cast<const char*>(w_gate);
  g.part = part; g.rows = rows; g.N = intermediate_dim; g.K = hidden_dim;
  g.n_slices = pl.slices_up; g.n_splits = pl.splits_up; g.chunks_per_split = pl.cps_up;
  g.packed = packed;
  launch_partial(g, 2, stream);
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  CombineParams c{};
  c.part = part; c.f = nullptr; c.out = s_buf; c.rows = rows; c.N = intermediate_dim; c.n_splits = pl.splits_up;
  {
    const size_t quads = (size_t)rows * intermediate_dim / 4;
    hipLaunchKernelGGL(combine_kernel<0>, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, c);
  }
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;

  // down projector and residual
  g.x[0] = s_buf; g.x[1] = nullptr; g.w[0] = static_cast<const char*>(w_down); g.w[1] = nullptr;
  g.N = hidden_dim; g.K = intermediate_dim;
  g.n_slices = pl.slices_down; g.n_splits = pl.splits_down; g.chunks_per_split = pl.cps_down;
  launch_partial(g, 1, stream);
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  c.f = static_cast<const char*>(f); c.out = static_cast<char*>(eta); c.N = hidden_dim; c.n_splits = pl.splits_down;
  c.residual = residual != 0;
  {
    const size_t quads = (size_t)rows * hidden_dim / 4;
    hipLaunchKernelGGL(combine_kernel<1>, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, c);
  }
  if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  return FSPAD_OK;
}

// ------------------------------------------------------------------------------------------------
// The draft decoder layer.
namespace {

size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

struct Stage {
  int slices, splits, cps;
};
Stage plan_stage(int N, int K, int problems) {
  Stage st{};
  st.slices = (N + kSliceRows - 1) / kSliceRows;
  plan_splits(st.slices, K / kChunkK, problems, st.splits, st.cps);
  return st;
}

struct LayerPlan {
  int rows, Hd, I, qkv_n, attn_n;
  Stage qkv, o, up, down;
  size_t xn_bytes, q_bytes, a_bytes, h_bytes, s_bytes, part_bytes, attn_ws_bytes;
};

bool layer_shape_ok(const fspad_draft_layer_desc* d) {
  const fspad_attn_desc& a = d->attn;
  if (a.batch < 1 || a.n_nodes_max < 1 || a.n_nodes_max > FSPAD_MAX_NODES) return false;
  if ((int64_t)a.batch * a.n_nodes_max > kMaxRows) return false;
  if (a.n_q_heads < 1 || a.n_kv_heads < 1 || a.n_q_heads % a.n_kv_heads) return false;
  if (a.head_dim != 64 && a.head_dim != 128) return false;
  if (d->hidden_dim < kChunkK || d->hidden_dim % kChunkK || d->hidden_dim > (1 << 16)) return false;
  if (d->intermediate_dim < kChunkK || d->intermediate_dim % kChunkK || d->intermediate_dim > (1 << 18)) return false;
  const int64_t attn_n = (int64_t)a.n_q_heads * a.head_dim;
  if (attn_n % kChunkK || attn_n > (1 << 16)) return false;
  if (!(d->rms_eps >= 0.0f) || !(d->rope_theta > 0.0f)) return false;
  if (d->weights_packed != 0 && d->weights_packed != 1) return false;
  return true;
}

LayerPlan make_layer_plan(const fspad_draft_layer_desc* d, int32_t max_kv_len) {
  LayerPlan pl{};
  const fspad_attn_desc& a = d->attn;
  pl.rows = a.batch * a.n_nodes_max;
  pl.Hd = d->hidden_dim;
  pl.I = d->intermediate_dim;
  pl.attn_n = a.n_q_heads * a.head_dim;
  pl.qkv_n = (a.n_q_heads + 2 * a.n_kv_heads) * a.head_dim;
  pl.qkv = plan_stage(pl.qkv_n, pl.Hd, 1);
  pl.o = plan_stage(pl.Hd, pl.attn_n, 1);
  pl.up = plan_stage(pl.I, pl.Hd, 2);
  pl.down = plan_stage(2 * pl.Hd, pl.I, 1);
  pl.xn_bytes = align256((size_t)pl.rows * pl.Hd * 2);
  pl.q_bytes = align256((size_t)pl.rows * pl.attn_n * 2);
  pl.a_bytes = pl.q_bytes;
  pl.h_bytes = pl.xn_bytes;
  pl.s_bytes = align256((size_t)pl.rows * pl.I * 2);
  size_t part = (size_t)pl.qkv.splits * pl.rows * pl.qkv_n;
  const size_t part_o = (size_t)pl.o.splits * pl.rows * pl.Hd;
  const size_t part_up = (size_t)2 * pl.up.splits * pl.rows * pl.I;
  const size_t part_down = (size_t)pl.down.splits * pl.rows * 2 * pl.Hd;
  if (part_o > part) part = part_o;
  if (part_up > part) part = part_up;
  if (part_down > part) part = part_down;
  pl.part_bytes = align256(part * 4);
  pl.attn_ws_bytes = align256(fspad_tree_attn_workspace_bytes(&d->attn, max_kv_len));
  return pl;
}

fspad_status linear_partials(const void* x0, const void* x1, const void* w0, const void* w1, int problems, int rows, int N,
                             int K, const Stage& st, float* part, bool packed, hipStream_t stream) {
  PartialGemmParams g{};
  g.x[0] = static_cast<const char*>(x0); g.x[1] = static_cast<const char*>(x1);
  g.w[0] = static_cast<const char*>(w0); g.w[1] = static_cast<const char*>(w1);
  g.part = part; g.rows = rows; g.N = N; g.K = K;
  g.n_slices = st.slices; g.n_splits = st.splits; g.chunks_per_split = st.cps;
  g.packed = packed;
  launch_partial(g, problems, stream);
  return hipGetLastError() == hipSuccess ? FSPAD_OK : FSPAD_ERR_HIP;
}

template <int MODE>
fspad_status combine(const float* part, const void* residual, void* out, void* out2, int rows, int N, int splits,
                     hipStream_t stream) {
  CombineParams c{};
  c.part = part; c.f = static_cast<const char*>(residual); c.out = static_cast<char*>(out);
  c.out2 = static_cast<char*>(out2); c.rows = rows; c.N = N; c.n_splits = splits; c.residual = residual != nullptr;
  const size_t quads = (size_t)rows * N / 4;
  hipLaunchKernelGGL(combine_kernel<MODE>, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, c);
  return hipGetLastError() == hipSuccess ? FSPAD_OK : FSPAD_ERR_HIP;
}

fspad_status rms_norm(const void* x, const void* gain, void* out, int rows, int Hd, float eps, hipStream_t stream) {
  RmsNormParams r{};
  r.x = static_cast<const char*>(x); r.gain = static_cast<const char*>(gain); r.out = static_cast<char*>(out);
  r.Hd = Hd; r.eps = eps;
  hipLaunchKernelGGL(rms_norm_kernel, dim3((unsigned)rows), dim3(256), 0, stream, r);
  return hipGetLastError() == hipSuccess ? FSPAD_OK : FSPAD_ERR_HIP;
}

}  // namespace

extern "C" size_t fspad_draft_layer_workspace_bytes(const fspad_draft_layer_desc* desc, int32_t max_kv_len) {
  if (!desc || max_kv_len < 0 || !layer_shape_ok(desc)) return 0;
  if (desc->attn.io_dtype != FSPAD_BF16 || desc->attn.out_dtype != FSPAD_BF16) return 0;
  const LayerPlan pl = make_layer_plan(desc, max_kv_len);
  return pl.xn_bytes + pl.q_bytes + pl.a_bytes + pl.h_bytes + pl.s_bytes + pl.part_bytes + pl.attn_ws_bytes;
}

extern "C" fspad_status fspad_draft_layer(const fspad_draft_layer_desc* desc, const fspad_draft_layer_weights* w,
                                          const void* eta, const int32_t* positions, const void* k_cache,
                                          const void* v_cache, const int32_t* kv_len, const int32_t* n_nodes,
                                          const uint64_t* anc_mask, void* k_tree, void* v_tree, void* f_tilde, void* f,
                                          void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!desc || !w || !eta || !positions || !kv_len || !n_nodes || !anc_mask || !k_tree || !v_tree || !f_tilde || !f)
    return FSPAD_ERR_NULL;
  if (!w->w_qkv || !w->w_o || !w->w_gate || !w->w_up || !w->w_down || !w->gain_attn || !w->gain_mlp) return FSPAD_ERR_NULL;
  if (desc->attn.io_dtype != FSPAD_BF16 || desc->attn.out_dtype != FSPAD_BF16) return FSPAD_ERR_DTYPE;
  if (!layer_shape_ok(desc)) return FSPAD_ERR_SHAPE;
  const uintptr_t all = (uintptr_t)eta | (uintptr_t)k_tree | (uintptr_t)v_tree | (uintptr_t)f_tilde | (uintptr_t)f |
                        (uintptr_t)w->w_qkv | (uintptr_t)w->w_o | (uintptr_t)w->w_gate | (uintptr_t)w->w_up |
                        (uintptr_t)w->w_down | (uintptr_t)w->gain_attn | (uintptr_t)w->gain_mlp;
  if (all & 15) return FSPAD_ERR_SHAPE;
  int32_t max_kv = 0;
  for (int b = 0; b < desc->attn.batch; ++b) {
    if (kv_len[b] < 0 || n_nodes[b] < 1 || n_nodes[b] > desc->attn.n_nodes_max) return FSPAD_ERR_SHAPE;
    if (kv_len[b] > max_kv) max_kv = kv_len[b];
  }
  if (!workspace || ((uintptr_t)workspace & 15) || workspace_bytes < fspad_draft_layer_workspace_bytes(desc, max_kv))
    return FSPAD_ERR_WORKSPACE;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const LayerPlan pl = make_layer_plan(desc, max_kv);
  const fspad_attn_desc& a = desc->attn;
  const bool packed = desc->weights_packed != 0;

  char* at = static_cast<char*>(workspace);
  char* xn = at; at += pl.xn_bytes;            // normalised input of a projection, [rows][Hd] bf16
  char* q = at; at += pl.q_bytes;              // [rows][Hq][D] bf16
  char* attn = at; at += pl.a_bytes;           // attention output, [rows][Hq][D] bf16
  char* h = at; at += pl.h_bytes;              // state after attention, [rows][Hd] bf16
  char* s = at; at += pl.s_bytes;              // SiLU(gate) * up, [rows][I] bf16
  float* part = reinterpret_cast<float*>(at); at += pl.part_bytes;
  char* attn_ws = at;

  fspad_status st;
  // q, k, v = rotary(W_qkv rmsnorm(eta))
  if ((st = rms_norm(eta, w->gain_attn, xn, pl.rows, pl.Hd, desc->rms_eps, stream)) != FSPAD_OK) return st;
  if ((st = linear_partials(xn, nullptr, w->w_qkv, nullptr, 1, pl.rows, pl.qkv_n, pl.Hd, pl.qkv, part, packed, stream)) != FSPAD_OK)
    return st;
  {
    QkvRopeParams r{};
    r.part = part; r.positions = positions; r.q = q; r.k = static_cast<char*>(k_tree); r.v = static_cast<char*>(v_tree);
    r.rows = pl.rows; r.Hq = a.n_q_heads; r.Hkv = a.n_kv_heads; r.D = a.head_dim; r.n_splits = pl.qkv.splits;
    r.neg_log2_theta_2_over_d = -2.0 * log2((double)desc->rope_theta) / (double)a.head_dim;
    const size_t threads = (size_t)pl.rows * (a.n_q_heads + 2 * a.n_kv_heads) * (a.head_dim / 8);
    hipLaunchKernelGGL(qkv_rope_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, r);
    if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  }
  // tree attention over the draft's own cache
  st = fspad_tree_attn(&desc->attn, q, k_tree, v_tree, k_cache, v_cache, kv_len, n_nodes, anc_mask, attn, attn_ws,
                       pl.attn_ws_bytes, hip_stream);
  if (st != FSPAD_OK) return st;
  // h = eta + W_o attn
  if ((st = linear_partials(attn, nullptr, w->w_o, nullptr, 1, pl.rows, pl.Hd, pl.attn_n, pl.o, part, packed, stream)) != FSPAD_OK)
    return st;
  // and its normalised form for the MLP (whose doubled down projection adds both halves to h)
  {
    CombineNormParams c{};
    c.part = part; c.residual = static_cast<const char*>(eta); c.gain = static_cast<const char*>(w->gain_mlp);
    c.h = h; c.out = xn; c.rows = pl.rows; c.Hd = pl.Hd; c.n_splits = pl.o.splits; c.eps = desc->rms_eps;
    hipLaunchKernelGGL(combine_norm_kernel, dim3((unsigned)pl.rows), dim3(1024), 0, stream, c);
    if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  }
  if ((st = linear_partials(xn, xn, w->w_up, w->w_gate, 2, pl.rows, pl.I, pl.Hd, pl.up, part, packed, stream)) != FSPAD_OK) return st;
  if ((st = combine<0>(part, nullptr, s, nullptr, pl.rows, pl.I, pl.up.splits, stream)) != FSPAD_OK) return st;
  if ((st = linear_partials(s, nullptr, w->w_down, nullptr, 1, pl.rows, 2 * pl.Hd, pl.I, pl.down, part, packed, stream)) != FSPAD_OK)
    return st;
  return combine<2>(part, h, f_tilde, f, pl.rows, 2 * pl.Hd, pl.down.splits, stream);
}

// ------------------------------------------------------------------------------------------------
// Weight repacking: row-major [N][K] -> tile order (see stream_gemm.h). One thread per 16 bytes.
namespace {
__global__ __launch_bounds__(256) void pack_weight_kernel(const char* w, char* packed, int32_t n_rows, int32_t K) {
  const int steps = K / 32;
  const size_t total = (size_t)((n_rows + 15) / 16) * steps * 64;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int lane = (int)(i & 63), n = lane & 15, g = lane >> 4;
  const size_t tile_step = i >> 6;
  const int step = (int)(tile_step % steps);
  const size_t row = (tile_step / steps) * 16 + n;
  bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
  if (row < (size_t)n_rows) v = *reinterpret_cast<const bf16x8*>(w + (row * K + 32 * step + 8 * g) * 2);
  *reinterpret_cast<bf16x8*>(packed + i * 16) = v;
}
}  // namespace

extern "C" size_t fspad_packed_weight_bytes(int32_t n_rows, int32_t k) {
  if (n_rows < 1 || k < 32 || k % 32) return 0;
  return (size_t)((n_rows + 15) / 16) * 16 * (size_t)k * 2;
}

extern "C" fspad_status fspad_pack_weight(int32_t n_rows, int32_t k, const void* w, void* packed, void* hip_stream) {
  if (!w || !packed) return FSPAD_ERR_NULL;
  if (n_rows < 1 || k < 32 || k % 32) return FSPAD_ERR_SHAPE;
  if ((((uintptr_t)w) | ((uintptr_t)packed)) & 15) return FSPAD_ERR_SHAPE;
  const size_t threads = fspad_packed_weight_bytes(n_rows, k) / 16;
  if ((threads + 255) / 256 > 0x7fffffffu) return FSPAD_ERR_SHAPE;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(hip_stream), static_cast<const char*>(w), static_cast<char*>(packed),
                     n_rows, k);
  return hipGetLastError() == hipSuccess ? FSPAD_OK : FSPAD_ERR_HIP;
}
