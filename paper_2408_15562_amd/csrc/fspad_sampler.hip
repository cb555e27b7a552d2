// Feature Sampler of the draft model (arXiv 2408.15562, Methodology, "Feature Sampling": an Up
// Projector for the feature f, a Gate Projector for the token embedding e, SiLU on the lifted
// embedding, element-wise product with the lifted feature, a Down Projector back to the hidden
// size, and the feature path's residual connection):
//
//     eta = W_down (SiLU(W_gate e) * (W_up f)) + f
//
// for the few rows of one draft step (sequences x expanded nodes). gfx950 (CDNA4) only.
//
// Three skinny GEMMs bound by streaming their weights once (3 x Hd x I bf16: 270 MB for a 4096 /
// 11008 model); they share the streaming core of the LM head. A projector has too few 128-row
// slices of its weight matrix to fill the chip (86 for the up / gate projectors, 32 for the down
// projector), so every slice is also cut along k: workgroup (slice, split) leaves an fp32 partial
// tile, and a small element-wise kernel sums the splits in a fixed order (no atomics: the result
// is the same from run to run) and applies what follows the projector -- SiLU and the product for
// up / gate, the residual for down.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "fspad.h"
#include "stream_gemm.h"

namespace {

using fspad_detail::bf16x8;
using fspad_detail::f32x4;
using fspad_detail::StreamGemm;

constexpr int kWaves = 8;            // wavefronts per workgroup, 16 weight rows each
constexpr int kSliceRows = 128;      // weight rows per workgroup
constexpr int kChunkK = 256;         // k is cut in multiples of this
constexpr int kMaxRows = 128;        // rows of X per call

struct PartialGemmParams {
  const char* x[2];        // [rows][K] bf16, one per problem (up / gate share a launch)
  const char* w[2];        // [N][K] bf16
  float* part;             // [problem][split][rows][N] fp32
  int32_t rows, N, K;
  int32_t n_slices, n_splits, chunks_per_split;
};

// Workgroup (slice, split) of problem blockIdx.y: X[rows, k range] . W[slice rows, k range]^T
template <int MT, int SPS>
__global__ __launch_bounds__(64 * kWaves, 2) void partial_gemm_kernel(const PartialGemmParams p) {
  typedef StreamGemm<MT, SPS, 16, kWaves, 1> G;
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
  G::run(xs, p.x[prob] + k_off, p.w[prob] + k_off, (size_t)p.K * 2, p.rows, p.N, 0, v0, chunks * (kChunkK / 32), 0, acc);

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
  char* out;               // [rows][N] bf16
  int32_t rows, N, n_splits, residual;
};

// MODE 0: out = SiLU(sum of the gate partials) * (sum of the up partials). MODE 1: out = sum of the
// partials (+ f). Four columns per thread.
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
  } else {
    if (p.residual) {
      const bf16x4 r = *reinterpret_cast<const bf16x4*>(p.f + 8 * q);
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] += (float)r[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = (__bf16)a[i];
  }
  *reinterpret_cast<bf16x4*>(p.out + 8 * q) = o;
}

// splits of a projector with n_slices slices and n_chunks k-chunks: as few as give a workgroup to
// about two thirds of the compute units (measured at 4096 / 11008 and 4096 / 14336: 76 and 93 us
// with this target, 83 and 95 us with one workgroup per unit, 84 and 97 us with two: a workgroup
// that streams few chunks is mostly set-up, and every split adds a partial tile to write and read
// back), never less than two chunks per split
int g_target_wgs = 180;
void plan_splits(int n_slices, int n_chunks, int problems, int& n_splits, int& chunks_per_split) {
  int want = (2 * g_target_wgs + n_slices * problems) / (2 * n_slices * problems);   // rounded to nearest
  if (want < 1) want = 1;
  chunks_per_split = (n_chunks + want - 1) / want;
  if (chunks_per_split < 2) chunks_per_split = n_chunks < 2 ? n_chunks : 2;
  n_splits = (n_chunks + chunks_per_split - 1) / chunks_per_split;
}

void launch_partial(const PartialGemmParams& g, int problems, hipStream_t stream) {
  const dim3 grid((unsigned)(g.n_slices * g.n_splits), (unsigned)problems);
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

// Experiment knob (not part of the declared interface): workgroups a projector launch aims for.
extern "C" void fspad_debug_set_sampler_target(int32_t wgs) { g_target_wgs = wgs < 1 ? 1 : wgs; }

extern "C" size_t fspad_feature_sampler_workspace_bytes(int32_t rows, int32_t hidden_dim, int32_t intermediate_dim) {
  if (rows < 1 || rows > kMaxRows || hidden_dim < kChunkK || hidden_dim % kChunkK || intermediate_dim < kChunkK ||
      intermediate_dim % kChunkK)
    return 0;
  const Plan pl = make_plan(rows, hidden_dim, intermediate_dim);
  return pl.s_bytes + ((pl.part_floats * 4 + 255) & ~(size_t)255);
}

extern "C" fspad_status fspad_feature_sampler(int32_t rows, int32_t hidden_dim, int32_t intermediate_dim, const void* f,
                                              const void* e, const void* w_up, const void* w_gate, const void* w_down,
                                              int32_t residual, void* eta, void* workspace, size_t workspace_bytes,
                                              void* hip_stream) {
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
