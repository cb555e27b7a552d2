// Tree-masked attention of the draft-tree tokens against the prefix KV cache and
// each other (arXiv 2408.15562, Preliminaries, validation phase: one forward of
// the target over the flattened tree, the tree mask introducing the
// dependencies). gfx950 (CDNA4) only.
//
// bf16 path: one wavefront owns up to 64 query rows (16-row tiles) of one kv head
// and streams 32-key blocks of K and V straight from HBM into registers, each
// byte read once: K rows arrive in the A-operand layout of
// v_mfma_f32_16x16x32_bf16, S^T = K Q^T lands one query row per lane column, so the
// running max / sum of the softmax and the O^T = V^T P^T accumulators of a row
// all live in the same lanes and P never leaves registers. V rows are loaded
// 16 bytes per lane (a whole 256-byte row per 16 lanes) and transposed in
// registers with byte permutes. Wavefronts of a workgroup either split the keys
// (few rows: MHA) and merge through LDS, or take different row slabs of the same
// keys (GQA). A second, tiny kernel merges the split-KV partials.
//
// fp32 path: plain VALU kernel, one wavefront per query row, used for the small
// fp32 parity configuration.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fspad.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

constexpr int kMaxBatchPerLaunch = 128;
constexpr int kBlockKeys = 32;          // keys per streamed block
constexpr float kNegBig = -1.0e30f;     // finite stand-in for "no key seen yet"
constexpr float kLog2e = 1.4426950408889634f;

struct AttnParams {
  const void* q;
  const void* k_tree;
  const void* v_tree;
  const void* k_cache;
  const void* v_cache;
  const uint64_t* anc_mask;
  void* out;
  float* part_o;   // [S][rows][D]   un-normalised partial outputs
  float* part_ml;  // [S][rows][2]   (running max in log2 units, running sum)
  int64_t stride_batch, stride_head, stride_token;  // cache strides, elements
  int32_t B, Nmax, Hq, Hkv, G;
  int32_t S;        // split-KV factor (grid.x)
  int32_t WS;       // row slabs per workgroup: 1, 2 or 4 (4/WS wavefronts share a slab and split its keys)
  int32_t NS;       // row slabs per kv head
  int32_t out_bf16;
  float scale;      // softmax scale
  int32_t kv_len[kMaxBatchPerLaunch];
  uint8_t n_nodes[kMaxBatchPerLaunch];
};

__device__ __forceinline__ float wave_xor_max_16_32(float v) {
  v = fmaxf(v, __shfl_xor(v, 16));
  v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}
__device__ __forceinline__ float wave_xor_sum_16_32(float v) {
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}

// One streamed block of 32 keys in registers.
template <int D>
struct KvBlock {
  static constexpr int KS = D / 32;
  static constexpr int VW = D / 32;  // 32-bit words of one lane's slice of a V row (D/16 bf16)
  bf16x8 k[2][KS];                   // A operands: key tile kt (16 keys), k-step ks (32 dims)
  unsigned v[8][VW];                 // 8 key rows, D/16 consecutive dims each
};

// Which key a lane's j-th V row / P element refers to inside a 32-key block:
// the accumulator layout of two 16-key S^T tiles puts keys 4*g4+i (tile 0) and
// 16+4*g4+i (tile 1) in lane group g4.
__device__ __forceinline__ int key_of(int g4, int j) { return (j < 4) ? 4 * g4 + j : 16 + 4 * g4 + (j - 4); }

template <int D>
__device__ __forceinline__ void load_block(KvBlock<D>& blk, const __bf16* kbase, const __bf16* vbase,
                                           int64_t stride, int nvalid, int col, int g4) {
  constexpr int KS = D / 32;
  constexpr int DT = D / 16;
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) {
    const int key = min(16 * kt + col, nvalid - 1);  // clamp: rows past the end are masked later
    const __bf16* row = kbase + (int64_t)key * stride + 8 * g4;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) blk.k[kt][ks] = *reinterpret_cast<const bf16x8*>(row + 32 * ks);
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int key = min(key_of(g4, j), nvalid - 1);
    const __bf16* row = vbase + (int64_t)key * stride + DT * col;
    if constexpr (D == 128) {
      const u32x4 w = *reinterpret_cast<const u32x4*>(row);
      blk.v[j][0] = w[0]; blk.v[j][1] = w[1]; blk.v[j][2] = w[2]; blk.v[j][3] = w[3];
    } else {
      const u32x2 w = *reinterpret_cast<const u32x2*>(row);
      blk.v[j][0] = w[0]; blk.v[j][1] = w[1];
    }
  }
}

template <int QT, int D>
struct RowState {
  static constexpr int DT = D / 16;
  f32x4 o[QT][DT];   // O^T accumulators: lane (col,g4), reg i <-> row 16t+col, dim DT*(4*g4+i)+e
  float m[QT];       // running max (log2 units, scaled)
  float l[QT];       // running sum, partial per lane until the final cross-lane add
};

// S^T = K Q^T for one block, mask, online softmax, O^T += V^T P^T.
// kind: 0 full prefix block, 1 prefix block with a ragged tail, 2 tree block.
template <int QT, int D>
__device__ __forceinline__ void compute_block(const KvBlock<D>& blk, const bf16x8 (&qf)[QT][D / 32],
                                              RowState<QT, D>& st, int kind, int nvalid, int tree_key0,
                                              const uint64_t (&mask_word)[QT], float c, int g4) {
  constexpr int KS = D / 32;
  constexpr int DT = D / 16;
  f32x4 s[2][QT];
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(blk.k[kt][ks], qf[t][ks], acc, 0, 0, 0);
      s[kt][t] = acc;
    }
  if (kind != 0) {
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = 16 * kt + 4 * g4 + i;
#pragma unroll
        for (int t = 0; t < QT; ++t) {
          bool visible = key < nvalid;
          if (kind == 2) visible = visible && ((mask_word[t] >> (tree_key0 + key)) & 1ull);
          if (!visible) s[kt][t][i] = -INFINITY;
        }
      }
  }
  // online softmax, one query row per (tile, lane column)
  float mnew[QT];
  bool grow = false;
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    float mx = fmaxf(fmaxf(fmaxf(s[0][t][0], s[0][t][1]), fmaxf(s[0][t][2], s[0][t][3])),
                     fmaxf(fmaxf(s[1][t][0], s[1][t][1]), fmaxf(s[1][t][2], s[1][t][3])));
    mx = wave_xor_max_16_32(mx);
    mnew[t] = fmaxf(st.m[t], mx * c);
    grow = grow || (mnew[t] > st.m[t]);
  }
  if (__any(grow)) {  // wavefront-uniform: after the first blocks the maxima rarely move
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      const float alpha = __builtin_amdgcn_exp2f(st.m[t] - mnew[t]);
      st.m[t] = mnew[t];
      st.l[t] *= alpha;
#pragma unroll
      for (int e = 0; e < DT; ++e) st.o[t][e] *= alpha;
    }
  }
  bf16x8 pf[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    float p[8];
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      p[j] = __builtin_amdgcn_exp2f(fmaf(s[j >> 2][t][j & 3], c, -st.m[t]));
      sum += p[j];
    }
    st.l[t] += sum;
#pragma unroll
    for (int j = 0; j < 8; ++j) pf[t][j] = (__bf16)p[j];
  }
  // O^T += V^T P^T; the 8x(D/16) V slice of a lane is transposed with byte permutes
#pragma unroll
  for (int e = 0; e < DT; ++e) {
    const unsigned sel = (e & 1) ? 0x07060302u : 0x05040100u;
    u32x4 w;
#pragma unroll
    for (int m2 = 0; m2 < 4; ++m2)
      w[m2] = __builtin_amdgcn_perm(blk.v[2 * m2 + 1][e >> 1], blk.v[2 * m2][e >> 1], sel);
    const bf16x8 va = __builtin_bit_cast(bf16x8, w);
#pragma unroll
    for (int t = 0; t < QT; ++t)
      st.o[t][e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pf[t], st.o[t][e], 0, 0, 0);
  }
}

template <int QT, int D>
__global__ __launch_bounds__(256) void tree_attn_bf16_kernel(const AttnParams p) {
  constexpr int KS = D / 32;
  constexpr int DT = D / 16;
  constexpr int ROWS = 16 * QT;
  // merge buffers: 3 wavefronts x (QT*DT accumulators + QT stats) x 64 lanes
  __shared__ f32x4 merge_o[3][QT * DT][64];
  __shared__ float2 merge_ml[3][QT][64];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, g4 = lane >> 4;
  const int b = blockIdx.z / p.Hkv, g = blockIdx.z % p.Hkv;
  const int slab_local = wave & (p.WS - 1);
  const int slab = blockIdx.y * p.WS + slab_local;
  const int KW = 4 / p.WS;           // wavefronts that split the keys of one slab
  const int kp = wave / p.WS;
  const int n = p.n_nodes[b];
  const int L = p.kv_len[b];
  const float c = p.scale * kLog2e;
  const bool slab_live = slab < p.NS;

  // rows of this lane: one per tile
  bool row_exists[QT], row_valid[QT];
  int row_out[QT];  // index of (b, node, h) in [B*Nmax*Hq)
  uint64_t mask_word[QT];
  bf16x8 qf[QT][KS];
  const uint64_t live_bits = (n >= 64) ? ~0ull : ((1ull << n) - 1ull);
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int r = slab * ROWS + 16 * t + col;
    const int node = r / p.G, hl = r - node * p.G;
    row_exists[t] = slab_live && r < p.Nmax * p.G;
    row_valid[t] = row_exists[t] && node < n;
    row_out[t] = (b * p.Nmax + node) * p.Hq + g * p.G + hl;
    mask_word[t] = row_valid[t] ? (p.anc_mask[b * p.Nmax + node] & live_bits) : 0ull;
    const __bf16* qrow = reinterpret_cast<const __bf16*>(p.q) + (int64_t)row_out[t] * D + 8 * g4;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 zero;
#pragma unroll
      for (int j = 0; j < 8; ++j) zero[j] = (__bf16)0.f;
      qf[t][ks] = row_valid[t] ? *reinterpret_cast<const bf16x8*>(qrow + 32 * ks) : zero;
    }
  }

  RowState<QT, D> st;
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    st.m[t] = kNegBig;
    st.l[t] = 0.f;
#pragma unroll
    for (int e = 0; e < DT; ++e) st.o[t][e] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // blocks of this sequence: prefix blocks first, then the tree blocks
  const int n_prefix_blocks = (L + kBlockKeys - 1) / kBlockKeys;
  const int n_blocks = n_prefix_blocks + (n + kBlockKeys - 1) / kBlockKeys;
  const int key_waves = p.S * KW;
  const int kw = blockIdx.x * KW + kp;
  const int blk_begin = (int)(((int64_t)kw * n_blocks) / key_waves);
  const int blk_end = (int)(((int64_t)(kw + 1) * n_blocks) / key_waves);

  const __bf16* kc = reinterpret_cast<const __bf16*>(p.k_cache) + b * p.stride_batch + g * p.stride_head;
  const __bf16* vc = reinterpret_cast<const __bf16*>(p.v_cache) + b * p.stride_batch + g * p.stride_head;
  const int64_t tree_stride = (int64_t)p.Hkv * D;
  const __bf16* ktr = reinterpret_cast<const __bf16*>(p.k_tree) + ((int64_t)b * p.Nmax * p.Hkv + g) * D;
  const __bf16* vtr = reinterpret_cast<const __bf16*>(p.v_tree) + ((int64_t)b * p.Nmax * p.Hkv + g) * D;

  auto issue = [&](KvBlock<D>& dst, int blk) {
    if (blk < n_prefix_blocks) {
      const int key0 = blk * kBlockKeys;
      load_block<D>(dst, kc + (int64_t)key0 * p.stride_token, vc + (int64_t)key0 * p.stride_token,
                    p.stride_token, min(kBlockKeys, L - key0), col, g4);
    } else {
      const int t0 = (blk - n_prefix_blocks) * kBlockKeys;
      load_block<D>(dst, ktr + (int64_t)t0 * tree_stride, vtr + (int64_t)t0 * tree_stride, tree_stride,
                    min(kBlockKeys, n - t0), col, g4);
    }
  };
  auto consume = [&](const KvBlock<D>& src, int blk) {
    if (blk < n_prefix_blocks) {
      const int nvalid = min(kBlockKeys, L - blk * kBlockKeys);
      compute_block<QT, D>(src, qf, st, nvalid == kBlockKeys ? 0 : 1, nvalid, 0, mask_word, c, g4);
    } else {
      const int t0 = (blk - n_prefix_blocks) * kBlockKeys;
      compute_block<QT, D>(src, qf, st, 2, min(kBlockKeys, n - t0), t0, mask_word, c, g4);
    }
  };

  if (slab_live && blk_begin < blk_end) {
    KvBlock<D> bufa, bufb;
    issue(bufa, blk_begin);
    for (int blk = blk_begin; blk < blk_end; blk += 2) {
      const bool has_b = blk + 1 < blk_end;
      if (has_b) issue(bufb, blk + 1);
      consume(bufa, blk);
      if (has_b) {
        if (blk + 2 < blk_end) issue(bufa, blk + 2);
        consume(bufb, blk + 1);
      }
    }
  }
#pragma unroll
  for (int t = 0; t < QT; ++t) st.l[t] = wave_xor_sum_16_32(st.l[t]);

  // merge the key-splitting wavefronts of a slab through LDS (lane-private slots)
  if (KW > 1) {
    if (kp > 0) {
      const int slot = (kp - 1) * p.WS + slab_local;
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        merge_ml[slot][t][lane] = make_float2(st.m[t], st.l[t]);
#pragma unroll
        for (int e = 0; e < DT; ++e) merge_o[slot][t * DT + e][lane] = st.o[t][e];
      }
    }
    __syncthreads();
    if (kp == 0) {
      for (int other = 1; other < KW; ++other) {
        const int slot = (other - 1) * p.WS + slab_local;
#pragma unroll
        for (int t = 0; t < QT; ++t) {
          const float2 ml = merge_ml[slot][t][lane];
          const float mm = fmaxf(st.m[t], ml.x);
          const float a0 = __builtin_amdgcn_exp2f(st.m[t] - mm), a1 = __builtin_amdgcn_exp2f(ml.x - mm);
          st.m[t] = mm;
          st.l[t] = st.l[t] * a0 + ml.y * a1;
#pragma unroll
          for (int e = 0; e < DT; ++e) st.o[t][e] = st.o[t][e] * a0 + merge_o[slot][t * DT + e][lane] * a1;
        }
      }
    }
  }
  if (kp != 0) return;

  // write: final rows when there is a single split, partials otherwise
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    if (!row_exists[t]) continue;
    if (p.S == 1) {
      const float inv = row_valid[t] ? 1.0f / st.l[t] : 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int d0 = DT * (4 * g4 + i);
        float vals[DT];
#pragma unroll
        for (int e = 0; e < DT; ++e) vals[e] = row_valid[t] ? st.o[t][e][i] * inv : 0.f;
        if (p.out_bf16) {
          __bf16* dst = reinterpret_cast<__bf16*>(p.out) + (int64_t)row_out[t] * D + d0;
          if constexpr (DT == 8) {
            bf16x8 pk;
#pragma unroll
            for (int e = 0; e < 8; ++e) pk[e] = (__bf16)vals[e];
            *reinterpret_cast<bf16x8*>(dst) = pk;
          } else {
#pragma unroll
            for (int e = 0; e < DT; ++e) dst[e] = (__bf16)vals[e];
          }
        } else {
          float* dst = reinterpret_cast<float*>(p.out) + (int64_t)row_out[t] * D + d0;
#pragma unroll
          for (int e = 0; e < DT; e += 4) *reinterpret_cast<f32x4*>(dst + e) = f32x4{vals[e], vals[e + 1], vals[e + 2], vals[e + 3]};
        }
      }
    } else if (row_valid[t]) {
      const int64_t rows_total = (int64_t)p.B * p.Nmax * p.Hq;
      const int64_t prow = (int64_t)blockIdx.x * rows_total + row_out[t];
      if (g4 == 0) *reinterpret_cast<float2*>(p.part_ml + prow * 2) = make_float2(st.m[t], st.l[t]);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float* dst = p.part_o + prow * D + DT * (4 * g4 + i);
#pragma unroll
        for (int e = 0; e < DT; e += 4)
          *reinterpret_cast<f32x4*>(dst + e) = f32x4{st.o[t][e][i], st.o[t][e + 1][i], st.o[t][e + 2][i], st.o[t][e + 3][i]};
      }
    }
  }
}

// Merge of the split-KV partials: out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
// One thread per 4 output dims; rows of nodes past n_nodes are written as zeros.
template <int D>
__global__ __launch_bounds__(256) void tree_attn_combine_kernel(const AttnParams p) {
  constexpr int TPR = D / 4;  // threads per row
  const int64_t rows_total = (int64_t)p.B * p.Nmax * p.Hq;
  const int64_t row = (int64_t)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;
  if (row >= rows_total) return;
  const int d0 = (threadIdx.x % TPR) * 4;
  const int b = (int)(row / ((int64_t)p.Nmax * p.Hq));
  const int node = (int)((row / p.Hq) % p.Nmax);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (node < p.n_nodes[b]) {
    float M = kNegBig;
    for (int s = 0; s < p.S; ++s) M = fmaxf(M, p.part_ml[(s * rows_total + row) * 2]);
    float denom = 0.f;
    for (int s = 0; s < p.S; ++s) {
      const float2 ml = *reinterpret_cast<const float2*>(p.part_ml + (s * rows_total + row) * 2);
      const float w = __builtin_amdgcn_exp2f(ml.x - M);
      denom += w * ml.y;
      acc += w * *reinterpret_cast<const f32x4*>(p.part_o + (s * rows_total + row) * D + d0);
    }
    acc *= 1.0f / denom;
  }
  if (p.out_bf16) {
    typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
    bf16x4 pk;
#pragma unroll
    for (int e = 0; e < 4; ++e) pk[e] = (__bf16)acc[e];
    *reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(p.out) + row * D + d0) = pk;
  } else {
    *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(p.out) + row * D + d0) = acc;
  }
}

// ---------------------------------------------------------------------------------------------
// fp32 path: one wavefront per (sequence, query head, node); lanes over keys for the scores,
// lanes over dims for the weighted sum. No matrix cores: fp32 inputs need fp32 products for
// the 1e-5 tolerance of the small parity configuration.
template <int D>
__global__ __launch_bounds__(256) void tree_attn_f32_kernel(const AttnParams p) {
  constexpr int DPL = D / 64;  // dims per lane in the PV phase
  __shared__ float q_sh[4][D];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = blockIdx.x, b = blockIdx.z;
  const int g = h / p.G;
  const int n = p.n_nodes[b], L = p.kv_len[b];
  const float* kc = reinterpret_cast<const float*>(p.k_cache) + b * p.stride_batch + g * p.stride_head;
  const float* vc = reinterpret_cast<const float*>(p.v_cache) + b * p.stride_batch + g * p.stride_head;
  const int64_t tree_stride = (int64_t)p.Hkv * D;
  const float* ktr = reinterpret_cast<const float*>(p.k_tree) + ((int64_t)b * p.Nmax * p.Hkv + g) * D;
  const float* vtr = reinterpret_cast<const float*>(p.v_tree) + ((int64_t)b * p.Nmax * p.Hkv + g) * D;

  for (int node = blockIdx.y * 4 + wave; node < p.Nmax; node += gridDim.y * 4) {
    const int64_t row = ((int64_t)b * p.Nmax + node) * p.Hq + h;
    float* out = reinterpret_cast<float*>(p.out) + row * D;
    if (node >= n) {
      for (int d = lane; d < D; d += 64) out[d] = 0.f;
      continue;
    }
    const float* qrow = reinterpret_cast<const float*>(p.q) + row * D;
    for (int d = lane; d < D; d += 64) q_sh[wave][d] = qrow[d];
    __builtin_amdgcn_wave_barrier();
    const uint64_t word = p.anc_mask[b * p.Nmax + node];
    float m = -INFINITY, l = 0.f;
    float acc[DPL];
#pragma unroll
    for (int e = 0; e < DPL; ++e) acc[e] = 0.f;
    const int total = L + n;
    for (int base = 0; base < total; base += 64) {
      const int j = base + lane;
      float s = -INFINITY;
      const float* krow = nullptr;
      if (j < L) krow = kc + (int64_t)j * p.stride_token;
      else if (j < total && ((word >> (j - L)) & 1ull)) krow = ktr + (int64_t)(j - L) * tree_stride;
      if (krow) {
        float dot = 0.f;
        for (int d = 0; d < D; d += 4) {
          const f32x4 kv = *reinterpret_cast<const f32x4*>(krow + d);
          dot = fmaf(q_sh[wave][d], kv[0], dot);
          dot = fmaf(q_sh[wave][d + 1], kv[1], dot);
          dot = fmaf(q_sh[wave][d + 2], kv[2], dot);
          dot = fmaf(q_sh[wave][d + 3], kv[3], dot);
        }
        s = dot * p.scale;
      }
      float mx = s;
      for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
      const float mnew = fmaxf(m, mx);   // finite from the first tile on: key 0 is always visible
      const float alpha = expf(m - mnew);
      const float pj = expf(s - mnew);
      float psum = pj;
      for (int off = 32; off > 0; off >>= 1) psum += __shfl_xor(psum, off);
      l = l * alpha + psum;
      m = mnew;
#pragma unroll
      for (int e = 0; e < DPL; ++e) acc[e] *= alpha;
      const int cnt = min(64, total - base);
      for (int jj = 0; jj < cnt; ++jj) {
        const float pw = __shfl(pj, jj);
        if (pw == 0.f) continue;  // masked (wavefront-uniform)
        const int key = base + jj;
        const float* vrow = key < L ? vc + (int64_t)key * p.stride_token : vtr + (int64_t)(key - L) * tree_stride;
#pragma unroll
        for (int e = 0; e < DPL; ++e) acc[e] = fmaf(pw, vrow[lane + 64 * e], acc[e]);
      }
    }
    const float inv = 1.0f / l;
#pragma unroll
    for (int e = 0; e < DPL; ++e) out[lane + 64 * e] = acc[e] * inv;
    __builtin_amdgcn_wave_barrier();
  }
}

// ---------------------------------------------------------------------------------------------
struct Plan {
  int QT, NS, WS, grid_y, S;
};

int g_forced_splits = 0;

Plan make_plan(const fspad_attn_desc& d, int max_kv_len) {
  Plan pl{};
  const int G = d.n_q_heads / d.n_kv_heads;
  const int rows = d.n_nodes_max * G;
  int best_cost = 1 << 30;
  for (int qt = 4; qt >= 1; --qt) {  // ties go to the larger tile: fewer re-reads of K/V
    const int ns = (rows + 16 * qt - 1) / (16 * qt);
    const int ws = ns == 1 ? 1 : (ns == 2 ? 2 : 4);
    const int gy = (ns + ws - 1) / ws;
    const int cost = gy * ws * qt;
    if (cost < best_cost) { best_cost = cost; pl.QT = qt; pl.NS = ns; pl.WS = ws; pl.grid_y = gy; }
  }
  const int KW = 4 / pl.WS;
  const int n_blocks = (max_kv_len + kBlockKeys - 1) / kBlockKeys + (d.n_nodes_max + kBlockKeys - 1) / kBlockKeys;
  const int64_t wgs_per_split = (int64_t)d.batch * d.n_kv_heads * pl.grid_y;
  // aim at two workgroups per compute unit, but leave every key-splitting wavefront >= 2 blocks
  int64_t s = (512 + wgs_per_split - 1) / wgs_per_split;
  const int64_t s_cap = n_blocks / (2 * KW);
  if (s > s_cap) s = s_cap;
  if (s < 1) s = 1;
  if (s > 64) s = 64;
  if (g_forced_splits > 0) s = g_forced_splits;
  pl.S = (int)s;
  return pl;
}

size_t partial_bytes(const fspad_attn_desc& d, int S) {
  if (S <= 1) return 0;
  const size_t rows = (size_t)d.batch * d.n_nodes_max * d.n_q_heads;
  return (size_t)S * rows * (d.head_dim + 2) * sizeof(float);
}

fspad_status check_desc(const fspad_attn_desc* d) {
  if (!d) return FSPAD_ERR_NULL;
  if (d->batch < 1 || d->n_nodes_max < 1 || d->n_nodes_max > FSPAD_MAX_NODES) return FSPAD_ERR_SHAPE;
  if (d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_q_heads % d->n_kv_heads != 0) return FSPAD_ERR_SHAPE;
  if (d->head_dim != 64 && d->head_dim != 128) return FSPAD_ERR_SHAPE;
  if (d->io_dtype != FSPAD_F32 && d->io_dtype != FSPAD_BF16) return FSPAD_ERR_DTYPE;
  if (d->out_dtype != FSPAD_F32 && d->out_dtype != d->io_dtype) return FSPAD_ERR_DTYPE;
  if (!(d->softmax_scale >= 0.f) || d->softmax_scale > 3.0e38f) return FSPAD_ERR_SHAPE;
  return FSPAD_OK;
}

template <int D>
void launch_bf16(const Plan& pl, const AttnParams& prm, dim3 grid, hipStream_t stream) {
  switch (pl.QT) {
    case 1: hipLaunchKernelGGL((tree_attn_bf16_kernel<1, D>), grid, dim3(256), 0, stream, prm); break;
    case 2: hipLaunchKernelGGL((tree_attn_bf16_kernel<2, D>), grid, dim3(256), 0, stream, prm); break;
    case 3: hipLaunchKernelGGL((tree_attn_bf16_kernel<3, D>), grid, dim3(256), 0, stream, prm); break;
    default: hipLaunchKernelGGL((tree_attn_bf16_kernel<4, D>), grid, dim3(256), 0, stream, prm); break;
  }
}

}  // namespace

extern "C" void fspad_tree_attn_set_splits(int32_t splits) { g_forced_splits = splits > 0 ? (splits > 64 ? 64 : splits) : 0; }

extern "C" size_t fspad_tree_attn_workspace_bytes(const fspad_attn_desc* desc, int32_t max_kv_len) {
  if (check_desc(desc) != FSPAD_OK || max_kv_len < 0) return 0;
  if (desc->io_dtype == FSPAD_F32) return 16;
  const Plan pl = make_plan(*desc, max_kv_len);
  const size_t need = partial_bytes(*desc, pl.S);
  return need < 16 ? 16 : need;
}

extern "C" fspad_status fspad_tree_attn(const fspad_attn_desc* desc, const void* q, const void* k_tree,
                                        const void* v_tree, const void* k_cache, const void* v_cache,
                                        const int32_t* kv_len, const int32_t* n_nodes,
                                        const uint64_t* anc_mask, void* out, void* workspace,
                                        size_t workspace_bytes, void* hip_stream) {
  const fspad_status st = check_desc(desc);
  if (st != FSPAD_OK) return st;
  if (!q || !k_tree || !v_tree || !kv_len || !n_nodes || !anc_mask || !out) return FSPAD_ERR_NULL;
  const fspad_attn_desc& d = *desc;
  const int esz = d.io_dtype == FSPAD_BF16 ? 2 : 4;
  int max_len = 0;
  for (int b = 0; b < d.batch; ++b) {
    if (kv_len[b] < 0 || n_nodes[b] < 1 || n_nodes[b] > d.n_nodes_max) return FSPAD_ERR_SHAPE;
    if (kv_len[b] > max_len) max_len = kv_len[b];
  }
  if (max_len > 0) {
    if (!k_cache || !v_cache) return FSPAD_ERR_NULL;
    const int64_t align = 16 / esz;
    if (d.cache_stride_token < d.head_dim || d.cache_stride_token % align || d.cache_stride_head % align ||
        d.cache_stride_batch % align || d.cache_stride_head < 0 || d.cache_stride_batch < 0)
      return FSPAD_ERR_SHAPE;
    if (((uintptr_t)k_cache | (uintptr_t)v_cache) & 15) return FSPAD_ERR_SHAPE;
  }
  if (((uintptr_t)q | (uintptr_t)k_tree | (uintptr_t)v_tree | (uintptr_t)out) & 15) return FSPAD_ERR_SHAPE;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);

  AttnParams prm{};
  prm.q = q; prm.k_tree = k_tree; prm.v_tree = v_tree; prm.k_cache = k_cache; prm.v_cache = v_cache;
  prm.anc_mask = anc_mask; prm.out = out;
  prm.stride_batch = d.cache_stride_batch; prm.stride_head = d.cache_stride_head; prm.stride_token = d.cache_stride_token;
  prm.B = d.batch; prm.Nmax = d.n_nodes_max; prm.Hq = d.n_q_heads; prm.Hkv = d.n_kv_heads;
  prm.G = d.n_q_heads / d.n_kv_heads;
  prm.out_bf16 = d.out_dtype == FSPAD_BF16;
  prm.scale = d.softmax_scale > 0.f ? d.softmax_scale : 1.0f / sqrtf((float)d.head_dim);

  Plan pl{};
  if (d.io_dtype == FSPAD_BF16) {
    pl = make_plan(d, max_len);
    const size_t need = partial_bytes(d, pl.S);
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15))) return FSPAD_ERR_WORKSPACE;
    prm.S = pl.S; prm.WS = pl.WS; prm.NS = pl.NS;
    prm.part_o = pl.S > 1 ? reinterpret_cast<float*>(workspace) : nullptr;
  } else {
    prm.S = 1; prm.WS = 1; prm.NS = 1;
  }

  // sequences are independent: slices of at most kMaxBatchPerLaunch sequences per launch (the
  // per-sequence lengths travel as kernel arguments), each slice reusing the workspace in stream order
  for (int b0 = 0; b0 < d.batch; b0 += kMaxBatchPerLaunch) {
    const int nb = d.batch - b0 < kMaxBatchPerLaunch ? d.batch - b0 : kMaxBatchPerLaunch;
    AttnParams sl = prm;
    sl.B = nb;
    const size_t q_rows = (size_t)b0 * d.n_nodes_max * d.n_q_heads * d.head_dim;
    const size_t kv_rows = (size_t)b0 * d.n_nodes_max * d.n_kv_heads * d.head_dim;
    sl.q = static_cast<const char*>(q) + q_rows * esz;
    sl.k_tree = static_cast<const char*>(k_tree) + kv_rows * esz;
    sl.v_tree = static_cast<const char*>(v_tree) + kv_rows * esz;
    if (k_cache) {
      sl.k_cache = static_cast<const char*>(k_cache) + (size_t)b0 * d.cache_stride_batch * esz;
      sl.v_cache = static_cast<const char*>(v_cache) + (size_t)b0 * d.cache_stride_batch * esz;
    }
    sl.anc_mask = anc_mask + (size_t)b0 * d.n_nodes_max;
    sl.out = static_cast<char*>(out) + q_rows * (d.out_dtype == FSPAD_BF16 ? 2 : 4);
    for (int i = 0; i < nb; ++i) { sl.kv_len[i] = kv_len[b0 + i]; sl.n_nodes[i] = (uint8_t)n_nodes[b0 + i]; }
    if (d.io_dtype == FSPAD_BF16) {
      const size_t rows = (size_t)nb * d.n_nodes_max * d.n_q_heads;
      sl.part_ml = sl.part_o ? sl.part_o + (size_t)pl.S * rows * d.head_dim : nullptr;
      dim3 grid((unsigned)pl.S, (unsigned)pl.grid_y, (unsigned)(nb * d.n_kv_heads));
      if (d.head_dim == 128) launch_bf16<128>(pl, sl, grid, stream); else launch_bf16<64>(pl, sl, grid, stream);
      if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
      if (pl.S > 1) {
        const int rpb = 256 / (d.head_dim / 4);
        dim3 cgrid((unsigned)((rows + rpb - 1) / rpb));
        if (d.head_dim == 128) hipLaunchKernelGGL(tree_attn_combine_kernel<128>, cgrid, dim3(256), 0, stream, sl);
        else hipLaunchKernelGGL(tree_attn_combine_kernel<64>, cgrid, dim3(256), 0, stream, sl);
        if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
      }
    } else {
      dim3 grid((unsigned)d.n_q_heads, (unsigned)((d.n_nodes_max + 3) / 4), (unsigned)nb);
      if (d.head_dim == 128) hipLaunchKernelGGL(tree_attn_f32_kernel<128>, grid, dim3(256), 0, stream, sl);
      else hipLaunchKernelGGL(tree_attn_f32_kernel<64>, grid, dim3(256), 0, stream, sl);
      if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
    }
  }
  return FSPAD_OK;
}
