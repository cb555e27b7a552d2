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
#include <stddef.h>
#include <stdint.h>

#include "fspad.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

constexpr int kMaxBatchPerLaunch = 128;
constexpr int64_t kMaxFlatBlocks = 1ll << 30;  // 32-key blocks of one launch, summed over its units
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
  float* part;     // partial slots: [slot][rows_per_unit][D] un-normalised outputs, then [rows_per_unit][2] (shift, sum)
  int64_t stride_batch, stride_head, stride_token;  // cache strides, elements
  int32_t B, Nmax, Hq, Hkv, G;
  int32_t WS;       // row slabs per workgroup: 1, 2 or 4 (4/WS wavefronts share a slab and split its keys)
  int32_t ws_shift; // log2(WS)
  int32_t NS;       // row slabs per kv head
  int32_t GY;       // slab groups per kv head: a (sequence, kv head, slab group) is one unit of work
  int32_t n_wgs;    // workgroups of the flat decomposition
  int32_t total_blocks;  // 32-key blocks summed over all units (T)
  int32_t wg_quot, wg_rem;  // T = wg_quot * n_wgs + wg_rem: workgroup w starts at w*wg_quot + w*wg_rem/n_wgs
  uint32_t g_magic, gy_magic;  // ceil(2^32 / G), ceil(2^32 / GY): division by multiplication (unused when the divisor is 1)
  int32_t out_bf16;
  float scale;      // softmax scale
  // when every sequence of the launch has the same prefix length and node count: the flat blocks of
  // one sequence (0 otherwise) and those two numbers, so that a workgroup finds its sequence and its
  // lengths by arithmetic instead of dependent loads from the arrays below
  int32_t seq_blocks, same_len, same_nodes;
  int32_t kv_len[kMaxBatchPerLaunch];
  int32_t bstart[kMaxBatchPerLaunch + 1];  // first flat block of each sequence; bstart[B] = total_blocks
  int32_t n_nodes[kMaxBatchPerLaunch];
};

// The scalar part of AttnParams as the kernels use it, fetched from the kernel-argument segment in
// ONE batch of scalar loads at the top of a kernel. Left to the compiler, the arguments are loaded
// where they are first needed: eight dependent round trips stood between a wavefront's start and
// its first K/V request (a kernel that lives for ten to a hundred microseconds notices each of
// them). The per-sequence arrays stay in the argument segment and are read from there.
typedef const __attribute__((address_space(4))) int32_t* KernargI32;
typedef const __attribute__((address_space(4))) char* KernargPtr;
struct AttnArgs {
  const void* q;
  const void* k_tree;
  const void* v_tree;
  const void* k_cache;
  const void* v_cache;
  const uint64_t* anc_mask;
  void* out;
  float* part;
  int64_t stride_batch, stride_head, stride_token;
  int32_t B, Nmax, Hq, Hkv, G, WS, ws_shift, NS, GY, n_wgs, total_blocks, wg_quot, wg_rem;
  uint32_t g_magic, gy_magic;
  int32_t out_bf16;
  float scale;
  int32_t seq_blocks, same_len, same_nodes;
  KernargI32 kv_len, bstart, n_nodes;
};
static_assert(offsetof(AttnParams, stride_batch) == 64 && offsetof(AttnParams, B) == 88 && offsetof(AttnParams, total_blocks) == 128 &&
              offsetof(AttnParams, scale) == 152 && offsetof(AttnParams, same_nodes) == 164 && offsetof(AttnParams, kv_len) == 168,
              "fetch_args reads the scalars by their offsets");

__device__ __forceinline__ AttnArgs fetch_args() {
  typedef int v16i __attribute__((ext_vector_type(16)));
  KernargPtr ka = (KernargPtr)__builtin_amdgcn_kernarg_segment_ptr();   // AttnParams is the first argument
  v16i a, b, c;
  asm volatile("s_load_dwordx16 %0, %3, 0x0\n\ts_load_dwordx16 %1, %3, 0x40\n\ts_load_dwordx16 %2, %3, 0x80\n\ts_waitcnt lgkmcnt(0)"
               : "=&s"(a), "=&s"(b), "=&s"(c) : "s"(ka));
  auto u64 = [](int lo, int hi) { return ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo; };
  AttnArgs r;
  r.q = reinterpret_cast<const void*>(u64(a[0], a[1]));
  r.k_tree = reinterpret_cast<const void*>(u64(a[2], a[3]));
  r.v_tree = reinterpret_cast<const void*>(u64(a[4], a[5]));
  r.k_cache = reinterpret_cast<const void*>(u64(a[6], a[7]));
  r.v_cache = reinterpret_cast<const void*>(u64(a[8], a[9]));
  r.anc_mask = reinterpret_cast<const uint64_t*>(u64(a[10], a[11]));
  r.out = reinterpret_cast<void*>(u64(a[12], a[13]));
  r.part = reinterpret_cast<float*>(u64(a[14], a[15]));
  r.stride_batch = (int64_t)u64(b[0], b[1]);
  r.stride_head = (int64_t)u64(b[2], b[3]);
  r.stride_token = (int64_t)u64(b[4], b[5]);
  r.B = b[6]; r.Nmax = b[7]; r.Hq = b[8]; r.Hkv = b[9]; r.G = b[10]; r.WS = b[11]; r.ws_shift = b[12]; r.NS = b[13];
  r.GY = b[14]; r.n_wgs = b[15];
  r.total_blocks = c[0]; r.wg_quot = c[1]; r.wg_rem = c[2]; r.g_magic = (uint32_t)c[3]; r.gy_magic = (uint32_t)c[4];
  r.out_bf16 = c[5];
  const int scale_bits = c[6];   // (a bit cast straight from the vector element reads element 0)
  r.scale = __builtin_bit_cast(float, scale_bits);
  r.seq_blocks = c[7]; r.same_len = c[8]; r.same_nodes = c[9];
  r.kv_len = (KernargI32)(ka + offsetof(AttnParams, kv_len));
  r.bstart = (KernargI32)(ka + offsetof(AttnParams, bstart));
  r.n_nodes = (KernargI32)(ka + offsetof(AttnParams, n_nodes));
  return r;
}
// sequence that flat block r0 belongs to, and the first flat block / lengths of a sequence
__device__ __forceinline__ int seq_of_block(const AttnArgs& p, unsigned r0) {
  if (p.seq_blocks > 0) return (int)(r0 / (unsigned)p.seq_blocks);
  int b = 0;
  while (b + 1 < p.B && r0 >= (unsigned)p.bstart[b + 1]) ++b;
  return b;
}
__device__ __forceinline__ unsigned seq_first_block(const AttnArgs& p, int b) {
  return p.seq_blocks > 0 ? (unsigned)b * (unsigned)p.seq_blocks : (unsigned)p.bstart[b];
}
__device__ __forceinline__ int seq_nodes(const AttnArgs& p, int b) { return p.seq_blocks > 0 ? p.same_nodes : p.n_nodes[b]; }
__device__ __forceinline__ int seq_len(const AttnArgs& p, int b) { return p.seq_blocks > 0 ? p.same_len : p.kv_len[b]; }

// x / d for x*d < 2^32, with magic = ceil(2^32 / d) (d >= 2) from the host
__device__ __forceinline__ unsigned div_magic(unsigned x, int d, unsigned magic) {
  return d == 1 ? x : __umulhi(x, magic);
}

// First flat block of workgroup w under the even split: floor(w * T / W), in 32-bit arithmetic
// (w * wg_rem < 2^30 because both stay below the 32768 workgroups a launch may have).
__device__ __forceinline__ unsigned wg_first_block(const AttnArgs& p, unsigned w) {
  return w * (unsigned)p.wg_quot + (w * (unsigned)p.wg_rem) / (unsigned)p.n_wgs;
}

__device__ __forceinline__ float wave_xor_max_16_32(float v) {
  v = fmaxf(v, __shfl_xor(v, 16));
  v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}

// Which key a lane's j-th V row / P element refers to inside a 32-key block:
// the accumulator layout of two 16-key S^T tiles puts keys 4*g4+i (tile 0) and
// 16+4*g4+i (tile 1) in lane group g4.
__device__ __forceinline__ int key_of(int g4, int j) { return (j < 4) ? 4 * g4 + j : 16 + 4 * g4 + (j - 4); }

// Where one 32-key block lives and how it is masked.
struct BlockSrc {
  const char* k;       // first key row of the block
  const char* v;
  unsigned row_bytes;  // bytes between consecutive keys
  int nvalid;          // keys of the block that exist (1..32)
  int kind;            // 0 full prefix block, 1 prefix block with a ragged tail, 2 tree block
  int tree_key0;       // first tree node of a tree block
};

// Per-lane byte offsets of a block's rows from its first row. They depend only on the row pitch
// and on how many rows exist (rows past the end of a ragged block are clamped and masked later),
// so they are recomputed only where a stream changes from full blocks to its tail or to the tree.
// K rows arrive in the A-operand layout of the 16x16x32 MFMA: lane (col, g4) holds key 16*kt+col,
// dims 32*ks + 8*g4 .. +7.
__device__ __forceinline__ void k_offsets(unsigned (&off)[2], unsigned row_bytes, int nvalid, int col, int g4) {
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) off[kt] = (unsigned)min(16 * kt + col, nvalid - 1) * row_bytes + 16u * g4;
}
// V rows: lane (col, g4) holds, for its 8 keys, the D/16 consecutive dims starting at (D/16)*col,
// i.e. 16 lanes read one whole row contiguously.
template <int D>
__device__ __forceinline__ void v_offsets(unsigned (&off)[8], unsigned row_bytes, int nvalid, int col, int g4) {
#pragma unroll
  for (int j = 0; j < 8; ++j) off[j] = (unsigned)min(key_of(g4, j), nvalid - 1) * row_bytes + (unsigned)(D / 8) * col;
}

// Scalar base + per-lane byte offset.
template <int D>
__device__ __forceinline__ void load_k(bf16x8 (&k)[2][D / 32], const char* base, const unsigned (&off)[2]) {
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) k[kt][ks] = *reinterpret_cast<const bf16x8*>(base + off[kt] + 64 * ks);
}
template <int D>
__device__ __forceinline__ void load_v(unsigned (&v)[8][D / 32], const char* base, const unsigned (&off)[8]) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    if constexpr (D == 128) {
      const u32x4 w = *reinterpret_cast<const u32x4*>(base + off[j]);
      v[j][0] = w[0]; v[j][1] = w[1]; v[j][2] = w[2]; v[j][3] = w[3];
    } else {
      const u32x2 w = *reinterpret_cast<const u32x2*>(base + off[j]);
      v[j][0] = w[0]; v[j][1] = w[1];
    }
  }
}

template <int QT, int D>
struct RowState {
  static constexpr int DT = D / 16;
  f32x4 o[QT][DT];   // O^T accumulators: lane (col,g4), reg i <-> row 16t+col, dim DT*(4*g4+i)+e
  float m[QT];       // softmax shift in use (log2 units, scaled): within kLazyLog2 of the running max
  f32x4 l[QT];       // running sum of the weights, formed on the matrix cores (all 4 entries equal)
};

// The shift of a row only moves when a score exceeds it by more than this (log2 units): weights
// then stay below 2^kLazyLog2, which fp32 sums and bf16 weights hold without loss, and the
// accumulators are rescaled (and lanes exchanged) almost never after the first blocks.
constexpr float kLazyLog2 = 8.0f;

// One 32-key block against the wavefront's 16*QT query rows, two row tiles at a time so that only
// 16 score and 8 weight registers are live and the matrix work of one tile pair can run under the
// vector work of the other:
//   S^T = K Q^T          s[kt][i] of tile t in lane (col,g4) is key 16*kt+4*g4+i against row 16*t+col
//   mask (ragged / tree blocks), lazy shift update, weights p = 2^(s*c - m) rounded to bf16
//   O^T += V^T P^T       V slice of a lane transposed once per block with byte permutes
//   l   += 1^T P^T       row sums on the matrix cores: sums of the bf16 weights actually used, so
//                        numerator and denominator agree (a dominant key is reproduced exactly),
//                        with no vector-ALU adds and no lane exchange.
// Q fragments come from registers, or (large row tiles) from lane-private LDS slots.
// `after_scores()` runs once the last product that reads k has been issued (the caller requests
// the next block's K there when it keeps a single K buffer). `after_transpose()` runs, for tiles
// done in several passes, once v has been transposed and is dead (the caller requests the next
// block's V into the same registers there: a whole block of lead time at no register cost).
// kVReady: `v` already holds the DT transposed operands (operand e = dwords 4e .. 4e+3 of the
// array, d = 16e + col) instead of the lane's raw 16-byte slices of 8 V rows.
template <int QT, int D, bool kVReady = false, typename QFn, typename MaskFn, typename AfterFn, typename AfterVFn>
__device__ __forceinline__ void process_block(RowState<QT, D>& st, const bf16x8 (&k)[2][D / 32],
                                              const unsigned (&v)[8][D / 32], QFn&& q_frag, const BlockSrc& src,
                                              MaskFn&& mask_of_tile, float c, int g4, AfterFn&& after_scores,
                                              AfterVFn&& after_transpose) {
  constexpr int DT = D / 16;
  constexpr int TP = QT >= 2 ? 2 : 1;  // tiles per pass
  bf16x8 ones;
#pragma unroll
  for (int j = 0; j < 8; ++j) ones[j] = (__bf16)1.0f;
  bf16x8 vt[DT];  // transposed V: A operand of d-tile e holds dims DT*col+e of the lane group's 8 keys
#pragma unroll
  for (int t0 = 0; t0 < QT; t0 += TP) {
    f32x4 s[TP][2];
#pragma unroll
    for (int tt = 0; tt < TP; ++tt) {
      if (t0 + tt >= QT) continue;
      f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < D / 32; ++ks) {
        const bf16x8 q = q_frag(t0 + tt, ks);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k[0][ks], q, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k[1][ks], q, acc1, 0, 0, 0);
      }
      s[tt][0] = acc0;
      s[tt][1] = acc1;
    }
    if (t0 + TP >= QT) after_scores();
    if (src.kind != 0) {  // wavefront-uniform: ragged tail and tree blocks only
#pragma unroll
      for (int tt = 0; tt < TP; ++tt) {
        if (t0 + tt >= QT) continue;
        // visibility of the block's 32 keys for this lane's row, then shifted to the lane's own keys
        unsigned vis = src.nvalid >= kBlockKeys ? ~0u : ((1u << src.nvalid) - 1u);
        if (src.kind == 2) vis &= (unsigned)(mask_of_tile(t0 + tt) >> src.tree_key0);
        vis >>= 4 * g4;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int i = 0; i < 4; ++i) s[tt][kt][i] = ((vis >> (16 * kt + i)) & 1u) ? s[tt][kt][i] : -INFINITY;
      }
    }
    // exponents of the weights under the shift in use: t = s*c - m. Their maximum decides whether
    // the shift has to move (results of an fma are canonical numbers: the maximum needs no
    // quieting of its inputs, unlike one over the raw outputs of the matrix instructions)
    float tv[TP][8];
    bool grow = false;
#pragma unroll
    for (int tt = 0; tt < TP; ++tt) {
      if (t0 + tt >= QT) continue;
      const float m = st.m[t0 + tt];
#pragma unroll
      for (int j = 0; j < 8; ++j) tv[tt][j] = fmaf(s[tt][j >> 2][j & 3], c, -m);
      const float mt = fmaxf(fmaxf(fmaxf(tv[tt][0], tv[tt][1]), fmaxf(tv[tt][2], tv[tt][3])),
                             fmaxf(fmaxf(tv[tt][4], tv[tt][5]), fmaxf(tv[tt][6], tv[tt][7])));
      grow = grow || (mt > kLazyLog2);
    }
    if (__any(grow)) {  // wavefront-uniform and rare: move these rows' shifts to their running maxima
#pragma unroll
      for (int tt = 0; tt < TP; ++tt) {
        if (t0 + tt >= QT) continue;
        const int t = t0 + tt;
        const float mx = fmaxf(fmaxf(fmaxf(s[tt][0][0], s[tt][0][1]), fmaxf(s[tt][0][2], s[tt][0][3])),
                               fmaxf(fmaxf(s[tt][1][0], s[tt][1][1]), fmaxf(s[tt][1][2], s[tt][1][3])));
        const float mnew = fmaxf(st.m[t], wave_xor_max_16_32(mx) * c);
        const float alpha = __builtin_amdgcn_exp2f(st.m[t] - mnew);
        st.m[t] = mnew;
        st.l[t] *= alpha;
#pragma unroll
        for (int e = 0; e < DT; ++e) st.o[t][e] *= alpha;
#pragma unroll
        for (int j = 0; j < 8; ++j) tv[tt][j] = fmaf(s[tt][j >> 2][j & 3], c, -mnew);
      }
    }
    bf16x8 pf[TP];
#pragma unroll
    for (int tt = 0; tt < TP; ++tt) {
      if (t0 + tt >= QT) continue;
#pragma unroll
      for (int j = 0; j < 8; ++j) pf[tt][j] = (__bf16)__builtin_amdgcn_exp2f(tv[tt][j]);
    }
    auto transposed = [&](int e) {  // A operand of d-tile e from the lane's 8 x DT slice of V
      if constexpr (kVReady) {
        const unsigned* flat = &v[0][0];
        return __builtin_bit_cast(bf16x8, u32x4{flat[4 * e], flat[4 * e + 1], flat[4 * e + 2], flat[4 * e + 3]});
      }
      const unsigned sel = (e & 1) ? 0x07060302u : 0x05040100u;
      u32x4 w;
#pragma unroll
      for (int m2 = 0; m2 < 4; ++m2) w[m2] = __builtin_amdgcn_perm(v[2 * m2 + 1][e >> 1], v[2 * m2][e >> 1], sel);
      return __builtin_bit_cast(bf16x8, w);
    };
    constexpr bool kSinglePass = QT <= TP;  // one pass: transpose on the fly, nothing to keep
    if (!kSinglePass && t0 == 0) {
#pragma unroll
      for (int e = 0; e < DT; ++e) vt[e] = transposed(e);
      after_transpose();
    }
#pragma unroll
    for (int tt = 0; tt < TP; ++tt) {
      if (t0 + tt >= QT) continue;
      st.l[t0 + tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pf[tt], st.l[t0 + tt], 0, 0, 0);
    }
#pragma unroll
    for (int e = 0; e < DT; ++e) {
      const bf16x8 va = kSinglePass ? transposed(e) : vt[e];
#pragma unroll
      for (int tt = 0; tt < TP; ++tt) {
        if (t0 + tt >= QT) continue;
        st.o[t0 + tt][e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pf[tt], st.o[t0 + tt][e], 0, 0, 0);
      }
    }
  }
}

// The (sequence, kv head, slab group) units and their 32-key blocks form one flat list of
// blocks; workgroup w owns the contiguous range [w*T/W, (w+1)*T/W) of it, so every workgroup
// streams the same number of bytes whatever the head count. A workgroup therefore works on one
// or a few *segments* (a run of blocks of one unit). A segment that is a whole unit is written
// to `out` directly; otherwise its un-normalised (O, max, sum) goes to partial slot unit+w and the
// merge kernel finishes the unit.
template <int QT, int D>
__global__ __launch_bounds__(256, (QT <= 2 ? 2 : 1)) void tree_attn_bf16_kernel(const AttnParams) {
  const AttnArgs p = fetch_args();
  constexpr int KS = D / 32;
  constexpr int DT = D / 16;
  constexpr int ROWS = 16 * QT;
  // merge buffers: 4 wavefronts x (QT*DT accumulators + QT stats) x 64 lanes. With large row tiles
  // the Q fragments of the 4 wavefronts live in lane-private LDS slots instead of registers; they are
  // dead once a segment's stream is done, so they share the space of the merge buffers.
  constexpr bool kQInLds = QT >= 3;
  // Tiles done in several passes run one wavefront per SIMD: they hide the memory latency by
  // themselves, keeping K and V of the next block in flight for a whole block
  constexpr bool kDeep = QT >= 3;
  constexpr int kMergeBytes = 4 * QT * DT * 64 * 16;
  constexpr int kQBytes = kQInLds ? 4 * QT * KS * 64 * 16 : 0;
  __shared__ __attribute__((aligned(16))) char lds_raw[kMergeBytes > kQBytes ? kMergeBytes : kQBytes];
  __shared__ float2 merge_ml[4][QT][64];
  typedef f32x4 (*MergeO)[QT * DT][64];
  MergeO merge_o = reinterpret_cast<MergeO>(lds_raw);

  // the wavefront index is the same in all 64 lanes: telling the compiler keeps everything that
  // derives from it (key split, block counters, base addresses) in scalar registers
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 15, g4 = lane >> 4;
  bf16x8* q_lds = reinterpret_cast<bf16x8*>(lds_raw) + wave * (QT * KS * 64) + lane;
  const int slab_local = wave & (p.WS - 1);
  const int KW = 4 >> p.ws_shift;  // wavefronts that split the keys of one slab
  const int kp = wave >> p.ws_shift;
  const float c = p.scale * kLog2e;
  const unsigned tree_row_bytes = (unsigned)p.Hkv * D * 2u;
  const unsigned cache_row_bytes = (unsigned)p.stride_token * 2u;
  const int rows_per_unit = p.WS * ROWS;

  // A kernel this short-lived spends much of its time fetching instructions it runs once: all
  // index arithmetic up to the first loads is 32-bit, and divisions by the launch's constants
  // are multiplications.
  const unsigned w = blockIdx.x;
  // [r0, r1) = [floor(w*T/W), floor((w+1)*T/W)) with T = wg_quot*W + wg_rem, from one division
  const unsigned wr = w * (unsigned)p.wg_rem, wq = wr / (unsigned)p.n_wgs;
  const unsigned r0 = w * (unsigned)p.wg_quot + wq;
  const unsigned r1 = r0 + (unsigned)p.wg_quot + ((wr - wq * (unsigned)p.n_wgs) + (unsigned)p.wg_rem >= (unsigned)p.n_wgs ? 1u : 0u);
  int b = seq_of_block(p, r0);

  for (unsigned r = r0; r < r1;) {
    const int n = seq_nodes(p, b);
    const int L = seq_len(p, b);
    const int n_prefix_blocks = (L + kBlockKeys - 1) / kBlockKeys;
    const int n_blocks = n_prefix_blocks + (n + kBlockKeys - 1) / kBlockKeys;
    const unsigned rel = r - seq_first_block(p, b);
    const int ub = (int)(rel / (unsigned)n_blocks);              // unit within the sequence: (g, y)
    const int seg_begin = (int)(rel - (unsigned)ub * (unsigned)n_blocks);
    const int seg_count = min(n_blocks - seg_begin, (int)(r1 - r));
    const int g = (int)div_magic((unsigned)ub, p.GY, p.gy_magic), y = ub - g * p.GY;
    const int unit = b * p.Hkv * p.GY + ub;
    const bool whole_unit = seg_count == n_blocks;
    const int slab = y * p.WS + slab_local;
    const bool slab_live = slab < p.NS;

    // the key-splitting wavefronts of a slab share the segment's blocks evenly
    // interleaved: wavefront kp takes blocks kp, kp+KW, ... so that the workgroup as a whole walks
    // one contiguous stretch of K and of V (neighbouring DRAM pages stay open)
    const int blk_begin = seg_begin + kp;
    const int blk_end = seg_begin + seg_count;
    const bool active = slab_live && blk_begin < blk_end;

    const char* kc = reinterpret_cast<const char*>(p.k_cache) + (b * p.stride_batch + g * p.stride_head) * 2;
    const char* vc = reinterpret_cast<const char*>(p.v_cache) + (b * p.stride_batch + g * p.stride_head) * 2;
    const char* ktr = reinterpret_cast<const char*>(p.k_tree) + ((int64_t)b * p.Nmax * p.Hkv + g) * (D * 2);
    const char* vtr = reinterpret_cast<const char*>(p.v_tree) + ((int64_t)b * p.Nmax * p.Hkv + g) * (D * 2);

    auto locate = [&](int blk) {
      BlockSrc src;
      if (blk < n_prefix_blocks) {
        const int key0 = blk * kBlockKeys;
        const int64_t byte0 = (int64_t)key0 * cache_row_bytes;
        src.k = kc + byte0;
        src.v = vc + byte0;
        src.row_bytes = cache_row_bytes;
        src.nvalid = min(kBlockKeys, L - key0);
        src.kind = src.nvalid == kBlockKeys ? 0 : 1;
        src.tree_key0 = 0;
      } else {
        const int t0 = (blk - n_prefix_blocks) * kBlockKeys;
        src.k = ktr + t0 * tree_row_bytes;
        src.v = vtr + t0 * tree_row_bytes;
        src.row_bytes = tree_row_bytes;
        src.nvalid = min(kBlockKeys, n - t0);
        src.kind = 2;
        src.tree_key0 = t0;
      }
      return src;
    };

    // The stream's first block is requested before anything else is set up. Small tiles (two
    // wavefronts per SIMD) keep one K and one V block in registers: K of the next block is requested
    // right after the scores of this one, V of the next block once this block's products are issued.
    // Large tiles (one wavefront per SIMD) request K of the next block at the top of this one into a
    // second buffer and V of the next block as soon as this block's V has been transposed, into the
    // registers that frees.
    bf16x8 kf[2][KS], kfn[kDeep ? 2 : 1][KS];
    unsigned vr[8][D / 32];
    unsigned koff[2], voff[8];
    unsigned k_rb = 0, v_rb = 0;   // row pitch and row count the offsets were last computed for
    int k_nv = 0, v_nv = 0;
    auto set_k = [&](const BlockSrc& s) {
      if (s.row_bytes != k_rb || s.nvalid != k_nv) {
        k_offsets(koff, s.row_bytes, s.nvalid, col, g4);
        k_rb = s.row_bytes; k_nv = s.nvalid;
      }
    };
    auto set_v = [&](const BlockSrc& s) {
      if (s.row_bytes != v_rb || s.nvalid != v_nv) {
        v_offsets<D>(voff, s.row_bytes, s.nvalid, col, g4);
        v_rb = s.row_bytes; v_nv = s.nvalid;
      }
    };
    BlockSrc cur{};
    if (active) {
      cur = locate(blk_begin);
      set_k(cur);
      load_k<D>(kf, cur.k, koff);
      set_v(cur);
      load_v<D>(vr, cur.v, voff);
    }

    // row of this lane in tile t: query row rr of the kv head's N*G rows = (node, head within group)
    struct RowInfo { bool exists, valid; int node; int64_t out; };
    auto row_info = [&](int t) {
      RowInfo ri;
      const int rr = slab * ROWS + 16 * t + col;
      ri.node = (int)div_magic((unsigned)rr, p.G, p.g_magic);
      const int hl = rr - ri.node * p.G;
      ri.exists = slab_live && rr < p.Nmax * p.G;
      ri.valid = ri.exists && ri.node < n;
      ri.out = ((int64_t)b * p.Nmax + ri.node) * p.Hq + g * p.G + hl;  // index of (b, node, h)
      return ri;
    };
    // every load of the set-up is issued before the first value of any of them is needed (memory
    // returns in order, so a wait for one is a wait for everything requested before it)
    bf16x8 qf[kQInLds ? 1 : QT][KS];
    uint64_t tree_mask[QT];  // ancestor words of the lane's rows (used by the tree blocks only)
    bf16x8 qtmp[kQInLds ? QT : 1][KS];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      const RowInfo ri = row_info(t);
      const __bf16* qrow = reinterpret_cast<const __bf16*>(p.q) + ri.out * D + 8 * g4;
      tree_mask[t] = ri.valid ? p.anc_mask[b * p.Nmax + ri.node] : 0ull;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 zero;
#pragma unroll
        for (int j = 0; j < 8; ++j) zero[j] = (__bf16)0.f;
        const bf16x8 frag = ri.valid ? *reinterpret_cast<const bf16x8*>(qrow + 32 * ks) : zero;
        if constexpr (kQInLds) qtmp[t][ks] = frag; else qf[t][ks] = frag;
      }
    }
    {
      const uint64_t live_bits = (n >= 64) ? ~0ull : ((1ull << n) - 1ull);
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        tree_mask[t] &= live_bits;
        if constexpr (kQInLds) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) q_lds[(t * KS + ks) * 64] = qtmp[t][ks];
        }
      }
    }
    auto q_frag = [&](int t, int ks) -> bf16x8 {
      if constexpr (kQInLds) return q_lds[(t * KS + ks) * 64]; else return qf[t][ks];
    };
    auto mask_of_tile = [&](int t) -> uint64_t { return tree_mask[t]; };

    RowState<QT, D> st;
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      st.m[t] = kNegBig;
      st.l[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int e = 0; e < DT; ++e) st.o[t][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    if (active) {
      int blk = blk_begin;
      if constexpr (kDeep) {
        // long streams of full prefix blocks: a loop of its own with nothing in it but the steady state
        // (the next block is a full block too, so bases advance by a constant and the offsets stay)
        const int full_end = min(blk_end, L / kBlockKeys);
        if (blk + KW < full_end) {
          const int64_t step = (int64_t)kBlockKeys * cache_row_bytes * KW;
          const char* kb = cur.k;
          const char* vb = cur.v;
          BlockSrc full{};  // kind 0
          full.nvalid = kBlockKeys;
          for (; blk + KW < full_end; blk += KW) {
            asm volatile("" ::: "memory");  // keep the Q reads inside the loop (they are the point)
            kb += step;
            vb += step;
            load_k<D>(kfn, kb, koff);
            process_block<QT, D>(st, kf, vr, q_frag, full, mask_of_tile, c, g4, [] {},
                                 [&] { load_v<D>(vr, vb, voff); });
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
              for (int ks = 0; ks < KS; ++ks) kf[kt][ks] = kfn[kt][ks];
          }
          cur = locate(blk);
        }
      }
      for (;; blk += KW) {
        if constexpr (kQInLds) asm volatile("" ::: "memory");  // keep the Q reads inside the loop (they are the point)
        const bool more = blk + KW < blk_end;
        BlockSrc nxt = cur;
        if (more) nxt = locate(blk + KW);
        if constexpr (kDeep) {
          if (more) { set_k(nxt); load_k<D>(kfn, nxt.k, koff); }
          process_block<QT, D>(st, kf, vr, q_frag, cur, mask_of_tile, c, g4, [] {},
                               [&] { if (more) { set_v(nxt); load_v<D>(vr, nxt.v, voff); } });
          if (more) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
              for (int ks = 0; ks < KS; ++ks) kf[kt][ks] = kfn[kt][ks];
          }
        } else {
          process_block<QT, D>(st, kf, vr, q_frag, cur, mask_of_tile, c, g4,
                               [&] { if (more) { set_k(nxt); load_k<D>(kf, nxt.k, koff); } }, [] {});
          if (more) { set_v(nxt); load_v<D>(vr, nxt.v, voff); }
        }
        if (!more) break;
        cur = nxt;
      }
    }
    float lsum[QT];  // the matrix-core row sums already cover every key of the wavefront's blocks
#pragma unroll
    for (int t = 0; t < QT; ++t) lsum[t] = st.l[t][0];

    // Writes 4 consecutive d-tiles (e0..e0+3) of row tile t: final rows when the segment is the whole
    // unit, a partial slot otherwise. o4[j][i] belongs to dim DT*(4*g4+i)+e0+j of row 16*t+col.
    auto write_quad = [&](int t, int e0, const f32x4 (&o4)[4], float m_row, float l_row) {
      const RowInfo ri = row_info(t);
      if (!ri.exists) return;
      if (whole_unit) {
        const float inv = ri.valid ? 1.0f / l_row : 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int d0 = DT * (4 * g4 + i) + e0;
          float vals[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) vals[j] = ri.valid ? o4[j][i] * inv : 0.f;
          if (p.out_bf16) {
            typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
            bf16x4 pk;
#pragma unroll
            for (int j = 0; j < 4; ++j) pk[j] = (__bf16)vals[j];
            *reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(p.out) + ri.out * D + d0) = pk;
          } else {
            *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(p.out) + ri.out * D + d0) =
                f32x4{vals[0], vals[1], vals[2], vals[3]};
          }
        }
      } else if (ri.valid) {
        float* slot = p.part + (int64_t)(unit + w) * rows_per_unit * (D + 2);
        const int lr = slab_local * ROWS + 16 * t + col;
        if (g4 == 0 && e0 == 0) *reinterpret_cast<float2*>(slot + (int64_t)rows_per_unit * D + 2 * lr) = make_float2(m_row, l_row);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          *reinterpret_cast<f32x4*>(slot + (int64_t)lr * D + DT * (4 * g4 + i) + e0) =
              f32x4{o4[0][i], o4[1][i], o4[2][i], o4[3][i]};
      }
    };

    if (KW > 1) {
      // The key-splitting wavefronts of a slab leave their states in lane-private LDS slots; after one
      // barrier each of them reduces and writes its own share of the (row tile, 4 d-tiles) quads, so
      // the tail of a short-lived workgroup is spread over all its wavefronts.
      if (kQInLds) __syncthreads();  // every wavefront is done with its Q slots before they are overwritten
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        merge_ml[wave][t][lane] = make_float2(st.m[t], lsum[t]);
#pragma unroll
        for (int e = 0; e < DT; ++e) merge_o[wave][t * DT + e][lane] = st.o[t][e];
      }
      __syncthreads();
      constexpr int kQuadsPerTile = DT / 4;
      for (int q = kp; q < QT * kQuadsPerTile; q += KW) {
        const int t = q / kQuadsPerTile, e0 = 4 * (q - t * kQuadsPerTile);
        float mm = kNegBig;
        for (int k = 0; k < KW; ++k) mm = fmaxf(mm, merge_ml[slab_local + k * p.WS][t][lane].x);
        float l_row = 0.f;
        f32x4 o4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) o4[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < KW; ++k) {  // in wavefront order: deterministic
          const int peer = slab_local + k * p.WS;
          const float2 ml = merge_ml[peer][t][lane];
          const float a = __builtin_amdgcn_exp2f(ml.x - mm);
          l_row += ml.y * a;
#pragma unroll
          for (int j = 0; j < 4; ++j) o4[j] += merge_o[peer][t * DT + e0 + j][lane] * a;
        }
        write_quad(t, e0, o4, mm, l_row);
      }
    } else {
#pragma unroll
      for (int t = 0; t < QT; ++t)
#pragma unroll
        for (int e0 = 0; e0 < DT; e0 += 4) {
          const f32x4 o4[4] = {st.o[t][e0], st.o[t][e0 + 1], st.o[t][e0 + 2], st.o[t][e0 + 3]};
          write_quad(t, e0, o4, st.m[t], lsum[t]);
        }
    }
    r += (unsigned)seg_count;
    if (b + 1 < p.B && r >= seq_first_block(p, b + 1)) ++b;
    if ((KW > 1 || kQInLds) && r < r1) __syncthreads();  // the LDS buffers are reused by the next segment
  }
}

// ---------------------------------------------------------------------------------------------
// GQA with many query rows per kv head: four wavefronts per workgroup, 32 rows each (128 rows of
// one kv head), two such sets per compute unit, i.e. two wavefronts per SIMD, so that the matrix
// work of one can run beside the vector work and the waits of the other (vector instructions behind a
// matrix instruction of the same wavefront do not overlap it on this machine). At 32 rows a wavefront
// cannot afford to fetch every K/V block for itself (four to eight copies of each block through the
// texture path is what would bound the kernel): the workgroup fetches each block once, every
// wavefront copying a quarter of it into an LDS stage with the global-to-LDS load (row-contiguous
// requests, no registers), and all of them pick their operands out of the stage. K is kept swizzled
// (16-byte chunk c of row r at slot c ^ f(r)) so that a fragment read, 16 rows by one chunk, touches
// 16 different bank groups; V (D = 128) is read with the transposing LDS load of gfx950, which hands
// every lane the four keys of one dim -- the A operand of V^T P^T as it is, without byte permutes
// (its 32-byte pieces are swizzled too). Three stages of one block each: stage i is read while i+1
// and i+2 are in flight. (WAVES and the blocks per stage are template parameters; only the
// four-wavefront, one-block form is instantiated.)
template <int D, int WAVES>
struct Stage {
  static constexpr int kChunks = D / 8;                      // 16-byte chunks per row
  static constexpr int kRowsPerLoad = 64 / kChunks;          // rows one copy instruction covers
  static constexpr int kLoads = kBlockKeys / kRowsPerLoad;   // copy instructions per tensor and block
  static constexpr int kTensorBytes = kBlockKeys * D * 2;
  static constexpr int kBytes = 2 * kTensorBytes;            // K then V
  static constexpr int kPerWave = 2 * kLoads / WAVES;        // copy instructions per wavefront and block
  __device__ static __forceinline__ int swizzle(int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); }
  // V, D = 128: read with the transposing LDS load, 16 lanes x 8 bytes = 4 keys x 32 bytes at a time;
  // 32-byte piece e of key r sits at piece e ^ (r & 7), so that the 16 keys one instruction touches
  // spread over all banks. D = 64: row-major, read as rows.
  __device__ static __forceinline__ int v_swizzle(int r) { return D == 128 ? 2 * (r & 7) : 0; }
};
typedef const __attribute__((address_space(1))) void* GlobalPtr;
typedef __attribute__((address_space(3))) void* LdsPtr;

// KG key groups: with KG = 2 (3 for head dim 64) a workgroup is two (three) such sets of four wavefronts on the same 128 rows;
// the sets take alternate blocks of the workgroup's segment, each through three stages of its own,
// and merge their states through LDS at the segment's end. One workgroup of eight wavefronts per
// compute unit holds as many wavefronts as two of four, but a cut unit leaves one partial result
// per workgroup: half as many partial bytes are written and read back.
template <int D, int WAVES, int KG>
__global__ __launch_bounds__(64 * WAVES * KG, (KG == 1 ? 2 : 1)) void tree_attn_gqa_kernel(const AttnParams) {
  const AttnArgs p = fetch_args();
  typedef Stage<D, WAVES> S;
  constexpr int QT = 2, KS = D / 32, DT = D / 16, ROWS = 32, kWaves = WAVES, kStages = 3;
  constexpr int kGroup = 1;   // blocks per stage
  constexpr int kStageBytes = kGroup * S::kBytes;
  constexpr int kGroupBytes = kStages * kStageBytes;
  // the merge of two key groups needs (DT + 1) 16-byte slots per lane, tile and wavefront of one group
  constexpr int kMergeBytes = (KG - 1) * kWaves * QT * (DT + 1) * 64 * 16;
  constexpr int kLdsBytes = KG * kGroupBytes > kMergeBytes ? KG * kGroupBytes : kMergeBytes;
  __shared__ __attribute__((aligned(16))) char lds_all[kLdsBytes];

  const int lane = threadIdx.x & 63, wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kg = KG == 1 ? 0 : wave_all / kWaves;          // key group of this wavefront
  const int wave = KG == 1 ? wave_all : wave_all % kWaves; // its row slab within the workgroup
  char* const stages = lds_all + kg * kGroupBytes;
  const int col = lane & 15, g4 = lane >> 4;
  const float c = p.scale * kLog2e;
  const unsigned tree_row_bytes = (unsigned)p.Hkv * D * 2u;
  const unsigned cache_row_bytes = (unsigned)p.stride_token * 2u;
  constexpr int rows_per_unit = kWaves * ROWS;

  // this wavefront's copy instructions: index x < kLoads is K rows, the others V rows
  int dma_tensor[S::kPerWave], dma_row[S::kPerWave], dma_chunk[S::kPerWave], dma_dst[S::kPerWave];
#pragma unroll
  for (int i = 0; i < S::kPerWave; ++i) {
    const int x = wave + kWaves * i;
    const int n = x % S::kLoads;
    dma_tensor[i] = x / S::kLoads;
    dma_row[i] = n * S::kRowsPerLoad + lane / S::kChunks;
    const int chunk = lane & (S::kChunks - 1);
    dma_chunk[i] = dma_tensor[i] == 0 ? (chunk ^ S::swizzle(dma_row[i])) : (chunk ^ S::v_swizzle(dma_row[i]));
    dma_dst[i] = dma_tensor[i] * S::kTensorBytes + n * 1024;
  }
  // this lane's operand reads: K fragments (key tile 0; tile 1 is 16 rows further), V rows
  unsigned kfrag[KS], vrow[8];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) kfrag[ks] = (unsigned)col * (D * 2) + 16u * ((4 * ks + g4) ^ S::swizzle(col));
#pragma unroll
  for (int j = 0; j < 8; ++j) vrow[j] = S::kTensorBytes + (unsigned)key_of(g4, j) * (D * 2) + (unsigned)(D / 8) * col;
  // transposing read (D = 128): lane (col, g4) points at key 4*g4 + col/4 (+16 for the second half),
  // dims 16e + 4*(col%4) .. +3, and receives dims 16e + col of the group's four keys
  const unsigned vtr_off = S::kTensorBytes + (unsigned)(4 * g4 + (col >> 2)) * (D * 2) + 8u * (col & 3) +
                       ((unsigned)((4 * g4 + (col >> 2)) & 7) << 5);

  const unsigned w = blockIdx.x;
  const unsigned wr = w * (unsigned)p.wg_rem, wq = wr / (unsigned)p.n_wgs;
  const unsigned r0 = w * (unsigned)p.wg_quot + wq;
  const unsigned r1 = r0 + (unsigned)p.wg_quot + ((wr - wq * (unsigned)p.n_wgs) + (unsigned)p.wg_rem >= (unsigned)p.n_wgs ? 1u : 0u);
  int b = seq_of_block(p, r0);

  for (unsigned r = r0; r < r1;) {
    const int n = seq_nodes(p, b);
    const int L = seq_len(p, b);
    const int n_prefix_blocks = (L + kBlockKeys - 1) / kBlockKeys;
    const int n_blocks = n_prefix_blocks + (n + kBlockKeys - 1) / kBlockKeys;
    const unsigned rel = r - seq_first_block(p, b);
    const int ub = (int)(rel / (unsigned)n_blocks);
    const int seg_begin = (int)(rel - (unsigned)ub * (unsigned)n_blocks);
    const int seg_count = min(n_blocks - seg_begin, (int)(r1 - r));
    const int g = (int)div_magic((unsigned)ub, p.GY, p.gy_magic), y = ub - g * p.GY;
    const int unit = b * p.Hkv * p.GY + ub;
    const bool whole_unit = seg_count == n_blocks;
    const int slab = y * kWaves + wave;
    const bool slab_live = slab < p.NS;

    const char* kc = reinterpret_cast<const char*>(p.k_cache) + (b * p.stride_batch + g * p.stride_head) * 2;
    const char* vc = reinterpret_cast<const char*>(p.v_cache) + (b * p.stride_batch + g * p.stride_head) * 2;
    const char* ktr = reinterpret_cast<const char*>(p.k_tree) + ((int64_t)b * p.Nmax * p.Hkv + g) * (D * 2);
    const char* vtr = reinterpret_cast<const char*>(p.v_tree) + ((int64_t)b * p.Nmax * p.Hkv + g) * (D * 2);

    auto locate = [&](int blk) {
      BlockSrc src;
      if (blk < n_prefix_blocks) {
        const int key0 = blk * kBlockKeys;
        const int64_t byte0 = (int64_t)key0 * cache_row_bytes;
        src.k = kc + byte0;
        src.v = vc + byte0;
        src.row_bytes = cache_row_bytes;
        src.nvalid = min(kBlockKeys, L - key0);
        src.kind = src.nvalid == kBlockKeys ? 0 : 1;
        src.tree_key0 = 0;
      } else {
        const int t0 = (blk - n_prefix_blocks) * kBlockKeys;
        src.k = ktr + t0 * tree_row_bytes;
        src.v = vtr + t0 * tree_row_bytes;
        src.row_bytes = tree_row_bytes;
        src.nvalid = min(kBlockKeys, n - t0);
        src.kind = 2;
        src.tree_key0 = t0;
      }
      return src;
    };
    // request this wavefront's share of a block into slot u of a stage (rows past the end are clamped; masked later)
    auto request_block = [&](const BlockSrc& s, int stage, int u) {
#pragma unroll
      for (int i = 0; i < S::kPerWave; ++i) {
        const unsigned off = (unsigned)min(dma_row[i], s.nvalid - 1) * s.row_bytes + 16u * dma_chunk[i];
        const char* src = (dma_tensor[i] == 0 ? s.k : s.v) + off;
        __builtin_amdgcn_global_load_lds((GlobalPtr)src, (LdsPtr)(stages + stage * kStageBytes + u * S::kBytes + dma_dst[i]), 16, 0, 0);
      }
    };
    // key group kg takes blocks kg, kg + KG, ... of the segment
    const int blk_begin = seg_begin + kg, blk_end = seg_begin + seg_count;
    auto request_group = [&](int first, int stage) {
      if (first < blk_end) request_block(locate(first), stage, 0);
    };
    auto group_size = [&](int first) { return first < blk_end ? 1 : 0; };

    request_group(blk_begin, 0);
    request_group(blk_begin + KG, 1);

    struct RowInfo { bool exists, valid; int node; int64_t out; };
    auto row_info = [&](int t) {
      RowInfo ri;
      const int rr = slab * ROWS + 16 * t + col;
      ri.node = (int)div_magic((unsigned)rr, p.G, p.g_magic);
      const int hl = rr - ri.node * p.G;
      ri.exists = slab_live && rr < p.Nmax * p.G;
      ri.valid = ri.exists && ri.node < n;
      ri.out = ((int64_t)b * p.Nmax + ri.node) * p.Hq + g * p.G + hl;
      return ri;
    };
    bf16x8 qf[QT][KS];
    uint64_t tree_mask[QT];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      const RowInfo ri = row_info(t);
      const __bf16* qrow = reinterpret_cast<const __bf16*>(p.q) + ri.out * D + 8 * g4;
      tree_mask[t] = ri.valid ? p.anc_mask[b * p.Nmax + ri.node] : 0ull;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 zero;
#pragma unroll
        for (int j = 0; j < 8; ++j) zero[j] = (__bf16)0.f;
        qf[t][ks] = ri.valid ? *reinterpret_cast<const bf16x8*>(qrow + 32 * ks) : zero;
      }
    }
    {
      const uint64_t live_bits = (n >= 64) ? ~0ull : ((1ull << n) - 1ull);
#pragma unroll
      for (int t = 0; t < QT; ++t) tree_mask[t] &= live_bits;
    }
    auto q_frag = [&](int t, int ks) -> bf16x8 { return qf[t][ks]; };
    auto mask_of_tile = [&](int t) -> uint64_t { return tree_mask[t]; };

    RowState<QT, D> st;
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      st.m[t] = kNegBig;
      st.l[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int e = 0; e < DT; ++e) st.o[t][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    int stage = 0;
    // every wavefront of the workgroup takes the same number of turns (the barriers are the whole
    // workgroup's): as many as key group 0 has blocks; a group whose blocks have run out idles
    const int n_turns = (seg_count + KG - 1) / KG;
    for (int turn = 0, first = blk_begin; turn < n_turns; ++turn, first += KG) {
      // this turn's copies have landed (the next turn's, requested after them, may still be in
      // flight); the barrier makes every wavefront's share visible and retires the stage that the
      // turn after the next is about to overwrite
      const int next_size = group_size(first + KG);
      if (next_size == 1) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(S::kPerWave) : "memory");
      else asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
      __syncthreads();
      request_group(first + 2 * KG, stage == 0 ? 2 : stage - 1);
      if (slab_live && first < blk_end) {
        {
          const BlockSrc cur = locate(first);
          const char* sbase = stages + stage * kStageBytes;
          bf16x8 kf[2][KS];
          unsigned vr[8][D / 32];
#pragma unroll
          for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
              kf[kt][ks] = *reinterpret_cast<const bf16x8*>(sbase + kt * 16 * (D * 2) + kfrag[ks]);
          if constexpr (D == 128) {
            // The transposing reads are written out as instructions: through the builtin the compiler
            // cannot tell them from the stages that the copies requested above are still filling, and
            // waits for every copy in flight (vmcnt(0)) before the first of them, which serialises the
            // prefetch. This stage's copies have landed (the wait and the barrier above).
            const unsigned sb = (unsigned)(uintptr_t)(LdsPtr)(sbase);
            u32x2 tr[2 * DT];
#pragma unroll
            for (int e = 0; e < DT; ++e) {
              const unsigned a0 = sb + (vtr_off ^ ((unsigned)e << 5));
              asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(tr[2 * e]) : "v"(a0));
              asm volatile("ds_read_b64_tr_b16 %0, %1 offset:4096" : "=v"(tr[2 * e + 1]) : "v"(a0));
            }
            static_assert(16 * (D * 2) == 4096, "second half of the keys: 16 rows further");
            asm volatile("s_waitcnt lgkmcnt(0)"
                         : "+v"(tr[0]), "+v"(tr[1]), "+v"(tr[2]), "+v"(tr[3]), "+v"(tr[4]), "+v"(tr[5]), "+v"(tr[6]), "+v"(tr[7]),
                           "+v"(tr[8]), "+v"(tr[9]), "+v"(tr[10]), "+v"(tr[11]), "+v"(tr[12]), "+v"(tr[13]), "+v"(tr[14]), "+v"(tr[15]));
            unsigned* flat = &vr[0][0];
#pragma unroll
            for (int e = 0; e < DT; ++e) {
              flat[4 * e] = tr[2 * e][0]; flat[4 * e + 1] = tr[2 * e][1]; flat[4 * e + 2] = tr[2 * e + 1][0]; flat[4 * e + 3] = tr[2 * e + 1][1];
            }
            process_block<QT, D, true>(st, kf, vr, q_frag, cur, mask_of_tile, c, g4, [] {}, [] {});
          } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              const u32x2 x = *reinterpret_cast<const u32x2*>(sbase + vrow[j]);
              vr[j][0] = x[0]; vr[j][1] = x[1];
            }
            process_block<QT, D>(st, kf, vr, q_frag, cur, mask_of_tile, c, g4, [] {}, [] {});
          }
        }
      }
      stage = stage == 2 ? 0 : stage + 1;
    }

    if constexpr (KG >= 2) {
      // the other key groups hand their states over in lane-private LDS slots (the stages are free
      // once every wavefront has left the loop); wavefront w of the first group and wavefront w of the
      // second hold the same rows in the same lanes, so the merge is lane by lane and in a fixed order
      __syncthreads();
      constexpr int kGroupSlots = kWaves * QT * (DT + 1) * 64;   // 16-byte slots one group hands over
      f32x4* const mbuf0 = reinterpret_cast<f32x4*>(lds_all) + (wave * QT * (DT + 1)) * 64 + lane;
      if (kg >= 1 && slab_live) {
        f32x4* mbuf = mbuf0 + (kg - 1) * kGroupSlots;
#pragma unroll
        for (int t = 0; t < QT; ++t) {
#pragma unroll
          for (int e = 0; e < DT; ++e) mbuf[(t * (DT + 1) + e) * 64] = st.o[t][e];
          mbuf[(t * (DT + 1) + DT) * 64] = f32x4{st.m[t], st.l[t][0], 0.f, 0.f};
        }
      }
      __syncthreads();
      if (kg == 0 && slab_live) {
#pragma unroll
        for (int other = 1; other < KG; ++other) {   // in group order: deterministic
        const f32x4* mbuf = mbuf0 + (other - 1) * kGroupSlots;
#pragma unroll
        for (int t = 0; t < QT; ++t) {
          const f32x4 ml = mbuf[(t * (DT + 1) + DT) * 64];
          const float mm = fmaxf(st.m[t], ml[0]);
          const float a0 = __builtin_amdgcn_exp2f(st.m[t] - mm), a1 = __builtin_amdgcn_exp2f(ml[0] - mm);
          st.m[t] = mm;
          st.l[t] = st.l[t] * a0 + ml[1] * a1;
#pragma unroll
          for (int e = 0; e < DT; ++e) st.o[t][e] = st.o[t][e] * a0 + mbuf[(t * (DT + 1) + e) * 64] * a1;
        }
        }
      }
    }

    // every wavefront (of the first key group) owns its rows: final rows or a partial slot, straight from registers
    if (slab_live && kg == 0) {
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        const RowInfo ri = row_info(t);
        if (!ri.exists) continue;
        const float l_row = st.l[t][0];
        if constexpr (D == 128) {
          // operands from the transposing read: accumulator e holds dims 16e + 4*g4 .. +3
          const float inv = ri.valid ? 1.0f / l_row : 0.f;
          float* slot = p.part + (int64_t)(unit + w) * rows_per_unit * (D + 2);
          const int lr = wave * ROWS + 16 * t + col;
          if (!whole_unit && ri.valid && g4 == 0)
            *reinterpret_cast<float2*>(slot + (int64_t)rows_per_unit * D + 2 * lr) = make_float2(st.m[t], l_row);
#pragma unroll
          for (int e = 0; e < DT; ++e) {
            const int d0 = 16 * e + 4 * g4;
            if (whole_unit) {
              float vals[4];
#pragma unroll
              for (int i = 0; i < 4; ++i) vals[i] = ri.valid ? st.o[t][e][i] * inv : 0.f;
              if (p.out_bf16) {
                typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
                bf16x4 pk;
#pragma unroll
                for (int i = 0; i < 4; ++i) pk[i] = (__bf16)vals[i];
                *reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(p.out) + ri.out * D + d0) = pk;
              } else {
                *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(p.out) + ri.out * D + d0) =
                    f32x4{vals[0], vals[1], vals[2], vals[3]};
              }
            } else if (ri.valid) {
              *reinterpret_cast<f32x4*>(slot + (int64_t)lr * D + d0) = st.o[t][e];
            }
          }
          continue;
        }
#pragma unroll
        for (int e0 = 0; e0 < DT; e0 += 4) {
          if (whole_unit) {
            const float inv = ri.valid ? 1.0f / l_row : 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int d0 = DT * (4 * g4 + i) + e0;
              float vals[4];
#pragma unroll
              for (int j = 0; j < 4; ++j) vals[j] = ri.valid ? st.o[t][e0 + j][i] * inv : 0.f;
              if (p.out_bf16) {
                typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
                bf16x4 pk;
#pragma unroll
                for (int j = 0; j < 4; ++j) pk[j] = (__bf16)vals[j];
                *reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(p.out) + ri.out * D + d0) = pk;
              } else {
                *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(p.out) + ri.out * D + d0) =
                    f32x4{vals[0], vals[1], vals[2], vals[3]};
              }
            }
          } else if (ri.valid) {
            float* slot = p.part + (int64_t)(unit + w) * rows_per_unit * (D + 2);
            const int lr = wave * ROWS + 16 * t + col;
            if (g4 == 0 && e0 == 0) *reinterpret_cast<float2*>(slot + (int64_t)rows_per_unit * D + 2 * lr) = make_float2(st.m[t], l_row);
#pragma unroll
            for (int i = 0; i < 4; ++i)
              *reinterpret_cast<f32x4*>(slot + (int64_t)lr * D + DT * (4 * g4 + i) + e0) =
                  f32x4{st.o[t][e0][i], st.o[t][e0 + 1][i], st.o[t][e0 + 2][i], st.o[t][e0 + 3][i]};
          }
        }
      }
    }
    r += (unsigned)seg_count;
    if (b + 1 < p.B && r >= seq_first_block(p, b + 1)) ++b;
    __syncthreads();  // every wavefront is done with the stages before the next segment refills them
  }
}

// Workgroup that owns flat block x under the even split: the w with first(w) <= x < first(w+1).
// A float estimate (off by one at most for the sizes a launch can have) and a correction.
__device__ __forceinline__ int owner_of(const AttnArgs& p, unsigned x) {
  int w = (int)((float)x * ((float)p.n_wgs / (float)p.total_blocks));
  w = min(w, p.n_wgs - 1);
  while (w > 0 && wg_first_block(p, (unsigned)w) > x) --w;
  while (w + 1 < p.n_wgs && wg_first_block(p, (unsigned)w + 1u) <= x) ++w;
  return w;
}

// Finishes every unit that was cut into several segments:
// out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s over the unit's partial slots.
// One thread per 4 output dims; rows of nodes past n_nodes are written as zeros.
template <int D>
__global__ __launch_bounds__(256) void tree_attn_combine_kernel(const AttnParams, int rows_per_slab) {
  const AttnArgs p = fetch_args();
  constexpr int TPR = D / 4;  // threads per row
  const int unit = blockIdx.y;
  const int units_per_seq = p.Hkv * p.GY;
  const int b = unit / units_per_seq, ub = unit - b * units_per_seq;
  const int g = (int)div_magic((unsigned)ub, p.GY, p.gy_magic), y = ub - g * p.GY;
  const int n_blocks = (seq_len(p, b) + kBlockKeys - 1) / kBlockKeys + (seq_nodes(p, b) + kBlockKeys - 1) / kBlockKeys;
  const unsigned fs = seq_first_block(p, b) + (unsigned)ub * (unsigned)n_blocks;
  const int w0 = owner_of(p, fs), w1 = owner_of(p, fs + (unsigned)n_blocks - 1u);
  if (w0 == w1) return;  // written directly by the one workgroup that held the whole unit
  const int rows_per_unit = p.WS * rows_per_slab;
  const int lr = blockIdx.x * (256 / TPR) + threadIdx.x / TPR;
  if (lr >= rows_per_unit) return;
  const int d0 = (threadIdx.x % TPR) * 4;
  const int slab_local = lr / rows_per_slab;
  const int rr = (y * p.WS + slab_local) * rows_per_slab + (lr - slab_local * rows_per_slab);
  if (rr >= p.Nmax * p.G) return;
  const int node = (int)div_magic((unsigned)rr, p.G, p.g_magic), hl = rr - node * p.G;
  const int64_t row = ((int64_t)b * p.Nmax + node) * p.Hq + g * p.G + hl;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (node < seq_nodes(p, b)) {
    const int64_t slot_floats = (int64_t)rows_per_unit * (D + 2);
    const float* o_base = p.part + (int64_t)(unit + w0) * slot_floats + (int64_t)lr * D + d0;
    const float* ml_base = p.part + (int64_t)(unit + w0) * slot_floats + (int64_t)rows_per_unit * D + 2 * lr;
    // slots in index order (deterministic), eight at a time so that their loads are in flight together
    float M = kNegBig, denom = 0.f;
    const int n_seg = w1 - w0 + 1;
    for (int s0 = 0; s0 < n_seg; s0 += 8) {
      float2 ml[8];
      f32x4 o[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int sidx = min(s0 + k, n_seg - 1);  // clamped duplicates get zero weight below
        ml[k] = *reinterpret_cast<const float2*>(ml_base + sidx * slot_floats);
        o[k] = *reinterpret_cast<const f32x4*>(o_base + sidx * slot_floats);
      }
      float mx = M;
#pragma unroll
      for (int k = 0; k < 8; ++k) mx = fmaxf(mx, ml[k].x);
      const float a = __builtin_amdgcn_exp2f(M - mx);
      acc *= a;
      denom *= a;
      M = mx;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float wgt = (s0 + k < n_seg) ? __builtin_amdgcn_exp2f(ml[k].x - M) : 0.f;
        denom += wgt * ml[k].y;
        acc += wgt * o[k];
      }
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
  bool shared_stage;   // the kernel whose wavefronts share K/V blocks through LDS (WS = 4 or 8 slabs of 32 rows)
  bool short_stream;   // few blocks per workgroup: one workgroup per compute unit, so that fewer partials are written
  int QT, NS, WS, GY;
  int rows_per_unit;
  int n_wgs;           // workgroups for the largest slice of sequences
  int64_t total_blocks;
};

constexpr int64_t kComputeUnits = 256;
constexpr int64_t kMaxWorkgroups = 32768;
constexpr int64_t kShortStreamBlocks = 16;  // blocks per workgroup below which a stream counts as short
constexpr int kMaxQT = 4;                   // 16-row tiles per wavefront at most
constexpr int kMaxForcedWorkgroups = 4096;  // upper limit of fspad_attn_desc.workgroups

// Row tiling of one kv head's N*G query rows: slabs of 16*QT rows, WS slabs per workgroup.
void plan_rows(const fspad_attn_desc& d, Plan& pl, int max_ws = 4) {
  pl.shared_stage = false;
  pl.short_stream = false;
  const int G = d.n_q_heads / d.n_kv_heads;
  const int rows = d.n_nodes_max * G;
  int best_cost = 1 << 30;
  for (int qt = kMaxQT; qt >= 1; --qt) {  // ties go to the larger tile: fewer re-reads of K/V
    const int ns = (rows + 16 * qt - 1) / (16 * qt);
    int ws = ns == 1 ? 1 : (ns == 2 ? 2 : 4);
    if (ws > max_ws) ws = max_ws;
    const int gy = (ns + ws - 1) / ws;
    const int cost = gy * ws * qt;
    if (cost < best_cost) { best_cost = cost; pl.QT = qt; pl.NS = ns; pl.WS = ws; pl.GY = gy; }
  }
  pl.rows_per_unit = pl.WS * 16 * pl.QT;
}

// The shared-stage kernel's plan: 32-row slabs, one per wavefront, four per workgroup.
bool gqa_plan_applies(const fspad_attn_desc& d) {
  return d.n_nodes_max * (d.n_q_heads / d.n_kv_heads) > 4 * 32;
}
void plan_rows_gqa(const fspad_attn_desc& d, Plan& pl) {
  pl.shared_stage = true;
  pl.short_stream = false;
  pl.QT = 2;
  pl.NS = (d.n_nodes_max * (d.n_q_heads / d.n_kv_heads) + 31) / 32;
  pl.WS = 4;
  pl.GY = (pl.NS + pl.WS - 1) / pl.WS;
  pl.rows_per_unit = 32 * pl.WS;
}

int blocks_of(int kv_len, int n_nodes) {
  return (kv_len + kBlockKeys - 1) / kBlockKeys + (n_nodes + kBlockKeys - 1) / kBlockKeys;
}

// Workgroup count for `total_blocks` flat blocks in `units` units: two resident workgroups per
// compute unit when the register budget allows it (one otherwise), but no workgroup with fewer
// than 2 blocks per key-splitting wave. When all units are equally long and short (a few blocks
// per wave), the count is a multiple of the unit count whenever that still fills three quarters of
// the compute units: every unit is then cut into the same number of pieces and no workgroup
// straddles two units (a second segment costs a short-lived workgroup as much as its blocks do).
// With one piece per unit nothing is cut and nothing is merged.
int plan_wgs(const Plan& pl, int64_t total_blocks, int64_t units, bool uniform, int forced) {
  // wavefront sets that split a workgroup's keys: the two key groups of the shared-stage kernel, or
  // the wavefronts that do not take a row slab of their own
  const int KW = pl.shared_stage ? 2 : (pl.WS >= 4 ? 1 : 4 / pl.WS);
  // (the shared-stage kernel's eight wavefronts of up to 256 registers fill a compute unit by themselves)
  const int64_t resident = (pl.QT <= 2 && !pl.shared_stage) ? 512 : 256;
  int64_t wgs = resident;
  const int64_t cap = total_blocks / (2 * KW);
  if (wgs > cap) wgs = cap;
  if (uniform && units <= total_blocks) {
    const int64_t rounds = (units + resident - 1) / resident;
    if (4 * units >= 3 * rounds * resident) {
      wgs = units;
    } else if (units <= kComputeUnits) {
      // short units: one workgroup per compute unit at most, since a second one on the same unit
      // shares its instruction issue and finishes last
      const int64_t blocks_per_unit = total_blocks / units;
      int64_t pieces = (blocks_per_unit + 2 * KW - 1) / (2 * KW);
      if (pieces > kComputeUnits / units) pieces = kComputeUnits / units;
      const bool short_pieces = pieces >= 1 && blocks_per_unit <= 4 * KW * pieces;  // at most 4 blocks per wave
      if (short_pieces && 4 * units * pieces >= 3 * (wgs < kComputeUnits ? wgs : kComputeUnits)) wgs = units * pieces;
    }
  }
  if (forced > 0) wgs = forced < kMaxForcedWorkgroups ? forced : kMaxForcedWorkgroups;
  if (wgs > kMaxWorkgroups) wgs = kMaxWorkgroups;  // the kernels form w * (T mod W) in 32 bits
  if (wgs > total_blocks) wgs = total_blocks;
  if (wgs < 1) wgs = 1;
  return (int)wgs;
}

int host_owner_of(int64_t x, int64_t T, int W) {
  int w = (int)((x * W) / T);
  if (((int64_t)(w + 1) * T) / W <= x) ++w;
  return w;
}

size_t slot_bytes(const fspad_attn_desc& d, const Plan& pl) {
  return (size_t)pl.rows_per_unit * (d.head_dim + 2) * sizeof(float);
}

fspad_status check_desc(const fspad_attn_desc* d) {
  if (!d) return FSPAD_ERR_NULL;
  if (d->batch < 1 || d->n_nodes_max < 1 || d->n_nodes_max > FSPAD_MAX_NODES) return FSPAD_ERR_SHAPE;
  if (d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_q_heads % d->n_kv_heads != 0) return FSPAD_ERR_SHAPE;
  if (d->head_dim != 64 && d->head_dim != 128) return FSPAD_ERR_SHAPE;
  if ((int64_t)d->n_kv_heads * d->head_dim > (1ll << 26)) return FSPAD_ERR_SHAPE;  // 32-bit byte offsets inside a block
  if (d->io_dtype != FSPAD_F32 && d->io_dtype != FSPAD_BF16) return FSPAD_ERR_DTYPE;
  if (d->out_dtype != FSPAD_F32 && d->out_dtype != d->io_dtype) return FSPAD_ERR_DTYPE;
  if (!(d->softmax_scale >= 0.f) || d->softmax_scale > 3.0e38f) return FSPAD_ERR_SHAPE;
  if (d->workgroups < 0) return FSPAD_ERR_SHAPE;
  return FSPAD_OK;
}

template <int D>
void launch_bf16(const Plan& pl, const AttnParams& prm, hipStream_t stream) {
  const dim3 grid((unsigned)prm.n_wgs);
  switch (pl.QT) {
    case 1: hipLaunchKernelGGL((tree_attn_bf16_kernel<1, D>), grid, dim3(256), 0, stream, prm); break;
    case 2: hipLaunchKernelGGL((tree_attn_bf16_kernel<2, D>), grid, dim3(256), 0, stream, prm); break;
    case 3: hipLaunchKernelGGL((tree_attn_bf16_kernel<3, D>), grid, dim3(256), 0, stream, prm); break;
    default: hipLaunchKernelGGL((tree_attn_bf16_kernel<4, D>), grid, dim3(256), 0, stream, prm); break;
  }
}

}  // namespace

extern "C" size_t fspad_tree_attn_workspace_bytes(const fspad_attn_desc* desc, int32_t max_kv_len) {
  if (check_desc(desc) != FSPAD_OK || max_kv_len < 0) return 0;
  if (desc->io_dtype == FSPAD_F32) return 16;
  // one partial slot per (unit, workgroup) boundary at most: units + workgroups of the largest slice;
  // the call may settle on either slab count (see kShortStreamBlocks), so both are sized
  size_t need = 0;
  for (int variant = 0; variant < 3; ++variant) {   // four slabs, two slabs, the shared-stage plan
    Plan pl{};
    if (variant < 2) plan_rows(*desc, pl, variant == 0 ? 4 : 2);
    else if (gqa_plan_applies(*desc)) plan_rows_gqa(*desc, pl);
    else break;
    const int nb = desc->batch < kMaxBatchPerLaunch ? desc->batch : kMaxBatchPerLaunch;
    const int64_t units = (int64_t)nb * desc->n_kv_heads * pl.GY;
    const int64_t total = units * blocks_of(max_kv_len, desc->n_nodes_max);
    int64_t wgs = plan_wgs(pl, total, units, true, desc->workgroups);
    const int64_t wgs_cut = plan_wgs(pl, total, units, false, desc->workgroups);  // a ragged batch of the same size
    if (wgs_cut > wgs) wgs = wgs_cut;
    const int64_t slots = units + wgs;
    const size_t bytes = (size_t)slots * slot_bytes(*desc, pl);
    if (bytes > need) need = bytes;
  }
  return need;
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
    if (d.cache_stride_token < d.head_dim || d.cache_stride_token > (1ll << 26) || d.cache_stride_token % align || d.cache_stride_head % align ||
        d.cache_stride_batch % align || d.cache_stride_head < 0 || d.cache_stride_batch < 0)
      return FSPAD_ERR_SHAPE;
    if (((uintptr_t)k_cache | (uintptr_t)v_cache) & 15) return FSPAD_ERR_SHAPE;
  }
  if (((uintptr_t)q | (uintptr_t)k_tree | (uintptr_t)v_tree | (uintptr_t)out) & 15) return FSPAD_ERR_SHAPE;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);

  AttnParams prm{};
  prm.anc_mask = anc_mask;
  prm.stride_batch = d.cache_stride_batch; prm.stride_head = d.cache_stride_head; prm.stride_token = d.cache_stride_token;
  prm.Nmax = d.n_nodes_max; prm.Hq = d.n_q_heads; prm.Hkv = d.n_kv_heads;
  prm.G = d.n_q_heads / d.n_kv_heads;
  prm.out_bf16 = d.out_dtype == FSPAD_BF16;
  prm.scale = d.softmax_scale > 0.f ? d.softmax_scale : 1.0f / sqrtf((float)d.head_dim);
  prm.WS = 1; prm.NS = 1; prm.GY = 1;
  prm.g_magic = prm.G > 1 ? (uint32_t)(((1ull << 32) + prm.G - 1) / prm.G) : 0u;

  if (d.io_dtype == FSPAD_BF16) prm.part = reinterpret_cast<float*>(workspace);

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
    for (int i = 0; i < nb; ++i) { sl.kv_len[i] = kv_len[b0 + i]; sl.n_nodes[i] = n_nodes[b0 + i]; }
    if (d.io_dtype == FSPAD_BF16) {
      bool uniform = true;
      int64_t seq_blocks = 0;
      for (int i = 0; i < nb; ++i) {
        uniform = uniform && blocks_of(sl.kv_len[i], sl.n_nodes[i]) == blocks_of(sl.kv_len[0], sl.n_nodes[0]);
        seq_blocks += blocks_of(sl.kv_len[i], sl.n_nodes[i]);
      }
      // Four row slabs per workgroup share every K/V block between its four wavefronts, but the
      // partial results of a cut unit grow with the rows a workgroup holds. With short streams
      // (few blocks per workgroup) those partials outweigh the K/V bytes: two slabs then.
      Plan pl{};
      plan_rows(d, pl);
      if (pl.WS == 4) {
        const int64_t units4 = (int64_t)nb * d.n_kv_heads * pl.GY;
        const int64_t total4 = (int64_t)d.n_kv_heads * pl.GY * seq_blocks;
        const bool short_stream = total4 < kShortStreamBlocks * plan_wgs(pl, total4, units4, uniform, d.workgroups);
        if (gqa_plan_applies(d)) {
          // more than four 32-row slabs per kv head: wavefronts of 32 rows that share every K/V
          // block through LDS (measured on a 32/8-head layer, 4096 keys, 60 nodes: 24.9 us against
          // 29.9 us for 64-row tiles with two slabs); with short streams one workgroup per compute unit
          plan_rows_gqa(d, pl);
          pl.short_stream = short_stream;
        } else if (short_stream) {
          plan_rows(d, pl, 2);
        }
      }
      sl.WS = pl.WS; sl.NS = pl.NS; sl.GY = pl.GY;
      sl.ws_shift = pl.WS == 4 ? 2 : (pl.WS == 2 ? 1 : 0);
      sl.gy_magic = pl.GY > 1 ? (uint32_t)(((1ull << 32) + pl.GY - 1) / pl.GY) : 0u;
      const int64_t units_per_seq = (int64_t)d.n_kv_heads * pl.GY;
      int64_t total = 0;
      for (int i = 0; i < nb; ++i) {
        sl.bstart[i] = (int32_t)total;
        total += units_per_seq * blocks_of(sl.kv_len[i], sl.n_nodes[i]);
        if (total > kMaxFlatBlocks) return FSPAD_ERR_SHAPE;  // the kernels index blocks with 32 bits
      }
      sl.bstart[nb] = (int32_t)total;
      sl.total_blocks = (int32_t)total;
      bool same = true;
      for (int i = 1; i < nb; ++i) same = same && sl.kv_len[i] == sl.kv_len[0] && sl.n_nodes[i] == sl.n_nodes[0];
      sl.seq_blocks = same ? (int32_t)(units_per_seq * blocks_of(sl.kv_len[0], sl.n_nodes[0])) : 0;
      sl.same_len = sl.kv_len[0];
      sl.same_nodes = sl.n_nodes[0];
      const int64_t units = (int64_t)nb * units_per_seq;
      sl.n_wgs = plan_wgs(pl, total, units, uniform, d.workgroups);
      sl.wg_quot = (int32_t)(total / sl.n_wgs);
      sl.wg_rem = (int32_t)(total % sl.n_wgs);
      const int64_t slots = units + sl.n_wgs;
      const size_t need = (size_t)slots * slot_bytes(d, pl);
      if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15)) return FSPAD_ERR_WORKSPACE;
      if (pl.shared_stage) {
        if (d.head_dim == 128) hipLaunchKernelGGL((tree_attn_gqa_kernel<128, 4, 2>), dim3((unsigned)sl.n_wgs), dim3(512), 0, stream, sl);
        // (head dim 64 leaves registers for three wavefronts per SIMD: three key groups; 43.1 -> 40.6 us on a
        // 64/8-head, 16384-key, 60-node call, 70.7 -> 64.5 us at 32768 keys)
        else hipLaunchKernelGGL((tree_attn_gqa_kernel<64, 4, 3>), dim3((unsigned)sl.n_wgs), dim3(768), 0, stream, sl);
      } else if (d.head_dim == 128) {
        launch_bf16<128>(pl, sl, stream);
      } else {
        launch_bf16<64>(pl, sl, stream);
      }
      if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
      // the merge pass runs only if some unit was cut across workgroups
      bool any_cut = false;
      for (int i = 0; i < nb && !any_cut; ++i) {
        const int64_t nblk = blocks_of(sl.kv_len[i], sl.n_nodes[i]);
        for (int64_t ub = 0; ub < units_per_seq && !any_cut; ++ub) {
          const int64_t fs = sl.bstart[i] + ub * nblk;
          any_cut = host_owner_of(fs, total, sl.n_wgs) != host_owner_of(fs + nblk - 1, total, sl.n_wgs);
        }
      }
      if (any_cut) {
        const int rows_per_slab = 16 * pl.QT;
        const int rpb = 256 / (d.head_dim / 4);
        dim3 cgrid((unsigned)((pl.rows_per_unit + rpb - 1) / rpb), (unsigned)units);
        if (d.head_dim == 128) hipLaunchKernelGGL(tree_attn_combine_kernel<128>, cgrid, dim3(256), 0, stream, sl, rows_per_slab);
        else hipLaunchKernelGGL(tree_attn_combine_kernel<64>, cgrid, dim3(256), 0, stream, sl, rows_per_slab);
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
