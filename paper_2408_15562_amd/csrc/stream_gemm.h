// Streaming core of the skinny bf16 GEMMs of this library (few rows of X, many rows of W, both
// row-major along k): internal to the library. gfx950 (CDNA4) only.
//
// With `v_mfma_f32_16x16x32_bf16`, A = 16 rows of W and B = 16 rows of X, both operands are "8
// consecutive k per lane", i.e. plain 16-byte loads of row-major data: W goes from HBM straight
// into registers, through a ring of k-steps per wavefront that is refilled as soon as a product is
// issued; X (small, L2-resident) is staged through LDS, XOR-swizzled by 16-byte chunk so that a
// 16-row operand read touches 16 different bank groups, double-buffered, with a barrier that orders
// LDS traffic only (the W requests in flight stay in flight).
#ifndef FSPAD_STREAM_GEMM_H
#define FSPAD_STREAM_GEMM_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fspad_detail {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// acc[t][nv] += sum over a k range of
//   X[row0 + 16t + n][k] * W[v0 + 16nv + 4g + i][k]      (lane (n, g), accumulator element i)
// for one wavefront of a workgroup of WAVES wavefronts that share X through LDS.
// MT: 16-row tiles of X per workgroup. SPS: k-steps (of 32) per LDS stage of X (stage = 16*MT rows
// x 32*SPS k). kRing: weight operands per 16-row weight tile that a wavefront keeps requested. VT:
// weight tiles per wavefront. x_base / w_base point at the first k of the range, rows are row_bytes
// apart; the range is n_steps k-steps (a multiple of 8) and is walked from first_step on, wrapping
// around (first_step a multiple of SPS; 0 unless n_steps is a multiple of SPS). xs: 2 stages of LDS.
// PACKED: W is stored tile by tile instead of row by row -- the 16 rows x 32 k of one operand are
// 1 KB in lane order (lane (n, g) at byte 16 * (n + 16 g)), the k-steps of a 16-row tile follow one
// another, then the next 16 rows. A wavefront's request is then one contiguous KB instead of sixteen
// 64-byte pieces a row pitch apart; row_bytes is still 2 K, v0 a multiple of 16, and w_base points at
// the first k-step of the range within tile row 0.
template <int MT, int SPS, int kRing, int WAVES, int VT, bool PACKED = false>
struct StreamGemm {
  static constexpr int kStageK = 32 * SPS;
  static constexpr int kRowBytes = kStageK * 2;                        // 256, 512 or 1024
  static constexpr int kStageBytes = MT * 16 * kRowBytes;
  static constexpr int kChunksPerRow = kRowBytes / 16;                 // 16, 32 or 64
  static constexpr int kRowsPerCopy = 1024 / kRowBytes;                // one copy instruction moves 1 KB
  static constexpr int kCopiesPerWave = kStageBytes / 1024 / WAVES;
  static_assert(kCopiesPerWave >= 1 && kRing % SPS == 0 && kRing % 4 == 0, "stage shape");

  __device__ static __forceinline__ void run(char* xs, const char* x_base, const char* w_base, size_t row_bytes,
                                             int n_xrows, int n_wrows, int row0, int v0, int n_steps, int first_step,
                                             f32x4 (&acc)[MT][VT]) {
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, g = lane >> 4;
    // weight rows of this lane (rows past the vocabulary are clamped; their columns are never taken)
    const char* wrow[VT];
#pragma unroll
    for (int nv = 0; nv < VT; ++nv)
      wrow[nv] = PACKED ? w_base + (size_t)min(v0 + 16 * nv, n_wrows - 16) * row_bytes + lane * 16
                        : w_base + (size_t)min(v0 + 16 * nv + n, n_wrows - 1) * row_bytes + g * 16;

    // hidden-state copies of this wavefront: LDS slot s of row r receives the row's 16-byte chunk
    // s ^ (r & 15) of the stage's k range (chunks past the end of the row are clamped: never used)
    const char* xsrc[kCopiesPerWave];
    int xcol[kCopiesPerWave];
#pragma unroll
    for (int i = 0; i < kCopiesPerWave; ++i) {
      const int r = kRowsPerCopy * (wave * kCopiesPerWave + i) + lane / kChunksPerRow, s = lane % kChunksPerRow;
      xsrc[i] = x_base + (size_t)min(row0 + r, n_xrows - 1) * row_bytes;
      xcol[i] = s ^ (r & 15);
    }
    const int last_chunk = 4 * n_steps - 1;
    // operand reads: lane (n, g) of tile t, k-step kk of the stage reads chunk 4*kk + g of row 16*t + n,
    // kept at slot (4*kk + g) ^ n = (4*kk) ^ (g ^ n)
    const unsigned xread = (unsigned)n * kRowBytes, xswz = (unsigned)(g ^ n) << 4;

    bf16x8 xr[kCopiesPerWave];
    auto fetch_x = [&](int stage_index) {
#pragma unroll
      for (int i = 0; i < kCopiesPerWave; ++i) {
        int stage = stage_index + first_step / SPS;
        stage -= stage * SPS >= n_steps ? n_steps / SPS : 0;
        const int chunk = min(stage * kChunksPerRow + xcol[i], last_chunk);
        xr[i] = *reinterpret_cast<const bf16x8*>(xsrc[i] + ((size_t)chunk << 4));
      }
    };
    auto store_x = [&](int stage_index) {
      char* dst = xs + (stage_index & 1) * kStageBytes + wave * kCopiesPerWave * 1024 + lane * 16;
#pragma unroll
      for (int i = 0; i < kCopiesPerWave; ++i) *reinterpret_cast<bf16x8*>(dst + i * 1024) = xr[i];
    };
    // workgroup barrier that orders LDS traffic only: the weight requests in flight stay in flight
    auto lds_barrier = [] {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };
    // k-step ks of the weights: lane (n, g) holds k = 32*ks + 8*g .. +7 of its row (steps past the end
    // re-read the last one, so that every turn of the loop issues the same number of requests)
    auto load_w = [&](int nv, int ks) {
      int step = min(ks, n_steps - 1) + first_step;
      step -= step >= n_steps ? n_steps : 0;
      return *reinterpret_cast<const bf16x8*>(wrow[nv] + (size_t)step * (PACKED ? 1024 : 64));
    };

    // The weights are requested kRing k-steps ahead, every operand register being requested again as
    // soon as its products are issued. The hidden states of stage j+1 are requested into registers at
    // the top of stage j and written to the other LDS stage at its end (by then they have long
    // arrived, and the weight requests issued after them stay in flight); the barrier at the top of a
    // stage publishes every wavefront's share of it and retires the other one.
    bf16x8 w[VT][kRing];
    fetch_x(0);
#pragma unroll
    for (int i = 0; i < kRing; ++i)
#pragma unroll
      for (int nv = 0; nv < VT; ++nv) w[nv][i] = load_w(nv, i);
    store_x(0);
    const int n_stages = (n_steps + SPS - 1) / SPS;
    for (int ks0 = 0; ks0 < n_steps; ks0 += kRing) {
#pragma unroll
      for (int kk = 0; kk < kRing; ++kk) {
        const int ks = ks0 + kk;
        if (kk % 4 == 0 && ks >= n_steps) break;   // K is a multiple of 256 and the ring of 4: the end falls on a multiple of 4 steps
        if (kk % SPS == 0) {
          lds_barrier();
          if (ks / SPS + 1 < n_stages) fetch_x(ks / SPS + 1);
        }
        const char* base = xs + ((ks / SPS) & 1) * kStageBytes + xread + ((((unsigned)kk % SPS) << 6) ^ xswz);
        bf16x8 xf[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t) xf[t] = *reinterpret_cast<const bf16x8*>(base + t * (16 * kRowBytes));
#pragma unroll
        for (int nv = 0; nv < VT; ++nv)
#pragma unroll
          for (int t = 0; t < MT; ++t)
            acc[t][nv] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[nv][kk], xf[t], acc[t][nv], 0, 0, 0);
#pragma unroll
        for (int nv = 0; nv < VT; ++nv) w[nv][kk] = load_w(nv, ks + kRing);
        if (kk % SPS == SPS - 1 && ks / SPS + 1 < n_stages) store_x(ks / SPS + 1);
      }
    }

  }
};

}  // namespace fspad_detail
#endif
