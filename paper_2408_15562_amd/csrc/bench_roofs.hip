// Measurement kernels of the benchmark, not part of the verification library: they are built into a
// library of their own (libfspad_roofs.so) so that libfspad.so exports the verification calls only.
//
//   roofs_hbm_read   a plain streaming read, 16 bytes per lane, eight loads in flight per lane: what
//                    this machine's HBM delivers to the simplest possible access pattern
//   roofs_hbm_copy   the same as a copy (reads and writes `bytes` each): a kernel of known traffic next to
//                    which the byte counters of the profiler are scaled
//   roofs_mfma_bf16  a register-resident loop of v_mfma_f32_16x16x32_bf16 (or 32x32x16), eight independent
//                    accumulator chains per wavefront, no memory access: what the matrix cores sustain
//   roofs_overlap    what runs at the same time on one SIMD: a matrix instruction followed by vector
//                    instructions in the same wavefront, or one wavefront of matrix instructions next to
//                    one of vector instructions (the facts the attention kernels' wavefront shapes rest on)
// Each returns 0 or a HIP error code; work is enqueued on the caller's stream, nothing is allocated.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kThreads = 256;
constexpr int kUnroll = 8;

__global__ __launch_bounds__(kThreads) void roofs_read_kernel(const u32x4* __restrict__ src, size_t n_vec, unsigned* sink) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (; i + (kUnroll - 1) * stride < n_vec; i += kUnroll * stride) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) v[k] = __builtin_nontemporal_load(src + i + k * stride);
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) acc ^= v[k];
  }
  for (; i < n_vec; i += stride) acc ^= __builtin_nontemporal_load(src + i);
  // data-dependent and practically never true: keeps the loads alive without a store per thread
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x5bd1e995u && acc[0] == 0x1b873593u) *sink = acc[1];
}

__global__ __launch_bounds__(kThreads) void roofs_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n_vec) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  for (; i + (kUnroll - 1) * stride < n_vec; i += kUnroll * stride) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) v[k] = src[i + k * stride];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) dst[i + k * stride] = v[k];
  }
  for (; i < n_vec; i += stride) dst[i] = src[i];
}

// eight independent chains per wavefront: the matrix unit never waits for a result
template <int SHAPE>
__global__ __launch_bounds__(kThreads) void roofs_mfma_kernel(int iters, float* sink) {
  bf16x8 a, b;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    a[j] = (__bf16)(float)((threadIdx.x + j) & 3);
    b[j] = (__bf16)(float)((threadIdx.x * 3 + j) & 1);
  }
  float total = 0.f;
  // (the instruction is written out with the accumulator as source and destination: left to the
  // register allocator, a loop of builtins gets copies between accumulator registers in every turn)
#define ROOFS_MFMA16(c) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b))
#define ROOFS_MFMA32(c) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b))
  if constexpr (SHAPE == 16) {
    f32x4 c0 = {0.f, 0.f, 0.f, 0.f}, c1 = c0, c2 = c0, c3 = c0, c4 = c0, c5 = c0, c6 = c0, c7 = c0;
    for (int it = 0; it < iters; ++it) {
      ROOFS_MFMA16(c0); ROOFS_MFMA16(c1); ROOFS_MFMA16(c2); ROOFS_MFMA16(c3);
      ROOFS_MFMA16(c4); ROOFS_MFMA16(c5); ROOFS_MFMA16(c6); ROOFS_MFMA16(c7);
    }
    const f32x4 s = ((c0 + c1) + (c2 + c3)) + ((c4 + c5) + (c6 + c7));
    total = s[0] + s[1] + s[2] + s[3];
  } else {
    f32x16 c0, c1, c2, c3;
#pragma unroll
    for (int e = 0; e < 16; ++e) { c0[e] = 0.f; c1[e] = 0.f; c2[e] = 0.f; c3[e] = 0.f; }
    for (int it = 0; it < iters; ++it) {
      ROOFS_MFMA32(c0); ROOFS_MFMA32(c1); ROOFS_MFMA32(c2); ROOFS_MFMA32(c3);
    }
    const f32x16 s = (c0 + c1) + (c2 + c3);
#pragma unroll
    for (int e = 0; e < 16; ++e) total += s[e];
  }
#undef ROOFS_MFMA16
#undef ROOFS_MFMA32
  if (total == -1.0f) *sink = total;   // sums of non-negative products: never true
}

// mode 0: every wavefront alternates one 32x32x16 matrix instruction with `nv` vector instructions
//         (one wavefront per SIMD: workgroups of 256 threads, one workgroup per compute unit)
// mode 1: workgroups of 512 threads, two wavefronts per SIMD: wavefronts 0-3 issue two matrix
//         instructions per turn, wavefronts 4-7 `nv` vector instructions per turn (sixteen for nv = 0)
// mode 2 / 3: mode 1 with only the matrix / only the vector wavefronts doing work
// trans: the vector instruction is v_exp_f32 instead of v_fma_f32
template <int NV, bool TRANS>
__device__ __forceinline__ void vector_ops(float (&x)[8]) {
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    if constexpr (TRANS) asm volatile("v_exp_f32 %0, %0" : "+v"(x[i % 8]));
    else asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(x[i % 8]) : "v"(x[(i + 3) % 8]));
  }
}

template <int NV, bool TRANS>
__global__ __launch_bounds__(512) void roofs_overlap_kernel(int mode, int iters, float* sink) {
  bf16x8 a, b;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    a[j] = (__bf16)(float)((threadIdx.x + j) & 3);
    b[j] = (__bf16)(float)((threadIdx.x * 3 + j) & 1);
  }
  f32x16 c0, c1;
#pragma unroll
  for (int e = 0; e < 16; ++e) { c0[e] = 0.f; c1[e] = 0.f; }
  float x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = 0.001f * (float)(threadIdx.x + i);
  const int role = threadIdx.x >> 8;
  if (mode == 0) {
    for (int it = 0; it < iters; ++it) {
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c0) : "v"(a), "v"(b));
      vector_ops<NV, TRANS>(x);
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c1) : "v"(a), "v"(b));
      vector_ops<NV, TRANS>(x);
    }
  } else if (role == 0 && mode != 3) {
    for (int it = 0; it < iters; ++it) {
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c0) : "v"(a), "v"(b));
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c1) : "v"(a), "v"(b));
    }
  } else if (role == 1 && mode != 2) {
    for (int it = 0; it < iters; ++it) vector_ops<(NV == 0 ? 16 : NV), TRANS>(x);
  }
  float total = 0.f;
#pragma unroll
  for (int e = 0; e < 16; ++e) total += c0[e] + c1[e];
#pragma unroll
  for (int i = 0; i < 8; ++i) total += x[i];
  if (total == -1.2345f) *sink = total;
}

}  // namespace

// One launch on 256 workgroups (one per compute unit). mode 0: nv in {0, 4, 8, 16} vector instructions
// after each matrix instruction; modes 1-3: see the kernel. The caller times it.
extern "C" int roofs_overlap(int mode, int nv, int trans, int iters, void* sink, void* hip_stream) {
  if (!sink || iters < 1 || mode < 0 || mode > 3) return -1;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const dim3 grid(256), block(mode == 0 ? 256 : 512);
  float* out = static_cast<float*>(sink);
#define ROOFS_OVERLAP(NV)                                                                                              \
  do {                                                                                                                 \
    if (trans) hipLaunchKernelGGL((roofs_overlap_kernel<NV, true>), grid, block, 0, stream, mode, iters, out);         \
    else hipLaunchKernelGGL((roofs_overlap_kernel<NV, false>), grid, block, 0, stream, mode, iters, out);              \
  } while (0)
  switch (nv) {
    case 0: ROOFS_OVERLAP(0); break;
    case 4: ROOFS_OVERLAP(4); break;
    case 8: ROOFS_OVERLAP(8); break;
    case 16: ROOFS_OVERLAP(16); break;
    default: return -1;
  }
#undef ROOFS_OVERLAP
  return (int)hipGetLastError();
}

extern "C" int roofs_hbm_read(const void* src, size_t bytes, void* sink, int workgroups, void* hip_stream) {
  if (!src || !sink || bytes < 16 || ((uintptr_t)src & 15) || workgroups < 1) return -1;
  hipLaunchKernelGGL(roofs_read_kernel, dim3((unsigned)workgroups), dim3(kThreads), 0, reinterpret_cast<hipStream_t>(hip_stream),
                     static_cast<const u32x4*>(src), bytes / 16, static_cast<unsigned*>(sink));
  return (int)hipGetLastError();
}

extern "C" int roofs_hbm_copy(const void* src, void* dst, size_t bytes, int workgroups, void* hip_stream) {
  if (!src || !dst || bytes < 16 || (((uintptr_t)src | (uintptr_t)dst) & 15) || workgroups < 1) return -1;
  hipLaunchKernelGGL(roofs_copy_kernel, dim3((unsigned)workgroups), dim3(kThreads), 0, reinterpret_cast<hipStream_t>(hip_stream),
                     static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), bytes / 16);
  return (int)hipGetLastError();
}

// flops of one launch = workgroups * 4 wavefronts * iters * (SHAPE 16: 8 x 16*16*32*2, SHAPE 32: 4 x 32*32*16*2)
extern "C" int roofs_mfma_bf16(int shape, int iters, int workgroups, void* sink, void* hip_stream) {
  if (!sink || iters < 1 || workgroups < 1 || (shape != 16 && shape != 32)) return -1;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  if (shape == 16) hipLaunchKernelGGL(roofs_mfma_kernel<16>, dim3((unsigned)workgroups), dim3(kThreads), 0, stream, iters, static_cast<float*>(sink));
  else hipLaunchKernelGGL(roofs_mfma_kernel<32>, dim3((unsigned)workgroups), dim3(kThreads), 0, stream, iters, static_cast<float*>(sink));
  return (int)hipGetLastError();
}
