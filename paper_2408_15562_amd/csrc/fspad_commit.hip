// Commit of the accepted path to the KV cache (arXiv 2408.15562, Preliminaries: the
// tokens that survive validation extend the sequence the next draft-verify cycle starts
// from; the paper does not spell the cache update out). The keys and values of the
// accepted tree nodes, computed by the verification forward, are appended to each
// sequence's cache in path order, so the next cycle's prefix already holds them.
//
// Pure data movement: a few hundred KB per call. One workgroup per (path position,
// sequence, K or V); each thread moves 16 bytes at a time.
#include "fspad.h"

#include <hip/hip_runtime.h>

namespace {

constexpr int kMaxBatchPerLaunch = 128;

struct CommitParams {
  const char* tree[2];   // k_tree, v_tree of this slice
  char* cache[2];        // k_cache, v_cache of this slice
  const int32_t* path;   // [B,Nmax]
  const int32_t* path_len;
  int32_t* kv_len_out;   // may be null
  int64_t stride_batch, stride_head, stride_token;  // bytes
  int32_t Nmax, Hkv, row_bytes;                     // row_bytes = D * element size
  int32_t kv_len[kMaxBatchPerLaunch];
};

__global__ __launch_bounds__(256) void kv_commit_kernel(const CommitParams p) {
  const int j = blockIdx.x, b = blockIdx.y, which = blockIdx.z;
  int len = p.path_len[b];
  len = len < 0 ? 0 : (len > p.Nmax ? p.Nmax : len);
  if (j == 0 && which == 0 && threadIdx.x == 0 && p.kv_len_out) p.kv_len_out[b] = p.kv_len[b] + len;
  if (j >= len) return;
  const int node = p.path[(size_t)b * p.Nmax + j];
  if (node < 0 || node >= p.Nmax) return;  // a malformed path moves nothing rather than reading out of bounds
  const int chunks_per_head = p.row_bytes >> 4;
  const int chunks = p.Hkv * chunks_per_head;
  const char* src = p.tree[which] + ((size_t)b * p.Nmax + node) * p.Hkv * p.row_bytes;
  char* dst = p.cache[which] + (size_t)b * p.stride_batch + (size_t)(p.kv_len[b] + j) * p.stride_token;
  for (int c = threadIdx.x; c < chunks; c += 256) {
    const int g = c / chunks_per_head, o = c - g * chunks_per_head;
    const uint4 v = *reinterpret_cast<const uint4*>(src + (size_t)c * 16);
    *reinterpret_cast<uint4*>(dst + (size_t)g * p.stride_head + (size_t)o * 16) = v;
  }
}

}  // namespace

extern "C" fspad_status fspad_kv_commit(const fspad_attn_desc* desc, const void* k_tree, const void* v_tree,
                                        void* k_cache, void* v_cache, int32_t cache_capacity,
                                        const int32_t* kv_len, const int32_t* path, const int32_t* path_len,
                                        int32_t* kv_len_out, void* hip_stream) {
  if (!desc) return FSPAD_ERR_NULL;
  const fspad_attn_desc& d = *desc;
  if (d.batch < 1 || d.n_nodes_max < 1 || d.n_nodes_max > FSPAD_MAX_NODES) return FSPAD_ERR_SHAPE;
  if (d.n_kv_heads < 1 || (d.head_dim != 64 && d.head_dim != 128)) return FSPAD_ERR_SHAPE;
  if (d.io_dtype != FSPAD_F32 && d.io_dtype != FSPAD_BF16) return FSPAD_ERR_DTYPE;
  if (!k_tree || !v_tree || !k_cache || !v_cache || !kv_len || !path || !path_len) return FSPAD_ERR_NULL;
  const int esz = d.io_dtype == FSPAD_BF16 ? 2 : 4;
  const int64_t align = 16 / esz;
  if (d.cache_stride_token < d.head_dim || d.cache_stride_token % align || d.cache_stride_head % align ||
      d.cache_stride_batch % align || d.cache_stride_head < 0 || d.cache_stride_batch < 0)
    return FSPAD_ERR_SHAPE;
  if (((uintptr_t)k_tree | (uintptr_t)v_tree | (uintptr_t)k_cache | (uintptr_t)v_cache) & 15) return FSPAD_ERR_SHAPE;
  // the path is only known on the device: room for the longest possible one is required
  for (int b = 0; b < d.batch; ++b)
    if (kv_len[b] < 0 || (int64_t)kv_len[b] + d.n_nodes_max > cache_capacity) return FSPAD_ERR_SHAPE;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);

  CommitParams prm{};
  prm.stride_batch = d.cache_stride_batch * esz;
  prm.stride_head = d.cache_stride_head * esz;
  prm.stride_token = d.cache_stride_token * esz;
  prm.Nmax = d.n_nodes_max; prm.Hkv = d.n_kv_heads; prm.row_bytes = d.head_dim * esz;
  for (int b0 = 0; b0 < d.batch; b0 += kMaxBatchPerLaunch) {
    const int nb = d.batch - b0 < kMaxBatchPerLaunch ? d.batch - b0 : kMaxBatchPerLaunch;
    CommitParams sl = prm;
    const size_t tree_off = (size_t)b0 * d.n_nodes_max * d.n_kv_heads * d.head_dim * esz;
    sl.tree[0] = static_cast<const char*>(k_tree) + tree_off;
    sl.tree[1] = static_cast<const char*>(v_tree) + tree_off;
    sl.cache[0] = static_cast<char*>(k_cache) + (size_t)b0 * prm.stride_batch;
    sl.cache[1] = static_cast<char*>(v_cache) + (size_t)b0 * prm.stride_batch;
    sl.path = path + (size_t)b0 * d.n_nodes_max;
    sl.path_len = path_len + b0;
    sl.kv_len_out = kv_len_out ? kv_len_out + b0 : nullptr;
    for (int i = 0; i < nb; ++i) sl.kv_len[i] = kv_len[b0 + i];
    hipLaunchKernelGGL(kv_commit_kernel, dim3((unsigned)d.n_nodes_max, (unsigned)nb, 2), dim3(256), 0, stream, sl);
    if (hipGetLastError() != hipSuccess) return FSPAD_ERR_HIP;
  }
  return FSPAD_OK;
}
