// Descent of the greedy walk (arXiv 2408.15562, Preliminaries, validation phase: the tree is
// compared strictly with the target's own tokens; a node whose token differs is dropped with all
// its descendants). Shared by the kernels that end in it; internal to the library.
#ifndef FSPAD_GREEDY_WALK_H
#define FSPAD_GREEDY_WALK_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fspad_detail {

// Called by all 64 lanes of one wavefront. target[i] (LDS) is the target's greedy token after
// node i; lane i brings parent and draft token of node i of sequence b (my_par = -2 for lanes
// past the tree; the caller fetches them early, they do not depend on the logits). Row offset
// o = b * Nmax. Writes path/tokens (unused slots -1) and the two lengths.
__device__ __forceinline__ void greedy_descend(const int* target, int n, int Nmax, int lane, int64_t o, int b,
                                               int my_par, int my_tok, int32_t* path, int32_t* tokens,
                                               int32_t* path_len, int32_t* n_tokens) {
  int my_path = -1, my_out = -1;  // lane j keeps path[j] and tokens[j]
  if (lane == 0) my_path = 0;
  int cur = 0, len = 1;
  for (int iter = 0; iter < Nmax && len < Nmax; ++iter) {  // bounded: a well-formed walk ends at a leaf
    const int a = target[cur];
    const bool hit = lane > 0 && lane < n && my_par == cur && my_tok == a;
    const unsigned long long bal = __ballot(hit);
    if (bal == 0ull) break;
    const int nxt = __ffsll(bal) - 1;  // lowest child index first
    if (lane == len) my_path = nxt;
    if (lane == len - 1) my_out = a;
    cur = nxt;
    ++len;
  }
  if (lane == len - 1) my_out = target[cur];  // bonus: the target's own token after the last accepted node
  if (lane < Nmax) { path[o + lane] = my_path; tokens[o + lane] = my_out; }
  if (lane == 0) { path_len[b] = len; n_tokens[b] = len; }
}

}  // namespace fspad_detail
#endif
