// Host-side helpers of the tree-verification library: status strings, ancestor
// bitmask construction and tree validation (arXiv 2408.15562, Preliminaries: the
// draft tokens are organised into a tree by their dependencies and the target's
// attention mask is derived from that tree before verification).
#include "fspad.h"

#include <vector>
#include <algorithm>

extern "C" const char* fspad_status_string(fspad_status status) {
  switch (status) {
    case FSPAD_OK: return "ok";
    case FSPAD_ERR_NULL: return "a required pointer is NULL";
    case FSPAD_ERR_SHAPE: return "unsupported or inconsistent shape, length or stride";
    case FSPAD_ERR_TREE: return "ill-formed tree (parent order, token range or duplicate sibling tokens)";
    case FSPAD_ERR_DTYPE: return "unsupported dtype combination";
    case FSPAD_ERR_WORKSPACE: return "workspace missing or too small";
    case FSPAD_ERR_TEMPERATURE: return "temperature must be finite and > 0";
    case FSPAD_ERR_HIP: return "HIP launch failed";
  }
  return "unknown status";
}

namespace {
// parent[0] == -1 and every later parent precedes its child
bool parents_ordered(const int32_t* parent, int32_t n) {
  if (parent[0] != -1) return false;
  for (int32_t i = 1; i < n; ++i)
    if (parent[i] < 0 || parent[i] >= i) return false;
  return true;
}
}  // namespace

extern "C" fspad_status fspad_tree_build_mask(int32_t B, int32_t Nmax, const int32_t* parent_host,
                                              const int32_t* n_nodes_host, uint64_t* mask_host) {
  if (!parent_host || !n_nodes_host || !mask_host) return FSPAD_ERR_NULL;
  if (B < 1 || Nmax < 1 || Nmax > FSPAD_MAX_NODES) return FSPAD_ERR_SHAPE;
  for (int32_t b = 0; b < B; ++b) {
    const int32_t n = n_nodes_host[b];
    if (n < 1 || n > Nmax) return FSPAD_ERR_SHAPE;
    const int32_t* parent = parent_host + (size_t)b * Nmax;
    uint64_t* mask = mask_host + (size_t)b * Nmax;
    if (!parents_ordered(parent, n)) return FSPAD_ERR_TREE;
    // topological order: a parent's word is complete before any child reads it
    mask[0] = 1;
    for (int32_t i = 1; i < n; ++i) mask[i] = mask[parent[i]] | ((uint64_t)1 << i);
    for (int32_t i = n; i < Nmax; ++i) mask[i] = 0;
  }
  return FSPAD_OK;
}

extern "C" fspad_status fspad_tree_validate(int32_t B, int32_t Nmax, int32_t V, const int32_t* parent_host,
                                            const int32_t* tokens_host, const int32_t* n_nodes_host) {
  if (!parent_host || !n_nodes_host) return FSPAD_ERR_NULL;
  if (B < 1 || Nmax < 1 || Nmax > FSPAD_MAX_NODES || V < 1) return FSPAD_ERR_SHAPE;
  std::vector<std::pair<int32_t, int32_t>> keyed;  // (parent, token) of every non-root node
  for (int32_t b = 0; b < B; ++b) {
    const int32_t n = n_nodes_host[b];
    if (n < 1 || n > Nmax) return FSPAD_ERR_SHAPE;
    const int32_t* parent = parent_host + (size_t)b * Nmax;
    if (!parents_ordered(parent, n)) return FSPAD_ERR_TREE;
    if (!tokens_host) continue;
    const int32_t* tok = tokens_host + (size_t)b * Nmax;
    keyed.clear();
    for (int32_t i = 0; i < n; ++i) {
      if (tok[i] < 0 || tok[i] >= V) return FSPAD_ERR_TREE;
      if (i > 0) keyed.emplace_back(parent[i], tok[i]);
    }
    std::sort(keyed.begin(), keyed.end());
    if (std::adjacent_find(keyed.begin(), keyed.end()) != keyed.end()) return FSPAD_ERR_TREE;
  }
  return FSPAD_OK;
}
