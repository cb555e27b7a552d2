// Exercises the CPU oracle (oracle/fspad_oracle.c) and the library's host helpers
// (csrc/fspad_host.cpp) on seeded small cases in one process built with
// -fsanitize=address,undefined: any out-of-bounds access, use of freed memory or undefined
// arithmetic aborts with a report. Built and run by tests/test_sanitizers.py; exit status 0 = clean.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "fspad.h"

extern "C" {
int fspad_oracle_dense_mask(int32_t N, const int32_t* parent, uint8_t* M);
int fspad_oracle_tree_attn(int32_t B, int32_t Nmax, int32_t Hq, int32_t Hkv, int32_t D, double scale, const double* q,
                           const double* k_tree, const double* v_tree, const double* k_cache, const double* v_cache,
                           int64_t Lcap, const int32_t* kv_len, const int32_t* n_nodes, const int32_t* parent,
                           const uint64_t* packed_mask, double* out, int32_t nthreads);
int fspad_oracle_accept_greedy(int32_t B, int32_t Nmax, int32_t V, const float* logits, int64_t row_stride,
                               const int32_t* draft_tokens, const int32_t* parent, const int32_t* n_nodes, int32_t* path,
                               int32_t* path_len, int32_t* tokens, int32_t* n_tokens);
int fspad_oracle_accept_sample(int32_t B, int32_t Nmax, int32_t V, const float* logits, int64_t row_stride,
                               const int32_t* draft_tokens, const int32_t* parent, const int32_t* n_nodes,
                               float temperature, const float* uniforms, int32_t* path, int32_t* path_len, int32_t* tokens,
                               int32_t* n_tokens, double* min_margin);
}

namespace {
uint64_t g_state = 0x9e3779b97f4a7c15ull;
uint32_t next_u32() {  // xorshift64*
  g_state ^= g_state >> 12; g_state ^= g_state << 25; g_state ^= g_state >> 27;
  return (uint32_t)((g_state * 0x2545f4914f6cdd1dull) >> 32);
}
double uniform() { return (next_u32() + 0.5) / 4294967296.0; }
double normal() { return std::sqrt(-2.0 * std::log(uniform())) * std::cos(6.283185307179586 * uniform()); }
int fails = 0;
void expect(bool ok, const char* what) { if (!ok) { std::fprintf(stderr, "sanitize_driver: %s\n", what); ++fails; } }
}  // namespace

int main() {
  for (int trial = 0; trial < 40; ++trial) {
    const int B = 1 + next_u32() % 3, N = 1 + next_u32() % 64, Hkv = 1 + next_u32() % 3, G = 1 + next_u32() % 3;
    const int Hq = Hkv * G, D = 4 << (next_u32() % 3), Lcap = next_u32() % 70, V = 1 + next_u32() % 300;
    std::vector<int32_t> parent((size_t)B * N, -1), n_nodes(B), kv_len(B), tokens((size_t)B * N);
    for (int b = 0; b < B; ++b) {
      n_nodes[b] = 1 + next_u32() % N;
      kv_len[b] = Lcap ? next_u32() % (Lcap + 1) : 0;
      for (int i = 1; i < N; ++i) parent[(size_t)b * N + i] = next_u32() % i;
      for (int i = 0; i < N; ++i) tokens[(size_t)b * N + i] = next_u32() % V;
    }
    // host helpers: mask, validation (valid trees; duplicate sibling tokens may legitimately be reported)
    std::vector<uint64_t> mask((size_t)B * N);
    expect(fspad_tree_build_mask(B, N, parent.data(), n_nodes.data(), mask.data()) == FSPAD_OK, "build_mask status");
    const fspad_status vs = fspad_tree_validate(B, N, V, parent.data(), tokens.data(), n_nodes.data());
    expect(vs == FSPAD_OK || vs == FSPAD_ERR_TREE, "validate status");
    expect(fspad_tree_validate(B, N, V, parent.data(), nullptr, n_nodes.data()) == FSPAD_OK, "validate without tokens");
    std::vector<uint8_t> dense((size_t)N * N);
    for (int b = 0; b < B; ++b) {
      expect(fspad_oracle_dense_mask(n_nodes[b], parent.data() + (size_t)b * N, dense.data()) == 0, "dense_mask status");
      for (int i = 0; i < n_nodes[b]; ++i)
        for (int t = 0; t < n_nodes[b]; ++t)
          expect(dense[(size_t)i * n_nodes[b] + t] == ((mask[(size_t)b * N + i] >> t) & 1u), "dense mask == packed mask");
    }
    // an ill-formed tree must be refused, not followed
    if (N > 2) {
      std::vector<int32_t> bad(parent);
      bad[1] = 1;
      std::vector<int32_t> nn(B, N);
      expect(fspad_tree_build_mask(B, N, bad.data(), nn.data(), mask.data()) == FSPAD_ERR_TREE, "bad tree refused (host)");
      expect(fspad_oracle_dense_mask(N, bad.data(), dense.data()) == -1, "bad tree refused (oracle)");
      fspad_tree_build_mask(B, N, parent.data(), n_nodes.data(), mask.data());
    }
    // attention oracle
    auto fill = [](std::vector<double>& v) { for (double& x : v) x = normal(); };
    std::vector<double> q((size_t)B * N * Hq * D), kt((size_t)B * N * Hkv * D), vt(kt.size()),
        kc((size_t)B * Hkv * (Lcap ? Lcap : 1) * D), vc(kc.size()), out(q.size());
    fill(q); fill(kt); fill(vt); fill(kc); fill(vc);
    expect(fspad_oracle_tree_attn(B, N, Hq, Hkv, D, 0.3, q.data(), kt.data(), vt.data(), Lcap ? kc.data() : nullptr,
                                  Lcap ? vc.data() : nullptr, Lcap, kv_len.data(), n_nodes.data(), parent.data(), mask.data(),
                                  out.data(), 1 + trial % 3) == 0, "tree_attn status");
    for (double x : out) expect(std::isfinite(x), "tree_attn output finite");
    // acceptance oracles, rows padded by a stride
    const int64_t stride = V + next_u32() % 5;
    std::vector<float> logits((size_t)B * N * stride), uni((size_t)B * 2 * N);
    for (float& x : logits) x = (float)(3.0 * normal());
    for (float& x : uni) x = (float)(next_u32() >> 8) / 16777216.0f;
    std::vector<int32_t> path((size_t)B * N), toks((size_t)B * N), plen(B), ntok(B);
    std::vector<double> margin(B);
    expect(fspad_oracle_accept_greedy(B, N, V, logits.data(), stride, tokens.data(), parent.data(), n_nodes.data(),
                                      path.data(), plen.data(), toks.data(), ntok.data()) == 0, "accept_greedy status");
    for (int b = 0; b < B; ++b) expect(plen[b] >= 1 && plen[b] <= n_nodes[b] && ntok[b] == plen[b], "greedy lengths");
    expect(fspad_oracle_accept_sample(B, N, V, logits.data(), stride, tokens.data(), parent.data(), n_nodes.data(),
                                      0.5f + (float)uniform(), uni.data(), path.data(), plen.data(), toks.data(),
                                      ntok.data(), margin.data()) == 0, "accept_sample status");
    for (int b = 0; b < B; ++b) {
      expect(plen[b] >= 1 && plen[b] <= n_nodes[b] && ntok[b] == plen[b], "sample lengths");
      expect(toks[(size_t)b * N + plen[b] - 1] >= 0 && toks[(size_t)b * N + plen[b] - 1] < V, "sampled token in range");
    }
    expect(fspad_oracle_accept_sample(B, N, V, logits.data(), stride, tokens.data(), parent.data(), n_nodes.data(), 0.0f,
                                      uni.data(), path.data(), plen.data(), toks.data(), ntok.data(), nullptr) == -6,
           "temperature refused");
  }
  for (int s = 0; s < 9; ++s) expect(fspad_status_string((fspad_status)s) != nullptr, "status string");
  std::printf("sanitize_driver: %s\n", fails ? "FAILED" : "clean");
  return fails ? 1 : 0;
}
