/*
 * fspad_oracle.c - TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, obviously-correct CPU statement of what one tree-verification
 * step of draft-then-verify speculative decoding computes (arXiv 2408.15562,
 * section "Preliminaries"). Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the GPU library shares no code with it.
 *
 * Everything floating point is fp64. The loops follow the definitions term by
 * term: a dense boolean mask, one score array per query row, a scalar walk down
 * the tree. The only parallelism is an optional OpenMP split over independent
 * (sequence, head) pairs; the arithmetic of a pair is untouched by it.
 *
 * Pins (tests/test_oracle_*.py): single node == textbook decode attention,
 * chain == causal attention (library routine), path linearisation, Q=0 closed
 * form, hand-computed 3-node case, greedy == sequential argmax decoding of a toy
 * model, exact enumeration of the sampling rule on a 4-token vocabulary.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_MAX_NODES 64

/* ------------------------------------------------------------------ tree + mask
 * Preliminaries, draft phase: the draft tokens form a tree by their
 * dependencies and the target's attention mask follows from that tree, so that
 * each token is verified given exactly the tokens it depends on. Reading: node
 * t is visible from node i iff t == i or t is an ancestor of i.
 *
 * M is [N][N] row-major, M[i][t] = 1 iff t is in {i} U ancestors(i).
 * Returns 0, or -1 for an ill-formed parent array. */
int fspad_oracle_dense_mask(int32_t N, const int32_t* parent, uint8_t* M) {
  if (N < 1 || N > ORACLE_MAX_NODES || parent[0] != -1) return -1;
  memset(M, 0, (size_t)N * (size_t)N);
  for (int32_t i = 0; i < N; ++i) {
    if (i > 0 && (parent[i] < 0 || parent[i] >= i)) return -1;
    /* climb from i to the root, marking every node met on the way */
    for (int32_t a = i; a >= 0; a = parent[a]) M[(size_t)i * N + a] = 1;
  }
  return 0;
}

/* ------------------------------------------------------------------ attention
 * Preliminaries, validation phase: the target runs once over the flattened
 * tree, the mask introducing the dependencies, and returns for every node what
 * ordinary decoding along that node's root path would have returned.
 *
 * Plain definition, per sequence b, query head h (kv head g = h / (Hq/Hkv)),
 * node i < n_nodes[b]:
 *     keys   j = 0 .. L-1      : prefix cache rows, all visible
 *     keys   j = L .. L+n-1    : tree tokens t = j-L, visible iff M[i][t]
 *     s_j    = scale * sum_d q[i,h,d] * K_j[g,d]        (masked: -inf)
 *     p_j    = exp(s_j - max_j s_j) / sum_j exp(s_j - max_j s_j)
 *     out[i,h,:] = sum_j p_j * V_j[g,:]
 * Rows i >= n_nodes[b] of out are set to 0.
 *
 * Layouts (dense, fp64): q,out [B,Nmax,Hq,D]; k_tree,v_tree [B,Nmax,Hkv,D];
 * k_cache,v_cache [B,Hkv,Lcap,D]; parent [B,Nmax]; packed_mask [B,Nmax] or NULL.
 * If packed_mask is given it must equal the dense mask built from parent
 * (bit t of word i <=> M[i][t]); a mismatch returns -2.
 * Returns 0 on success, -1 ill-formed tree / shape, -2 mask mismatch, -3 no memory. */
int fspad_oracle_tree_attn(int32_t B, int32_t Nmax, int32_t Hq, int32_t Hkv, int32_t D,
                           double scale,
                           const double* q, const double* k_tree, const double* v_tree,
                           const double* k_cache, const double* v_cache, int64_t Lcap,
                           const int32_t* kv_len, const int32_t* n_nodes,
                           const int32_t* parent, const uint64_t* packed_mask,
                           double* out, int32_t nthreads) {
  if (B < 1 || Nmax < 1 || Nmax > ORACLE_MAX_NODES || Hkv < 1 || Hq % Hkv != 0 || D < 1) return -1;
  const int32_t G = Hq / Hkv;
  int status = 0;
  uint8_t* masks = (uint8_t*)malloc((size_t)B * Nmax * Nmax);
  if (!masks) return -3;
  for (int32_t b = 0; b < B; ++b) {
    const int32_t n = n_nodes[b];
    if (n < 1 || n > Nmax || kv_len[b] < 0 || kv_len[b] > Lcap) { free(masks); return -1; }
    uint8_t* M = masks + (size_t)b * Nmax * Nmax;
    if (fspad_oracle_dense_mask(n, parent + (size_t)b * Nmax, M) != 0) { free(masks); return -1; }
    if (packed_mask) {
      for (int32_t i = 0; i < n; ++i) {
        uint64_t word = 0;
        for (int32_t t = 0; t < n; ++t)
          if (M[(size_t)i * n + t]) word |= (uint64_t)1 << t;
        if (word != packed_mask[(size_t)b * Nmax + i]) { free(masks); return -2; }
      }
    }
  }
  memset(out, 0, sizeof(double) * (size_t)B * Nmax * Hq * D);

#ifdef _OPENMP
#pragma omp parallel for collapse(2) num_threads(nthreads > 0 ? nthreads : 1) schedule(dynamic, 1)
#endif
  for (int32_t b = 0; b < B; ++b) {
    for (int32_t h = 0; h < Hq; ++h) {
      const int32_t n = n_nodes[b];
      const int32_t L = kv_len[b];
      const int32_t g = h / G;
      const uint8_t* M = masks + (size_t)b * Nmax * Nmax; /* [n][n] */
      double* s = (double*)malloc(sizeof(double) * (size_t)(L + n));
      if (!s) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
        status = -3;
        continue;
      }
      const double* Kc = k_cache ? k_cache + ((size_t)b * Hkv + g) * (size_t)Lcap * D : NULL;
      const double* Vc = v_cache ? v_cache + ((size_t)b * Hkv + g) * (size_t)Lcap * D : NULL;
      for (int32_t i = 0; i < n; ++i) {
        const double* qi = q + (((size_t)b * Nmax + i) * Hq + h) * D;
        double* oi = out + (((size_t)b * Nmax + i) * Hq + h) * D;
        /* scores */
        for (int32_t j = 0; j < L; ++j) {
          const double* kj = Kc + (size_t)j * D;
          double dot = 0.0;
          for (int32_t d = 0; d < D; ++d) dot += qi[d] * kj[d];
          s[j] = scale * dot;
        }
        for (int32_t t = 0; t < n; ++t) {
          if (M[(size_t)i * n + t]) {
            const double* kt = k_tree + (((size_t)b * Nmax + t) * Hkv + g) * D;
            double dot = 0.0;
            for (int32_t d = 0; d < D; ++d) dot += qi[d] * kt[d];
            s[L + t] = scale * dot;
          } else {
            s[L + t] = -INFINITY;
          }
        }
        /* softmax with max subtraction (the node itself is always visible, so max is finite) */
        double mx = -INFINITY;
        for (int32_t j = 0; j < L + n; ++j) if (s[j] > mx) mx = s[j];
        double denom = 0.0;
        for (int32_t j = 0; j < L + n; ++j) { s[j] = exp(s[j] - mx); denom += s[j]; }
        /* weighted sum of values */
        for (int32_t d = 0; d < D; ++d) oi[d] = 0.0;
        for (int32_t j = 0; j < L; ++j) {
          const double p = s[j] / denom;
          const double* vj = Vc + (size_t)j * D;
          for (int32_t d = 0; d < D; ++d) oi[d] += p * vj[d];
        }
        for (int32_t t = 0; t < n; ++t) {
          const double p = s[L + t] / denom;
          if (p == 0.0) continue; /* masked */
          const double* vt = v_tree + (((size_t)b * Nmax + t) * Hkv + g) * D;
          for (int32_t d = 0; d < D; ++d) oi[d] += p * vt[d];
        }
      }
      free(s);
    }
  }
  free(masks);
  return status;
}

/* ------------------------------------------------------------------ row argmax
 * fp32 comparison; ties go to the lowest index; -0 == +0. The paper assumes
 * finite logits; the reading taken for NaN is that it ranks as -infinity, so it
 * never beats a number (a row of only NaN / -inf gives token 0). */
static int32_t row_argmax(const float* row, int32_t V) {
  int32_t best = 0;
  float bestv = -INFINITY;
  for (int32_t v = 0; v < V; ++v) {
    const float x = (row[v] != row[v]) ? -INFINITY : row[v];
    if (x > bestv) { best = v; bestv = x; }
  }
  return best;
}

/* ------------------------------------------------------------------ greedy acceptance
 * Preliminaries, validation phase: the tree is compared strictly with the
 * target's own results; a token that differs is dropped together with all its
 * descendants. With a[i] the target's (argmax) choice after node i, node c
 * survives iff its parent survives and draft_tokens[c] == a[parent[c]]; the
 * root always survives. The step emits the draft tokens of the deepest
 * surviving path and then the target's own choice after its last node.
 *
 * Layouts: logits fp32, row (b,i) at (b*Nmax+i)*row_stride; draft_tokens, parent,
 * path, tokens [B,Nmax] i32; n_nodes, path_len, n_tokens [B].
 * path/tokens entries past the length are -1. Returns 0 or -1 (ill-formed tree). */
int fspad_oracle_accept_greedy(int32_t B, int32_t Nmax, int32_t V,
                               const float* logits, int64_t row_stride,
                               const int32_t* draft_tokens, const int32_t* parent,
                               const int32_t* n_nodes,
                               int32_t* path, int32_t* path_len,
                               int32_t* tokens, int32_t* n_tokens) {
  if (B < 1 || Nmax < 1 || Nmax > ORACLE_MAX_NODES || V < 1) return -1;
  for (int32_t b = 0; b < B; ++b) {
    const int32_t n = n_nodes[b];
    const int32_t* par = parent + (size_t)b * Nmax;
    const int32_t* tok = draft_tokens + (size_t)b * Nmax;
    int32_t* pth = path + (size_t)b * Nmax;
    int32_t* out = tokens + (size_t)b * Nmax;
    if (n < 1 || n > Nmax || par[0] != -1) return -1;
    for (int32_t i = 1; i < n; ++i) if (par[i] < 0 || par[i] >= i) return -1;
    for (int32_t i = 0; i < Nmax; ++i) { pth[i] = -1; out[i] = -1; }

    int32_t cur = 0, len = 1;
    pth[0] = 0;
    for (;;) {
      const int32_t a = row_argmax(logits + ((size_t)b * Nmax + cur) * row_stride, V);
      int32_t next = -1;
      for (int32_t c = cur + 1; c < n; ++c)
        if (par[c] == cur && tok[c] == a) { next = c; break; }
      if (next < 0) { out[len - 1] = a; break; } /* bonus: the target's own token */
      out[len - 1] = tok[next];
      pth[len] = next;
      ++len;
      cur = next;
    }
    path_len[b] = len;
    n_tokens[b] = len;
  }
  return 0;
}

/* ------------------------------------------------------------------ sampling acceptance
 * Experiments "Settings" (temperature 1) and the caption of Table 1: the
 * acceptance condition is not relaxed, so the emitted text is distributed as
 * the target's own sampling. The rule is the accept-or-resample test of the
 * speculative sampling the paper's Introduction builds on, with the draft
 * proposal at a child a point mass (the children are a deterministic top-k,
 * Preliminaries, last paragraph): accept child token x with probability p(x)
 * under the current (residual) target distribution p; on rejection remove x from
 * p and renormalise; when no child is accepted draw the step's last token from
 * the residual. All randomness comes in as uniforms in [0,1).
 *
 * Unnormalised weights keep the arithmetic to what is written here:
 *   w[v] = exp((l[v] - max l) / T),  Z = sum_v w[v]  (vocabulary order)
 *   accept x   <=>  u_acc * Z < w[x]          (strict: p = 0 never accepts)
 *   reject x   :    Z -= w[x]; w[x] = 0
 *   bonus      :    t = u_bonus * Z; first v whose running sum of w exceeds t;
 *                   if rounding leaves none, the last v with w[v] > 0 (0 if none)
 * NaN logits carry zero weight and are skipped by the max.
 *
 * uniforms [B,2,Nmax] fp32: [b,0,i] tested when node i is proposed, [b,1,i] used
 * when the walk stops at node i.
 * min_margin [B] (may be NULL): the smallest relative distance of any decision
 * from its threshold, |u*Z - w[x]| / Z for tests and the distance of t from the
 * two running-sum values that bracket the bonus token, / Z. A caller comparing
 * another fp64 implementation bit-for-bit should discard cases whose margin is
 * near rounding level.
 * Returns 0, -1 (shape/tree), -3 (no memory), -6 (temperature). */
int fspad_oracle_accept_sample(int32_t B, int32_t Nmax, int32_t V,
                               const float* logits, int64_t row_stride,
                               const int32_t* draft_tokens, const int32_t* parent,
                               const int32_t* n_nodes,
                               float temperature, const float* uniforms,
                               int32_t* path, int32_t* path_len,
                               int32_t* tokens, int32_t* n_tokens,
                               double* min_margin) {
  if (B < 1 || Nmax < 1 || Nmax > ORACLE_MAX_NODES || V < 1) return -1;
  if (!(temperature > 0.0f) || isinf(temperature)) return -6;
  const double T = (double)temperature;
  double* w = (double*)malloc(sizeof(double) * (size_t)V);
  if (!w) return -3;
  for (int32_t b = 0; b < B; ++b) {
    const int32_t n = n_nodes[b];
    const int32_t* par = parent + (size_t)b * Nmax;
    const int32_t* tok = draft_tokens + (size_t)b * Nmax;
    const float* u_acc = uniforms + (size_t)b * 2 * Nmax;
    const float* u_bonus = u_acc + Nmax;
    int32_t* pth = path + (size_t)b * Nmax;
    int32_t* out = tokens + (size_t)b * Nmax;
    if (n < 1 || n > Nmax || par[0] != -1) { free(w); return -1; }
    for (int32_t i = 1; i < n; ++i) if (par[i] < 0 || par[i] >= i) { free(w); return -1; }
    for (int32_t i = 0; i < Nmax; ++i) { pth[i] = -1; out[i] = -1; }

    double margin = INFINITY;
    int32_t cur = 0, len = 1;
    pth[0] = 0;
    for (;;) {
      const float* row = logits + ((size_t)b * Nmax + cur) * row_stride;
      double mx = -INFINITY;
      for (int32_t v = 0; v < V; ++v) if (row[v] == row[v] && (double)row[v] > mx) mx = (double)row[v];
      double Z = 0.0;
      for (int32_t v = 0; v < V; ++v) {
        w[v] = (row[v] == row[v]) ? exp(((double)row[v] - mx) / T) : 0.0;
        Z += w[v];
      }
      int32_t next = -1;
      for (int32_t c = cur + 1; c < n && next < 0; ++c) {
        if (par[c] != cur) continue;
        const int32_t x = tok[c];
        const double wx = (x >= 0 && x < V) ? w[x] : 0.0;
        const double lhs = (double)u_acc[c] * Z;
        const double m = fabs(lhs - wx) / Z;
        if (m < margin) margin = m;
        if (lhs < wx) {
          next = c;
        } else {
          Z -= wx;
          if (x >= 0 && x < V) w[x] = 0.0;
        }
      }
      if (next >= 0) {
        out[len - 1] = tok[next];
        pth[len] = next;
        ++len;
        cur = next;
        continue;
      }
      /* no child accepted: draw the last token from the residual */
      const double t = (double)u_bonus[cur] * Z;
      double run = 0.0, before = 0.0;
      int32_t bonus = -1, last_pos = -1;
      for (int32_t v = 0; v < V; ++v) {
        if (w[v] > 0.0) last_pos = v;
        before = run;
        run += w[v];
        if (run > t) { bonus = v; break; }
      }
      if (bonus >= 0) {
        const double lo = (t - before) / Z, hi = (run - t) / Z;
        if (lo < margin) margin = lo;
        if (hi < margin) margin = hi;
      } else {
        bonus = last_pos < 0 ? 0 : last_pos;
        margin = 0.0; /* decided by the rounding fallback: not a robust case */
      }
      out[len - 1] = bonus;
      break;
    }
    path_len[b] = len;
    n_tokens[b] = len;
    if (min_margin) min_margin[b] = margin;
  }
  free(w);
  return 0;
}
