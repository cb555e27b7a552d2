/*
 * fspad.h - C ABI of the tree-verification hot path of draft-then-verify
 * lossless speculative decoding (arXiv 2408.15562, section "Preliminaries").
 *
 * One verification step of the target model over a flattened draft tree:
 *   1. tree-masked attention: every tree node attends to the whole prefix
 *      KV cache and, among the tree tokens, only to its ancestors and itself
 *      (Preliminaries: the draft phase ends by deriving the target's attention
 *      mask from the token tree; the validation phase applies it);
 *   2. lossless acceptance over the per-node logits: strict comparison of the
 *      tree with the target's results, differing tokens and their descendants
 *      discarded (Preliminaries, validation-phase paragraph), either greedy
 *      (temperature 0) or by rejection sampling that leaves the target's output
 *      distribution unchanged (Experiments, "Settings": temperature 1, and the
 *      caption of Table 1: acceptance conditions are not relaxed); also in the
 *      general form for drafts sampled from a draft distribution
 *      (fspad_tree_accept_sample_draft).
 * and the calls around that step:
 *   3. the same acceptance straight from the target's last hidden states, fused
 *      with the LM head (fspad_tree_accept_{greedy,sample}_lm_head);
 *   4. the commit of the accepted path's keys / values to the cache
 *      (fspad_kv_commit);
 *   5. on the draft side: the Feature Sampler (Methodology, "Feature Sampling":
 *      fspad_feature_sampler), the draft decoder layer with the doubled MLP
 *      output ("Partial Alignment Distillation": fspad_draft_layer), the top-k cut of
 *      a draft step's output and the
 *      choice of the tree from the candidates (Preliminaries, last paragraph:
 *      fspad_draft_topk, fspad_tree_build).
 *
 * Conventions that hold for every entry point:
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host
 *     addresses. Every buffer is owned by the caller. The library allocates
 *     nothing, frees nothing and never synchronises: device work is enqueued
 *     on the caller's HIP stream (`hip_stream` is a hipStream_t, NULL = the
 *     default stream) and the call returns at once.
 *   - The return code covers what the host can see (null pointers, shapes,
 *     workspace size, launch errors). Tree well-formedness of device arrays is
 *     the caller's contract; fspad_tree_validate checks host copies.
 *   - Results are deterministic from call to call (no floating-point atomics).
 *   - Tree layout: nodes 0..N-1 in topological order, node 0 is the root (the
 *     last token the target already emitted, always accepted; its K/V are not
 *     yet in the cache). parent[0] = -1 and 0 <= parent[i] < i. Siblings are
 *     ordered by draft rank; that order is the order of the rejection tests.
 */
#ifndef FSPAD_H
#define FSPAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FSPAD_MAX_NODES 64 /* one 64-bit ancestor word per node */

typedef enum {
  FSPAD_OK = 0,
  FSPAD_ERR_NULL = 1,        /* a required pointer is NULL */
  FSPAD_ERR_SHAPE = 2,       /* B<1, N<1, N>64, D not in {64,128}, Hq%Hkv!=0, V<1, n_nodes[b] not in 1..Nmax,
                                kv_len[b]<0, strides too small or not 16-byte multiples, row_stride<V */
  FSPAD_ERR_TREE = 3,        /* validate(): parent[0]!=-1, parent[i] not in [0,i), token not in [0,V),
                                two siblings with the same token */
  FSPAD_ERR_DTYPE = 4,       /* io_dtype / out_dtype combination not supported */
  FSPAD_ERR_WORKSPACE = 5,   /* workspace NULL or smaller than *_workspace_bytes() says */
  FSPAD_ERR_TEMPERATURE = 6, /* temperature <= 0 or not finite */
  FSPAD_ERR_HIP = 7          /* a HIP launch failed; hipGetLastError() has the cause */
} fspad_status;

typedef enum { FSPAD_F32 = 0, FSPAD_BF16 = 1 } fspad_dtype;

/* Geometry of one attention call. All strides are in elements of io_dtype. */
typedef struct {
  int32_t batch;           /* B >= 1 */
  int32_t n_nodes_max;     /* Nmax, 1..64: row pitch of every [B,Nmax,...] array */
  int32_t n_q_heads;       /* Hq */
  int32_t n_kv_heads;      /* Hkv, divides Hq; query head h reads kv head h / (Hq/Hkv) */
  int32_t head_dim;        /* D: 64 or 128, contiguous in every array */
  int32_t io_dtype;        /* fspad_dtype of q, k_tree, v_tree, k_cache, v_cache */
  int32_t out_dtype;       /* FSPAD_F32, or the same as io_dtype */
  float softmax_scale;     /* 0 => 1/sqrt(D) */
  int64_t cache_stride_batch; /* k_cache/v_cache element (b,g,j,d) is at                */
  int64_t cache_stride_head;  /*   b*stride_batch + g*stride_head + j*stride_token + d  */
  int64_t cache_stride_token; /* >= D; all three multiples of 8 elements (16 bytes bf16) */
  int32_t workgroups;      /* tuning: 0 = the built-in choice; 1..4096 forces the number of workgroups the
                              bf16 path spreads its key blocks over. Results do not depend on it beyond
                              fp32 rounding of the merge; fspad_tree_attn_workspace_bytes reads it too, so
                              sizing and call must see the same value */
  int32_t reserved;        /* 0 */
} fspad_attn_desc;

/*
 * Tree-masked attention (Preliminaries, validation phase: one forward of the
 * target over the flattened tree with the tree mask).
 *
 *   out[b,i,h,:] = sum_j softmax_j( scale * q[b,i,h,:] . K_j ) * V_j
 * where j runs over the kv_len[b] prefix positions of kv head g = h/(Hq/Hkv)
 * (all visible) followed by the tree tokens t < n_nodes[b] whose bit t is set
 * in anc_mask[b,i] (the ancestors of i and i itself).
 *
 *   q        dev [B,Nmax,Hq,D]   io_dtype (already position-encoded)
 *   k_tree   dev [B,Nmax,Hkv,D]  io_dtype, keys of the tree tokens
 *   v_tree   dev [B,Nmax,Hkv,D]  io_dtype
 *   k_cache  dev strided [B,Hkv,>=kv_len,D] io_dtype (may be NULL if all kv_len are 0)
 *   v_cache  dev strided, same strides
 *   kv_len   HOST [B] prefix lengths >= 0 (host, so that the split plan needs no device read)
 *   n_nodes  HOST [B] 1..Nmax
 *   anc_mask dev [B,Nmax] u64, bit t of word [b,i] set <=> t is i or an ancestor of i
 *   out      dev [B,Nmax,Hq,D] out_dtype; rows i >= n_nodes[b] are written as zeros
 *   workspace dev, at least fspad_tree_attn_workspace_bytes(desc, max_b kv_len[b]) bytes,
 *            16-byte aligned; contents on entry are ignored, undefined on exit.
 *            Two calls that may overlap in time need different workspaces.
 * Accumulation is fp32; bf16 inputs are multiplied on the matrix cores with
 * probabilities rounded to bf16.
 */
size_t fspad_tree_attn_workspace_bytes(const fspad_attn_desc* desc, int32_t max_kv_len);

fspad_status fspad_tree_attn(const fspad_attn_desc* desc,
                             const void* q, const void* k_tree, const void* v_tree,
                             const void* k_cache, const void* v_cache,
                             const int32_t* kv_len, const int32_t* n_nodes,
                             const uint64_t* anc_mask, void* out,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Greedy lossless acceptance (Preliminaries, validation phase: strict
 * comparison, differing tokens and their descendants discarded).
 *
 *   a[i]   = argmax_v logits[b,i,v]   (fp32 compare; ties -> lowest v; NaN never wins)
 *   walk   : cur = 0; while some child c of cur (lowest index first) has
 *            draft_tokens[c] == a[cur]: cur = c
 *   path   = root .. cur ; tokens = draft tokens of path[1..] then the bonus a[cur]
 *
 *   logits       dev [B,Nmax,V] fp32, row (b,i) starts at (b*Nmax+i)*row_stride
 *   draft_tokens dev [B,Nmax] i32; [b,0] is the root's token (not compared)
 *   parent       dev [B,Nmax] i32; [b,0] = -1, parent[i] < i
 *   n_nodes      dev [B] i32, 1..Nmax
 *   path         dev [B,Nmax] i32 out; path[b,0] = 0; entries >= path_len[b] are -1
 *   path_len     dev [B] i32 out, >= 1
 *   tokens       dev [B,Nmax] i32 out; tokens[b,0..len-2] = draft tokens of path[b,1..len-1],
 *                tokens[b,len-1] = bonus token (the next step's root); later entries -1
 *   n_tokens     dev [B] i32 out, = path_len[b]
 *   workspace    dev, >= fspad_tree_accept_workspace_bytes(B,Nmax,V), 16-byte aligned
 */
size_t fspad_tree_accept_workspace_bytes(int32_t B, int32_t Nmax, int32_t V);

fspad_status fspad_tree_accept_greedy(int32_t B, int32_t Nmax, int32_t V,
                                      const float* logits, int64_t row_stride,
                                      const int32_t* draft_tokens, const int32_t* parent,
                                      const int32_t* n_nodes,
                                      int32_t* path, int32_t* path_len,
                                      int32_t* tokens, int32_t* n_tokens,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * fspad_tree_accept_greedy for callers that cannot allocate device memory or pass a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels, arguments and results, with the per-(row, chunk) statistics kept in a fixed device
 * array that is part of the library image instead of a caller workspace.
 *
 *   limit   fspad_tree_accept_workspace_bytes(B,Nmax,V) <= FSPAD_STATIC_SCRATCH_BYTES (1 MiB; e.g.
 *           B*Nmax = 512 rows of V = 128256); larger problems return FSPAD_ERR_WORKSPACE and
 *           nothing is launched
 *   memory  every GPU the library runs on holds the 1 MiB array until the process ends; its
 *           address is looked up once per device, on the first call there
 *   calls   allocates nothing, frees nothing, never synchronises. All calls on one GPU share that
 *           GPU's array: two calls that may overlap in time (different streams) race; calls
 *           on one stream are ordered and need nothing cleared between them
 * Errors otherwise as for fspad_tree_accept_greedy; FSPAD_ERR_HIP if the array's address cannot
 * be resolved.
 */
#define FSPAD_STATIC_SCRATCH_BYTES (1u << 20)
fspad_status fspad_tree_accept_greedy_static(int32_t B, int32_t Nmax, int32_t V,
                                             const float* logits, int64_t row_stride,
                                             const int32_t* draft_tokens, const int32_t* parent,
                                             const int32_t* n_nodes,
                                             int32_t* path, int32_t* path_len,
                                             int32_t* tokens, int32_t* n_tokens, void* hip_stream);

/*
 * Sampling (temperature > 0) lossless acceptance: rejection sampling down the
 * tree against the residual distribution, with caller-supplied uniforms, so
 * that the emitted tokens are distributed exactly as the target's own samples
 * (Experiments "Settings", temperature 1; caption of Table 1). The draft
 * proposal at a child is a point mass (children are a deterministic top-k of
 * the draft's output, Preliminaries, last paragraph), which reduces the
 * accept-or-resample rule of the speculative sampling the paper builds on to:
 *
 *   cur = 0
 *   loop: w[v] = exp((logits[cur,v] - max_v logits[cur,v]) / T), Z = sum_v w[v]   (fp64)
 *         for each child c of cur, lowest index first, x = draft_tokens[c]:
 *             if u_acc[c] * Z < w[x]: accept, cur = c, restart loop
 *             else: Z -= w[x]; w[x] = 0         (residual: p with x removed, renormalised)
 *         none accepted: t = u_bonus[cur] * Z;
 *             bonus = first v in vocabulary order whose running sum of w exceeds t
 *             (if rounding leaves none: the last v with w[v] > 0); stop.
 *
 * Arguments as for greedy, plus:
 *   temperature  > 0, finite
 *   uniforms     dev [B,2,Nmax] fp32 in [0,1): [b,0,i] = u_acc(i) tested when node i is
 *                proposed, [b,1,i] = u_bonus(i) used if the walk stops at node i
 * w, Z and the running sums are fp64. A result is only defined bit-for-bit when
 * every comparison above has a relative margin well above fp64 rounding (the
 * tests require 1e-9).
 */
fspad_status fspad_tree_accept_sample(int32_t B, int32_t Nmax, int32_t V,
                                      const float* logits, int64_t row_stride,
                                      const int32_t* draft_tokens, const int32_t* parent,
                                      const int32_t* n_nodes,
                                      float temperature, const float* uniforms,
                                      int32_t* path, int32_t* path_len,
                                      int32_t* tokens, int32_t* n_tokens,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Lossless acceptance for drafts that were SAMPLED from a draft distribution (Introduction: the
 * draft-then-verify scheme of speculative sampling, whose accept-or-resample rule is what keeps the
 * target's output distribution; fspad_tree_accept_sample is its special case for the deterministic
 * top-k drafts of the paper's trees, where the draft distribution is a point mass).
 *
 * At a node with target distribution p = softmax(logits / T) and draft distribution
 * q = softmax(draft_logits / T), the children -- drawn from q one after another without
 * replacement, stored in that order -- are tested in order:
 *   accept x  <=>  u_acc * q(x) < p(x)                       (probability min(1, p(x) / q(x)))
 *   reject x   :   p <- max(p - q, 0) / sum_v max(p - q, 0);  q(x) <- 0,  q <- q / sum_v q
 * When no child is accepted (or the node is a leaf) the step's last token is the first v whose
 * running sum of p (vocabulary order) exceeds u_draw * sum_v p. Every emitted token then follows
 * the target's distribution at its position.
 *
 *   logits, draft_logits  dev [B,Nmax,V] fp32 with the same row_stride (>= V); row (b,i) of
 *                draft_logits is the distribution node i's children were drawn from. NaN
 *                entries carry no mass.
 *   draft_tokens, parent, n_nodes, temperature, uniforms, path, path_len, tokens, n_tokens:
 *                as for fspad_tree_accept_sample (tokens outside [0,V) are never accepted)
 *   workspace    dev, 16-byte aligned, >= fspad_tree_accept_sample_draft_workspace_bytes(B,Nmax,V)
 *                (3 V fp64 entries per sequence and the chunk statistics of both logit arrays); two
 *                calls that may overlap need different ones
 * All arithmetic that takes a decision is fp64. With at most 256 sequences and a vocabulary of at
 * most 524288 entries a sequence is walked by up to 64 workgroups that keep their shares of the
 * node's two rows in registers and meet after every rejection (a cooperative launch: all of them
 * resident; every wait is bounded all the same); otherwise, or where the device refuses such a
 * launch, by one workgroup. Either way the cost is a few passes over the two rows of every node on
 * the accepted path (not over all B*Nmax rows).
 * Error reporting on the device: path_len[b] = n_tokens[b] = -1 says that the workgroups of
 * sequence b stopped waiting for one another (they could not run side by side); the other outputs
 * of that sequence are then undefined. It cannot happen while the launch itself succeeds as a
 * cooperative one, which the runtime only grants when the whole grid fits.
 */
size_t fspad_tree_accept_sample_draft_workspace_bytes(int32_t B, int32_t Nmax, int32_t V);
fspad_status fspad_tree_accept_sample_draft(int32_t B, int32_t Nmax, int32_t V,
                                            const float* logits, const float* draft_logits, int64_t row_stride,
                                            const int32_t* draft_tokens, const int32_t* parent,
                                            const int32_t* n_nodes,
                                            float temperature, const float* uniforms,
                                            int32_t* path, int32_t* path_len,
                                            int32_t* tokens, int32_t* n_tokens,
                                            void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Greedy acceptance straight from the target's last hidden states, fused with the LM head
 * (Methodology, "LM Head": the final linear map from features to the vocabulary distribution;
 * Preliminaries, validation phase; Experiments "Settings": temperature 0). The [B*Nmax, V]
 * logits are never written to memory:
 *
 *   logits[b,i,v] = sum_k hidden[b,i,k] * lm_head[v,k]     bf16 inputs, exact products, fp32 sums
 *   target[b,i]   = the v with the largest logit (lowest v among equals; NaN never wins; a row
 *                   with nothing above -infinity takes token 0)
 *   then the walk of fspad_tree_accept_greedy with target[] in place of the row argmaxes.
 *
 *   hidden       dev [B,Nmax,hidden_dim] bf16, contiguous, 16-byte aligned (rows of unused tree
 *                slots are read but never used)
 *   lm_head      dev [V,hidden_dim] bf16, contiguous, 16-byte aligned (the weight matrix as the
 *                models store it: one row per token)
 *   flags        0, or FSPAD_WEIGHTS_PACKED (defined below): lm_head went through
 *                fspad_pack_weight(V, hidden_dim, ...) and is in tile order (same results, faster)
 *   hidden_dim   multiple of 256, 256..65536
 *   draft_tokens, parent, n_nodes, path, path_len, tokens, n_tokens: as for fspad_tree_accept_greedy
 *   node_target  dev [B,Nmax] i32 out, may be NULL: target[b,i] (-1 in unused slots)
 *   node_top     dev [B,Nmax] f32 out, may be NULL: the winning logit (-infinity in unused slots)
 *   workspace    dev, 16-byte aligned, >= fspad_tree_accept_lm_head_workspace_bytes(B,Nmax,V)
 * The sums are accumulated in fp32 by the matrix cores in an order of the library's choosing: a
 * target token is only defined bit-for-bit where the winning logit leads the runner-up by more
 * than the fp32 accumulation error (about 1e-6 of sum_k |hidden*lm_head|); the tests require that.
 * Identical weight rows give identical logits (and the lower token wins) only inside one aligned
 * group of 128 tokens: each group sums over k starting from a different offset. Results are
 * the same from run to run.
 * More than 256 rows (B*Nmax) are processed in equal groups of at most 256 that each stream the
 * weights again.
 * Errors as for fspad_tree_accept_greedy; never synchronises, allocates nothing.
 */
size_t fspad_tree_accept_lm_head_workspace_bytes(int32_t B, int32_t Nmax, int32_t V);
fspad_status fspad_tree_accept_greedy_lm_head(int32_t B, int32_t Nmax, int32_t V, int32_t hidden_dim,
                                              const void* hidden, const void* lm_head, int32_t flags,
                                              const int32_t* draft_tokens, const int32_t* parent,
                                              const int32_t* n_nodes,
                                              int32_t* path, int32_t* path_len,
                                              int32_t* tokens, int32_t* n_tokens,
                                              int32_t* node_target, float* node_top,
                                              void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Tree rejection sampling straight from the target's last hidden states, fused with the LM head
 * (Methodology, "LM Head"; Preliminaries, validation phase; Experiments "Settings": temperature 1,
 * acceptance not relaxed). The walk of fspad_tree_accept_sample over
 *
 *   logits[b,i,v] = sum_k hidden[b,i,k] * lm_head[v,k]     bf16 inputs, exact products, fp32 sums
 *
 * without the [B*Nmax, V] logits ever being written: the GEMM leaves, per row and group of 128
 * tokens, the maximum and the sum of exp((l - max)/T), and sets aside the logit of every node's
 * own token under its parent's row; the last token is drawn by locating the group that holds the
 * crossing of u_bonus * Z and recomputing that group's 128 logits.
 *
 * Arguments as for fspad_tree_accept_greedy_lm_head (without node_target / node_top) plus
 * temperature and uniforms as for fspad_tree_accept_sample; same workspace size.
 * The exponentials are evaluated in fp32 on fp32 sums of the library's own order (the recomputed
 * group is summed in yet another order), the sums in fp64: a decision (an accept test, the
 * crossing of the last draw) is only defined where its relative margin is above about 1e-5; the
 * tests compare sequences whose smallest margin exceeds 1e-4.
 * Errors as for fspad_tree_accept_sample; never synchronises, allocates nothing.
 */
fspad_status fspad_tree_accept_sample_lm_head(int32_t B, int32_t Nmax, int32_t V, int32_t hidden_dim,
                                              const void* hidden, const void* lm_head, int32_t flags,
                                              const int32_t* draft_tokens, const int32_t* parent,
                                              const int32_t* n_nodes,
                                              float temperature, const float* uniforms,
                                              int32_t* path, int32_t* path_len,
                                              int32_t* tokens, int32_t* n_tokens,
                                              void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Commit of the accepted path to the KV cache. The paper leaves this step implied
 * (Preliminaries: the tokens that pass validation extend the sequence from which the
 * next draft phase starts): the keys and values the verification forward computed for
 * the accepted nodes are appended to the cache in path order, so that the next
 * cycle's prefix holds them and its root is the bonus token.
 *
 *   for j < path_len[b], every kv head g:
 *       k_cache[b,g,kv_len[b]+j,:] = k_tree[b,path[b,j],g,:]      (v likewise)
 *   kv_len_out[b] = kv_len[b] + path_len[b]
 *
 *   desc     batch, n_nodes_max, n_kv_heads, head_dim, io_dtype and the cache strides are
 *            read; the other fields are ignored
 *   k_tree, v_tree   dev [B,Nmax,Hkv,D] io_dtype (this layer's tree keys / values)
 *   k_cache, v_cache dev strided, written; every (b,g) row must hold cache_capacity tokens
 *   cache_capacity   tokens per (b,g) row; kv_len[b] + Nmax <= cache_capacity is required
 *            (FSPAD_ERR_SHAPE otherwise: the path length is only known on the device)
 *   kv_len   HOST [B] prefix lengths before the commit (the ones the attention call took)
 *   path, path_len   dev [B,Nmax], [B]: outputs of an acceptance call. Entries outside
 *            [0,Nmax) and lengths outside [0,Nmax] are not followed (nothing is moved for them)
 *   kv_len_out       dev [B] i32 out, may be NULL
 * Cache positions other than kv_len[b] .. kv_len[b]+path_len[b]-1 are left untouched.
 */
fspad_status fspad_kv_commit(const fspad_attn_desc* desc, const void* k_tree, const void* v_tree,
                             void* k_cache, void* v_cache, int32_t cache_capacity,
                             const int32_t* kv_len, const int32_t* path, const int32_t* path_len,
                             int32_t* kv_len_out, void* hip_stream);

/*
 * Tile order for the weights of the skinny projections (an option of fspad_feature_sampler,
 * fspad_draft_layer and the LM-head acceptance; no passage of the paper: it is a storage format). A row-major [n_rows][k] bf16
 * matrix is cut into tiles of 16 rows x 32 columns, stored tile row by tile row, within a tile row
 * along k; the 1 KB of a tile holds, at byte 16 * (n + 16 g), the eight values
 * w[16 t + n][32 s + 8 g .. + 7] (t: tile row, s: tile along k, n in 0..15, g in 0..3). Rows past
 * n_rows in the last tile row are zeros. A wavefront then streams contiguous kilobytes instead of
 * sixteen 64-byte pieces a row pitch apart, which HBM serves faster (Feature Sampler at
 * 4096 / 11008: 60 instead of 74 us); results are bit-identical to those from row-major weights.
 *
 *   n_rows >= 1; k a multiple of 32; w dev [n_rows][k] bf16; packed dev,
 *   fspad_packed_weight_bytes(n_rows, k) = ceil(n_rows / 16) * 16 * k * 2 bytes (0 = bad shape);
 *   both 16-byte aligned and not overlapping. Done once per weight matrix, ahead of time.
 */
#define FSPAD_SAMPLER_RESIDUAL 1 /* fspad_feature_sampler flags: add the residual f */
#define FSPAD_WEIGHTS_PACKED 2   /* flags of fspad_feature_sampler and of the LM-head acceptance: the weight
                                    matrices are in tile order */
size_t fspad_packed_weight_bytes(int32_t n_rows, int32_t k);
fspad_status fspad_pack_weight(int32_t n_rows, int32_t k, const void* w, void* packed, void* hip_stream);

/*
 * Feature Sampler of the draft model (Methodology, "Feature Sampling": three projectors and a
 * sampling operation in the intermediate space). The Up Projector lifts the feature f, the Gate
 * Projector lifts the token embedding e, the lifted embedding goes through SiLU and multiplies the
 * lifted feature element by element, the Down Projector maps the product back to the hidden size,
 * and the residual connection of the feature path is added:
 *
 *   eta[r,:] = W_down (SiLU(W_gate e[r,:]) * (W_up f[r,:])) + f[r,:]
 *   (without "+ f" unless flags has FSPAD_SAMPLER_RESIDUAL)
 *
 *   rows              1..128: the tokens of one draft step (sequences x expanded nodes)
 *   hidden_dim, intermediate_dim   multiples of 256
 *   f, e              dev [rows,hidden_dim] bf16
 *   w_up, w_gate      dev [intermediate_dim,hidden_dim] bf16 (one row per intermediate channel)
 *   w_down            dev [hidden_dim,intermediate_dim] bf16
 *   flags             FSPAD_SAMPLER_RESIDUAL | FSPAD_WEIGHTS_PACKED (the three weight matrices are then
 *                     each in the tile order of fspad_pack_weight); other bits are an error
 *   eta               dev [rows,hidden_dim] bf16 out
 *   workspace         dev, 16-byte aligned, >= fspad_feature_sampler_workspace_bytes(...)
 * All pointers 16-byte aligned, all arrays contiguous. bf16 products are exact, sums are fp32 (in a
 * fixed order: the result is the same from run to run); the gated product is rounded to bf16 before
 * the Down Projector, eta once more at the end. Never synchronises, allocates nothing.
 */
size_t fspad_feature_sampler_workspace_bytes(int32_t rows, int32_t hidden_dim, int32_t intermediate_dim);
fspad_status fspad_feature_sampler(int32_t rows, int32_t hidden_dim, int32_t intermediate_dim,
                                   const void* f, const void* e,
                                   const void* w_up, const void* w_gate, const void* w_down,
                                   int32_t flags, void* eta,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The draft model: one transformer decoder layer over the draft's token tree (Methodology, first
 * paragraph: the draft model is a Transformer Decoder Layer that maps the sequence eta to the next
 * features; "Partial Alignment Distillation": the output dimension of its MLP is doubled and both
 * halves share one residual connection, which gives the two features f~ (mapped to tokens by the
 * LM head) and f (the Feature Sampler's input of the next step)).
 *
 *   x        = eta
 *   q, k, v  = split(W_qkv rmsnorm(x; gain_attn)); q and k rotary-encoded at `positions`
 *   h        = x + W_o attn          attn = fspad_tree_attn(q, k, v | draft cache, anc_mask)
 *   m        = W_down (SiLU(W_gate rmsnorm(h; gain_mlp)) * (W_up rmsnorm(h; gain_mlp)))
 *   f~       = h + m[:, :Hd]         f = h + m[:, Hd:]
 *
 * The layer is LLaMA's: rmsnorm(x; g) = x / sqrt(mean(x^2) + rms_eps) * g; the rotary encoding
 * turns the pair (entry i, entry i + D/2) of every query and key head by
 * positions[b,n] * rope_theta^(-2i/D); no biases. The caller commits the accepted rows of k_tree /
 * v_tree to the draft's cache with fspad_kv_commit.
 *
 *   desc.attn   geometry of the draft's attention and of its cache as for fspad_tree_attn;
 *               io_dtype and out_dtype FSPAD_BF16; batch * n_nodes_max <= 128;
 *               n_q_heads * head_dim a multiple of 256
 *   hidden_dim, intermediate_dim  Hd, I: multiples of 256
 *   weights     dev bf16, row-major [out][in], 16-byte aligned: w_qkv [(Hq+2Hkv) D, Hd] (query,
 *               key, value rows in that order), w_o [Hd, Hq D], w_gate and w_up [I, Hd],
 *               w_down [2 Hd, I] (rows 0..Hd-1 produce f~, rows Hd.. produce f), gain_attn and
 *               gain_mlp [Hd]; with weights_packed = 1 the five matrices are each in the tile order
 *               of fspad_pack_weight (the gains stay as they are)
 *   eta         dev [B,Nmax,Hd] bf16
 *   positions   dev [B,Nmax] i32 (prefix length + depth of the node)
 *   k_cache, v_cache, kv_len (HOST), n_nodes (HOST), anc_mask: as for fspad_tree_attn
 *   k_tree, v_tree  dev [B,Nmax,Hkv,D] bf16 OUT: keys (rotary-encoded) and values of the nodes
 *   f_tilde, f  dev [B,Nmax,Hd] bf16 OUT; rows of unused tree slots hold unspecified values
 *   workspace   dev, 16-byte aligned, at least fspad_draft_layer_workspace_bytes(desc,
 *               max_b kv_len[b]) bytes (0 = unsupported shape); contents ignored on entry, undefined on
 *               exit; two calls that may overlap in time need different workspaces
 * Products of bf16 values are summed in fp32 in a fixed order; the activations between the
 * projections (normalised inputs, q / k / v, attention output, h, the gated product) are rounded to
 * bf16 once each, as a bf16 model stores them.
 */
typedef struct {
  fspad_attn_desc attn;
  int32_t hidden_dim;
  int32_t intermediate_dim;
  float rms_eps;     /* >= 0 */
  float rope_theta;  /* > 0, e.g. 10000 */
  int32_t weights_packed; /* 0: row-major weight matrices; 1: tile order */
} fspad_draft_layer_desc;

typedef struct {
  const void* w_qkv;
  const void* w_o;
  const void* w_gate;
  const void* w_up;
  const void* w_down;
  const void* gain_attn;
  const void* gain_mlp;
} fspad_draft_layer_weights;

size_t fspad_draft_layer_workspace_bytes(const fspad_draft_layer_desc* desc, int32_t max_kv_len);

fspad_status fspad_draft_layer(const fspad_draft_layer_desc* desc, const fspad_draft_layer_weights* weights,
                               const void* eta, const int32_t* positions,
                               const void* k_cache, const void* v_cache,
                               const int32_t* kv_len, const int32_t* n_nodes, const uint64_t* anc_mask,
                               void* k_tree, void* v_tree, void* f_tilde, void* f,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Top-k cut of a draft step's output (Preliminaries, last paragraph: the output of every draft
 * step is cut to its k most probable tokens, and the joint probabilities of the tree follow from
 * their probabilities). Per row:
 *
 *   tokens[r,0..k-1] = the k entries with the largest logit, best first (equal logits: lower
 *                      token first; NaN counts as -infinity; -0 == +0)
 *   logp[r,j]        = logits[r,tokens[r,j]] - log(sum_v exp(logits[r,v]))      (log-softmax)
 *
 *   rows        1..65535 (one per node expanded in this draft step, over all sequences)
 *   logits      dev [rows] rows of V fp32, row_stride elements apart (>= V); finite, -infinity
 *               or NaN (+infinity is not supported)
 *   k           1..min(V, FSPAD_MAX_TOPK)
 *   tokens      dev [rows,k] i32 out;  logp dev [rows,k] f32 out -- what fspad_tree_build takes as
 *               cand_token / cand_logp of the new candidates
 *   workspace   dev, 16-byte aligned, >= fspad_draft_topk_workspace_bytes(rows,V,k)
 * The sum is formed from fp32 exponentials accumulated in fp64 (logp agrees with an fp64
 * evaluation to about 1e-6); the tokens are exact. A row without a finite entry yields tokens
 * 0..k-1 and logp -infinity. V * k <= 2^24 is required. Never synchronises, allocates nothing.
 */
#define FSPAD_MAX_TOPK 16
size_t fspad_draft_topk_workspace_bytes(int32_t rows, int32_t V, int32_t k);
fspad_status fspad_draft_topk(int32_t rows, int32_t V, int32_t k, const float* logits, int64_t row_stride,
                              int32_t* tokens, float* logp,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Dynamic draft tree from its candidates (Preliminaries, last paragraph: the output of every
 * draft step is cut to its top-k, joint probabilities follow from the dependencies between the
 * tokens, and one more top-k over all tokens yields a valid tree of bounded size; the
 * paragraph before it: the tokens are then organised into a tree and the attention mask is
 * derived from it). This call covers everything after the per-step top-k: it accumulates the
 * joint scores, picks the tree, flattens it and emits the arrays the verification calls consume.
 *
 *   joint[0] = 0;  joint[c] = joint[cand_parent[c]] + cand_logp[c]    (one fp32 addition per edge)
 *   kept = root + the n_keep-1 non-root candidates with the highest joint (ties: lower index);
 *          a kept candidate whose parent is not kept is dropped with its descendants (cannot
 *          happen when all cand_logp <= 0)
 *   nodes = kept candidates in candidate order (parents precede children, siblings keep their
 *          order); parent / draft_tokens / anc_mask as every other call here expects them
 *
 *   cand_parent dev [B,M] i32: candidate index of the parent, < own index; [b,0] = -1 (root)
 *   cand_token  dev [B,M] i32
 *   cand_logp   dev [B,M] f32: conditional log-probability given the parent's path; [b,0] is
 *               ignored; NaN counts as -infinity
 *   n_cand      dev [B] i32, 1..M;  M <= FSPAD_MAX_CANDIDATES
 *   n_keep      nodes to keep, root included, 1..Nmax (Nmax <= 64)
 *   parent, draft_tokens, node_cand dev [B,Nmax] i32 out (-1 in unused slots); node_cand[b,i] is
 *               the candidate node i came from; n_nodes dev [B] i32 out; anc_mask dev [B,Nmax] u64 out
 * A parent index outside [0, own index) makes that candidate (and its descendants) unreachable:
 * it is never kept. No workspace.
 */
#define FSPAD_MAX_CANDIDATES 1024
fspad_status fspad_tree_build(int32_t B, int32_t M, int32_t Nmax, const int32_t* cand_parent,
                              const int32_t* cand_token, const float* cand_logp, const int32_t* n_cand,
                              int32_t n_keep, int32_t* parent, int32_t* draft_tokens, int32_t* n_nodes,
                              uint64_t* anc_mask, int32_t* node_cand, void* hip_stream);

/*
 * Host helpers for the tree (Preliminaries: tokens organised into a tree by
 * their dependencies, then the mask derived from the tree).
 *
 * fspad_tree_build_mask: mask_host[b,i] = bit i | mask_host[b,parent[b,i]] for
 *   i < n_nodes_host[b]; words of nodes >= n_nodes_host[b] are 0. All arrays on the
 *   host, [B,Nmax] / [B]. Returns FSPAD_ERR_TREE for an ill-formed parent array.
 * fspad_tree_validate: checks parent order, token range (tokens_host may be
 *   NULL to skip the token checks) and that no two siblings carry the same token.
 */
fspad_status fspad_tree_build_mask(int32_t B, int32_t Nmax, const int32_t* parent_host,
                                   const int32_t* n_nodes_host, uint64_t* mask_host);
fspad_status fspad_tree_validate(int32_t B, int32_t Nmax, int32_t V, const int32_t* parent_host,
                                 const int32_t* tokens_host, const int32_t* n_nodes_host);

/* Static, NUL-terminated description of a status code. */
const char* fspad_status_string(fspad_status status);

#ifdef __cplusplus
}
#endif
#endif /* FSPAD_H */
