/*
 * evict.h — C ABI of the MI355X (gfx950) library for target-side verification of a draft
 * token tree on a sparse Mixture-of-Experts transformer layer, and for EVICT's cost-aware
 * choice of the tree prefix that is worth verifying.
 *
 * Conventions (all entry points)
 *   - Plain C, no exceptions cross the boundary. Every call returns an int status:
 *     EVICT_OK, EVICT_E_INVALID (bad argument, detected on the host before anything is
 *     launched), EVICT_E_UNSUPPORTED (shape outside what the kernels cover) or EVICT_E_HIP
 *     (a HIP runtime error). evict_last_error() returns a thread-local message.
 *   - Pointers marked [dev] are device pointers owned by the caller, 16-byte aligned;
 *     pointers marked [host] are host pointers. The library owns only evict_ctx and the
 *     scratch memory inside it, allocated once in evict_create.
 *   - Work is enqueued on the caller's hipStream_t (passed as void*; NULL = default
 *     stream); nothing allocates after evict_create, and only the calls that hand a value
 *     back to the host synchronise the stream (evict_device_status, evict_profile_cost*,
 *     evict_stage_times; each says so).
 *   - Inputs are never written. Verification reads the KV cache only: keys/values of the
 *     draft nodes go to caller buffers, and only evict_kv_commit* writes them into a cache.
 *   - Trees are batched CSR-style: tree_off int32[B+1] with tree_off[0] = 0 and
 *     tree_off[B] = T (the calls that take T rely on it), node arrays concatenated, parent
 *     ids are tree-local with parent[0] = -1 and parent[i] < i (node 0 is the root
 *     x_{t+1}, which is sampled from the target and therefore always accepted and always
 *     part of every prefix; Sec. 2.1).
 *   - dtype: storage type of weights and activations; accumulation is always fp32.
 *   - A context's scratch is shared by every call that takes it: calls on one context must be
 *     ordered (same stream, or made dependent by the caller); calls that overlap on the GPU race.
 *     Separate contexts are independent. Host-side, a context is not to be used from two
 *     threads at once. Results are deterministic: no floating-point atomics, fixed summation
 *     orders, so a call repeated on the same inputs returns the same bits.
 */
#ifndef EVICT_H_
#define EVICT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EVICT_OK 0
#define EVICT_E_INVALID 1
#define EVICT_E_UNSUPPORTED 2
#define EVICT_E_HIP 3

#define EVICT_F32 0
#define EVICT_BF16 1

#define EVICT_MAX_TREE_NODES 128   /* nodes per tree in evict_verify_layer (ancestor bitmask) */
#define EVICT_MAX_SELECT_NODES 1024 /* nodes per tree in evict_select_prefix / evict_accept_path */

typedef struct evict_ctx evict_ctx;

/* Shape of one MoE decoder layer. */
typedef struct evict_model_desc {
  int32_t dtype;      /* EVICT_F32 or EVICT_BF16 */
  int32_t d;          /* model width */
  int32_t Hq;         /* query heads */
  int32_t Hkv;        /* key/value heads (Hq % Hkv == 0) */
  int32_t D;          /* head dimension (64 or 128) */
  int32_t E;          /* routed experts (the N of Sec. 2.2) */
  int32_t k;          /* experts selected per token (Eq. 4) */
  int32_t F;          /* expert hidden width */
  int32_t n_shared;   /* always-on shared experts, not part of the union */
  float rms_eps;      /* RMSNorm epsilon */
  float rope_theta;   /* rotary base; 0 disables the rotation */
  int32_t vocab;      /* vocabulary size for evict_lm_head_argmax (multiple of 16), 0 = no LM head */
  int32_t router_norm; /* weights of the k selected scores (Sec. 2.2): 0 softmax over them; 1 sigmoid of
                        * each, divided by the sum of the k sigmoids */
} evict_model_desc;

/* Device pointers to one layer's weights. Matrices are in the packed streaming layout
 * written by the evict_pack_* calls; gains are plain vectors in the storage dtype. */
typedef struct evict_layer_weights {
  const void* g_attn;        /* [dev] [d] gain of the pre-attention RMSNorm */
  const void* g_moe;         /* [dev] [d] gain of the pre-MoE RMSNorm */
  const void* wqkv_packed;   /* [dev] from evict_pack_qkv */
  const void* wo_packed;     /* [dev] from evict_pack_dense(W_o [d, Hq*D]) */
  const void* wg_packed;     /* [dev] router matrix W_g from evict_pack_dense(W_g [E, d]) */
  const void* w_gateup_packed; /* [dev] from evict_pack_experts */
  const void* w_down_packed;   /* [dev] from evict_pack_experts */
  const void* ws_gateup_packed; /* [dev] shared experts, or NULL when n_shared == 0 */
  const void* ws_down_packed;   /* [dev] shared experts, or NULL */
} evict_layer_weights;

/* Optional per-stage outputs of evict_verify_layer, each [dev] and nullable. */
typedef struct evict_layer_aux {
  void* h;              /* [T, d] storage dtype: hidden state after attention + residual */
  void* h_norm;         /* [T, d] storage dtype: RMSNorm(h), the router/expert input */
  float* router_logits; /* [T, E] W_g h_norm (Eq. 4) */
  int32_t* topk_idx;    /* [T, k] selected experts, by score descending, index ascending on ties */
  float* topk_w;        /* [T, k] softmax over the selected scores */
  int32_t* union_ids;   /* [E] activated experts ascending, tail -1 (Eq. 5) */
  int32_t* union_count; /* [1] */
  int32_t* hist;        /* [E] (token, slot) pairs per expert */
  void* q;              /* [T, Hq, D] storage dtype, after rotation */
  void* attn_out;       /* [T, Hq, D] storage dtype, attention output before W_o */
} evict_layer_aux;

int evict_version(void);
const char* evict_last_error(void);

/* Create a context for one model shape. max_tokens bounds T (sum of tree sizes in a call),
 * max_batch bounds B, max_ctx bounds any sequence's KV context length. Allocates all
 * scratch memory on the current device. Limits (EVICT_E_UNSUPPORTED beyond them):
 * max_tokens * k <= 8192, at most EVICT_MAX_TREE_NODES nodes per tree, max_ctx <= 1048576 for
 * bf16 storage and <= 12160 for fp32 storage, head dimension 64 or 128, E <= 1024 in multiples
 * of 16, rows of d elements up to 16 KiB. */
int evict_create(evict_ctx** out, const evict_model_desc* m, int max_tokens, int max_batch, int max_ctx);
int evict_destroy(evict_ctx* ctx);

/* Size in bytes of the packed form of a [rows, cols] matrix. */
size_t evict_packed_bytes(int dtype, int rows, int cols);

/* One-off weight packing, off the hot path. Sources are [dev], row-major with the
 * contraction dimension contiguous: W_q [Hq*D, d], W_k, W_v [Hkv*D, d], W_o [d, Hq*D],
 * expert W_gate, W_up [n_experts, F, d], W_down [n_experts, d, F]. Packing only reorders
 * bytes (16-row strips, 64-byte column blocks, one 1 KiB block per wavefront load). */
int evict_pack_dense(int dtype, const void* w, int rows, int cols, void* dst, void* stream);
int evict_pack_qkv(const evict_model_desc* m, const void* wq, const void* wk, const void* wv, void* dst, void* stream);
int evict_pack_experts(const evict_model_desc* m, int n_experts, const void* w_gate, const void* w_up,
                       const void* w_down, void* dst_gateup, void* dst_down, void* stream);

/* Verify all T nodes of B draft trees in one pass through one MoE decoder layer
 * (Sec. 2.1: one forward pass with the tree attention mask of Fig. 4(c); Sec. 2.2: router
 * TopK, expert union, weighted sum of the selected experts).
 *   tree_off [dev] int32[B+1], parent [dev] int32[T] (tree-local), 1 <= tree size <= 128.
 *   k_cache, v_cache [dev]: sequence b, head g, position p, channel c at
 *     base + b*kv_seq_stride + g*kv_head_stride + p*D + c (strides in elements); keys are
 *     already position-encoded. ctx_len [dev] int32[B], each <= max_ctx_host <= max_ctx.
 *   x_in [dev] [T, d] -> x_out [dev] [T, d]; k_new, v_new [dev] [T, Hkv, D] receive the
 *     draft nodes' keys (rotated at position ctx_len + depth) and values.
 *   aux: nullable, and each field nullable. */
int evict_verify_layer(evict_ctx* ctx, const evict_layer_weights* w,
                       const int32_t* tree_off, const int32_t* parent, int B, int T,
                       const void* k_cache, const void* v_cache, int64_t kv_seq_stride, int64_t kv_head_stride,
                       const int32_t* ctx_len, int max_ctx_host,
                       const void* x_in, void* x_out, void* k_new, void* v_new,
                       const evict_layer_aux* aux, void* stream);

/* The same pass through a stack of n_layers decoder layers (the target's forward over the tree,
 * Sec. 2.1): layers [host] array of n_layers weight structs; k_caches, v_caches [host] arrays
 * of n_layers [dev] cache pointers with the layout and strides of evict_verify_layer;
 * k_new, v_new [host] arrays of n_layers [dev] output pointers [T, Hkv, D]. The tree is
 * prepared once; x_out must not alias x_in. */
int evict_verify_stack(evict_ctx* ctx, const evict_layer_weights* layers, int n_layers,
                       const int32_t* tree_off, const int32_t* parent, int B, int T,
                       const void* const* k_caches, const void* const* v_caches, int64_t kv_seq_stride,
                       int64_t kv_head_stride, const int32_t* ctx_len, int max_ctx_host,
                       const void* x_in, void* x_out, void* const* k_new, void* const* v_new, void* stream);

/* On-device dispatch of the verification length (Sec. 3.3: the selected length picks the verification
 * without host logic in between). After evict_dynamic_tokens(ctx, count_dev) every call on this context
 * that takes a token count T (evict_verify_layer / _stack / _stack_paged, evict_lm_head_argmax / _logits,
 * evict_accept_path_sampled) treats T as an upper bound -- launch shapes, scratch and output rows are sized
 * for it -- and the kernels read the actual count from count_dev [dev] int32[1] when they run, clamped to
 * [1, T]. Pointing it at new_tree_off + B of evict_select_prefix makes select -> gather -> verify -> LM head
 * -> accept -> commit one sequence of launches with no host read-back, capturable as one graph. With B == 1
 * the tree size then comes from tree_off (not from T), so tree_off[B] must equal the value at count_dev.
 * Rows past the actual count are neither computed nor written. count_dev == NULL switches back to host
 * counts. evict_profile_cost* refuse to run while it is set. */
int evict_dynamic_tokens(evict_ctx* ctx, const int32_t* count_dev);

/* Target token after every node: final RMSNorm, logits = W_lm x, next = argmax over the
 * vocabulary, lowest index on equal values (the p(. | prefix of node) of Sec. 2.1 at
 * temperature 0; feeds evict_accept_path).
 *   x [dev] [T, d]; g_final [dev] [d]; wlm_packed [dev] from evict_pack_dense(W_lm [vocab, d]);
 *   next [dev] int32[T]; best_logit [dev] float[T], nullable; x_norm_out [dev] [T, d] storage
 *   dtype, nullable: the normalised input the logits were formed from. Needs vocab > 0 in the
 *   model description given to evict_create. */
int evict_lm_head_argmax(evict_ctx* ctx, const void* x, const void* g_final, const void* wlm_packed, int T,
                         int32_t* next, float* best_logit, void* x_norm_out, void* stream);

/* LM head with the full score rows kept (what acceptance under sampling needs): as
 * evict_lm_head_argmax up to the scores, written to logits [dev] float32 [T][vocab] row-major
 * (vocab from the context's model description, a multiple of 16; 16-byte aligned). */
int evict_lm_head_logits(evict_ctx* ctx, const void* x, const void* g_final, const void* wlm_packed, int T,
                         float* logits, void* x_norm_out, void* stream);

/* Offline cost profiling (Sec. 3.2.3): for every verification length k = 1..Kmax, the mean
 * latency in milliseconds of evict_verify_stack on the first k nodes of one tree (B = 1; any
 * prefix of a topologically numbered tree is a tree), `reps` timed runs after one warm-up,
 * written to cost_host [host] float[Kmax+1] (cost_host[0] = 0). Synchronises the stream.
 * The table holds the layer stack's share of an iteration only. Sec. 3.2.3 defines C(k) as the
 * latency of the whole speculative step, and a term that is constant in k (LM head, acceptance,
 * commit, drafting) moves the maximiser of Eq. 10 towards larger k: the caller adds its measured
 * per-iteration constant to every entry before uploading the table for evict_select_prefix. */
int evict_profile_cost(evict_ctx* ctx, const evict_layer_weights* layers, int n_layers, const int32_t* tree_off,
                       const int32_t* parent, int Kmax, const void* const* k_caches, const void* const* v_caches,
                       int64_t kv_head_stride, const int32_t* ctx_len, int max_ctx_host, const void* x_in, void* x_out,
                       void* const* k_new, void* const* v_new, int reps, float* cost_host, void* stream);

/* The same profiling run, also reporting what the cost grew with (Sec. 2.2, Eq. 5; App. A
 * relates the union size to the token count): union_mean_host [host] float[Kmax+1] receives,
 * for every k, the number of activated experts |union| averaged over the layers and runs of
 * that k (union_mean_host[0] = 0; NULL = not wanted). One call gives the points
 * (k, union_mean[k], cost[k]) of a cost surface over (verification length, expert union) for
 * the inputs it ran on; calls on inputs with other routing spread (wider or narrower unions
 * at the same k) fill in the second axis. 1 <= reps <= 4096. */
int evict_profile_cost_union(evict_ctx* ctx, const evict_layer_weights* layers, int n_layers, const int32_t* tree_off,
                             const int32_t* parent, int Kmax, const void* const* k_caches, const void* const* v_caches,
                             int64_t kv_head_stride, const int32_t* ctx_len, int max_ctx_host, const void* x_in,
                             void* x_out, void* const* k_new, void* const* v_new, int reps, float* cost_host,
                             float* union_mean_host, void* stream);

/* Running total of |union| (Eq. 5) over every layer pass this context has run since the last reset: what the
 * cost of a step grew with (Sec. 2.2), for callers that time stacks themselves. total_host [host] int64[1]
 * (the device counter is 32 bits wide and wraps: reset it before a measurement); reset != 0 clears the
 * counter behind the read. Synchronises the stream; not inside a graph capture. */
int evict_union_total(evict_ctx* ctx, int64_t* total_host, int reset, void* stream);

/* Cost model on the host (Sec. 3.2.3, App. A). These five take host arrays only, touch no GPU and
 * need no context; they turn the profiling points above into the table evict_select_prefix divides by.
 *
 * evict_cost_expected_union_host: out[i] = M (1 - (1 - K/M)^t[i]), the number of distinct experts
 *   t tokens activate under independent uniform top-K routing over M experts (App. A); t >= 0, not
 *   necessarily whole. t, out [host] double[n].
 * evict_cost_fit_surface_host: least squares of ms ~ a + b k + c U over n >= 3 points
 *   (k[i], u[i], ms[i]) [host] double[n]; coef [host] double[3] receives (a, b, c), *rms (NULL = not
 *   wanted) the root-mean-square residual. EVICT_E_INVALID when the points lie on one line of the
 *   (k, U) plane (the two axes cannot be told apart: profile inputs of another routing spread).
 * evict_cost_collapse_host: cost[kk] = a + b kk + c U(kk) for kk = 0..k_max, [host] float[k_max+1],
 *   with U(kk) = union_of_k[kk] where kk < n_union and the entry is > 0 (a union measured at that
 *   length), the closed form of App. A otherwise; entry 0 repeats entry 1. EVICT_E_INVALID when an
 *   entry is not positive and finite (Eq. 10 divides by it).
 * evict_cost_table_save_host / _load_host: the table as a text file, one header line
 *   "evict-cost-table 1 <k_max> <key>" and then k_max+1 values, one per line, with 9 significant digits
 *   (a float survives the round trip). key: what the table was profiled for (device, model shape,
 *   storage type, context length ...), 1 to 255 printable characters without white space, chosen by the
 *   caller. Load refuses a file whose key differs from expect_key (NULL = any key). Load with
 *   cost = NULL only reports *k_max; otherwise capacity (entries of `cost`) must be at least k_max+1, and
 *   every entry must be a positive number. */
int evict_cost_expected_union_host(int n_experts, int top_k, const double* t, int n, double* out);
int evict_cost_fit_surface_host(const double* k, const double* u, const double* ms, int n, double* coef, double* rms);
int evict_cost_collapse_host(const double* coef, int k_max, int n_experts, int top_k, const double* union_of_k,
                             int n_union, float* cost);
int evict_cost_table_save_host(const char* path, const float* cost, int k_max, const char* key);
int evict_cost_table_load_host(const char* path, const char* expect_key, float* cost, int capacity, int* k_max);

/* Union of activated experts over all verified nodes (Eq. 5) and the grouping it induces.
 *   topk_idx [dev] int32[T, k] with values in [0, E).
 *   union_ids [dev] int32[E]: activated experts ascending, tail -1; union_count [dev] int32[1];
 *   hist [dev] int32[E]; offsets [dev] int32[E+1] = exclusive prefix sum of hist;
 *   perm [dev] int32[T*k]: pair ids (token*k + slot) grouped by expert, ascending inside a
 *   group; inv [dev] int32[T*k]: position of each pair in perm. T*k <= 8192, E <= 1024. */
int evict_expert_union(evict_ctx* ctx, const int32_t* topk_idx, int T, int k, int E,
                       int32_t* union_ids, int32_t* union_count, int32_t* hist, int32_t* offsets,
                       int32_t* perm, int32_t* inv, void* stream);

/* Greedy (temperature 0) acceptance: the deterministic case of the sequential sibling rule
 * of Sec. 2.1. From the root, the first child (ascending index) whose draft token equals
 * the target's next token at the current node is accepted; the walk stops when none does.
 *   draft_tok, target_next [dev] int32[T]; path [dev] int32[B, path_stride] tree-local ids,
 *   tail -1; path_len [dev] int32[B] (>= 1); bonus_tok [dev] int32[B] = target_next at the
 *   last accepted node. Trees up to 1024 nodes; path_stride >= 1 (longer paths are
 *   truncated in `path` but counted in path_len). ctx may be NULL. */
int evict_accept_path(evict_ctx* ctx, const int32_t* tree_off, const int32_t* parent,
                      const int32_t* draft_tok, const int32_t* target_next, int B,
                      int32_t* path, int path_stride, int32_t* path_len, int32_t* bonus_tok, void* stream);

/* Acceptance under sampling: the sequential sibling rule of Sec. 2.1 (Eq. 3). The target
 * distribution after node u is softmax(logits[u] / temperature) over `vocab` tokens
 * (logits [dev] float32 [T][vocab], e.g. from evict_lm_head_logits; temperature > 0). At the
 * surviving node the children are tried in ascending index: child c is accepted when
 * u_node[c] < its token's current probability; on rejection that mass is removed and the rest
 * renormalised (Eq. 3); when no child is left, bonus_tok is drawn from the remaining
 * distribution by inverting its cumulative sum (ascending token id) at u_bonus[b]. The random
 * numbers are inputs: u_node [dev] float32 [T] (one per node, the root's is unused), u_bonus
 * [dev] float32 [B], all in [0, 1). Outputs as evict_accept_path. Arithmetic is fp32; a
 * decision whose random number lies within rounding of its threshold may differ from a
 * higher-precision evaluation. Invalid token ids (outside [0, vocab)) are never accepted and
 * set the context's status word. Needs a context (scratch for the per-node softmax
 * statistics): B <= max_batch, T <= max_tokens. */
int evict_accept_path_sampled(evict_ctx* ctx, const int32_t* tree_off, const int32_t* parent,
                              const int32_t* draft_tok, const float* logits, int vocab, float temperature,
                              const float* u_node, const float* u_bonus, int B, int T, int32_t* path,
                              int path_stride, int32_t* path_len, int32_t* bonus_tok, void* stream);

/* For callers that cannot allocate device memory (code under HIP-graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): evict_accept_path_sampled without a context's scratch.
 * The per-node softmax statistics (two floats per node) live in a static device array inside the
 * library, sized for EVICT_NOALLOC_MAX_NODES nodes per call (32 KiB, held on every GPU the library
 * runs on until the process ends); its device address is looked up on the first call on a device.
 * The call itself allocates and frees nothing. Arguments, outputs and results are exactly those of
 * evict_accept_path_sampled; ctx may be NULL (then invalid ids are not reported). T above
 * EVICT_NOALLOC_MAX_NODES returns EVICT_E_UNSUPPORTED. All calls on one GPU share the array:
 * calls that overlap on that GPU (different streams) race; calls ordered on one stream do not.
 * Nothing in the array has to start at zero (the rows a call reads it has written before). */
#define EVICT_NOALLOC_MAX_NODES 4096
int evict_accept_path_sampled_noalloc(evict_ctx* ctx, const int32_t* tree_off, const int32_t* parent,
                                      const int32_t* draft_tok, const float* logits, int vocab, float temperature,
                                      const float* u_node, const float* u_bonus, int B, int T, int32_t* path,
                                      int path_stride, int32_t* path_len, int32_t* bonus_tok, void* stream);

/* EVICT prefix selection, entirely on the device (Sec. 3.1-3.2): node score = product of
 * draft probabilities along the root path (Eq. 7, root counted as 1), nodes ranked by score
 * (Sec. 3.2.1; equal scores: lower index first, which keeps every prefix ancestor-closed),
 * S_k = running fp32 sum of the k best scores (Eq. 8), k* = smallest k in 1..min(N, Kmax)
 * maximising S_k / cost[k] (Eq. 10, evaluated as cumulative sums, division, argmax:
 * Sec. 3.2.3). All arithmetic is single IEEE fp32 operations in a fixed order.
 *   node_prob [dev] float[T] in (0, 1]; cost [dev] float[Kmax+1], cost[0] unused, all > 0.
 *   The ancestor-closure of the prefixes (Sec. 3.2.1) rests on these ranges: a probability outside
 *   [0, 1] or NaN is clamped (to 1, resp. 0) and a cost entry that is not > 0 is never selected;
 *   with a context both set a bit of its status word (EVICT_ST_BAD_PROB, EVICT_ST_BAD_COST).
 *   k_star [dev] int32[B]; keep [dev] int32[T]: kept nodes of tree b, ascending tree-local
 *   ids, written at new_tree_off[b]; new_parent [dev] int32[T] parents re-indexed into the
 *   kept set; new_tree_off [dev] int32[B+1]; est_len [dev] float[B] = S_{k*};
 *   order [dev] int32[T] nullable: full ranking per tree at tree_off[b];
 *   prefix_sum [dev] float[T] nullable: S_1..S_N per tree at tree_off[b].
 * Trees up to 1024 nodes. ctx may be NULL (then nothing is flagged). */
int evict_select_prefix(evict_ctx* ctx, const int32_t* tree_off, const int32_t* parent,
                        const float* node_prob, int B, int T, const float* cost, int Kmax,
                        int32_t* k_star, int32_t* keep, int32_t* new_parent, int32_t* new_tree_off,
                        float* est_len, int32_t* order, float* prefix_sum, void* stream);

/* Cost-agnostic ablation of the selection (Sec. 4.3.2): same ranking and prefix sums, but
 * k*[b] = the smallest k in 1..min(N_b, Kmax) with S_k / S_{N_b} >= rho (one IEEE fp32 division
 * and comparison per k; the whole budget min(N_b, Kmax) when no such k exists). rho in [0, 1];
 * rho = 1 keeps every node whose score still changes the fp32 running sum. All other
 * arguments and outputs as evict_select_prefix. */
int evict_select_prefix_coverage(evict_ctx* ctx, const int32_t* tree_off, const int32_t* parent,
                                 const float* node_prob, int B, int T, float rho, int Kmax, int32_t* k_star,
                                 int32_t* keep, int32_t* new_parent, int32_t* new_tree_off, float* est_len,
                                 int32_t* order, float* prefix_sum, void* stream);

/* Host twins of evict_accept_path, evict_select_prefix(_coverage) and evict_expert_union: the same contracts
 * (Sec. 2.1; Sec. 3.1-3.2, Eq. 7, 8, 10; Eq. 5) evaluated by plain sequential code on HOST arrays, for callers that
 * hold these small arrays on the host (a scheduler choosing a verification length, tests of the error
 * conventions). Every argument has the meaning, layout and limits of its device namesake, with [host] pointers
 * throughout; there is no context and no stream. Outputs equal the device entry points' bit for bit (selection:
 * the same single fp32 operations in the same order). Inputs the device entry points clamp and flag are
 * clamped the same way and their EVICT_ST_* bits are ORed into *status_out (nullable). They touch no GPU, are
 * not called by the device path and are no fallback for it. */
int evict_accept_path_host(const int32_t* tree_off, const int32_t* parent, const int32_t* draft_tok,
                           const int32_t* target_next, int B, int32_t* path, int path_stride, int32_t* path_len,
                           int32_t* bonus_tok);
int evict_select_prefix_host(const int32_t* tree_off, const int32_t* parent, const float* node_prob, int B, int T,
                             const float* cost, int Kmax, int32_t* k_star, int32_t* keep, int32_t* new_parent,
                             int32_t* new_tree_off, float* est_len, int32_t* order, float* prefix_sum,
                             int32_t* status_out);
int evict_select_prefix_coverage_host(const int32_t* tree_off, const int32_t* parent, const float* node_prob, int B,
                                      int T, float rho, int Kmax, int32_t* k_star, int32_t* keep, int32_t* new_parent,
                                      int32_t* new_tree_off, float* est_len, int32_t* order, float* prefix_sum,
                                      int32_t* status_out);
int evict_expert_union_host(const int32_t* topk_idx, int T, int k, int E, int32_t* union_ids, int32_t* union_count,
                            int32_t* hist, int32_t* offsets, int32_t* perm, int32_t* inv, int32_t* status_out);

/* Commit of the accepted path to the KV cache of one layer (what follows acceptance in every
 * speculative iteration, Sec. 2.1): for sequence b and j < path_len[b], the draft key/value row
 * of node path[b][j] (k_new / v_new [dev] [T][Hkv][D], storage dtype, as written by
 * evict_verify_layer: rotated at position ctx_len[b] + depth, and the j-th node of an accepted
 * path has depth j) becomes row ctx_len[b] + j of every KV head of k_cache / v_cache [dev]
 * (element strides kv_seq_stride between sequences, kv_head_stride between heads, `capacity`
 * rows per head). ctx_len_out[b] = ctx_len[b] + path_len[b]; it must not alias ctx_len (all
 * workgroups read the old length). Rows past the capacity are dropped and the length clamped;
 * that, a length outside [0, capacity] or a path entry outside its tree set the status word of
 * ctx (ctx may be NULL: no status). The commit needs the whole path: path_stride >= path_len[b].
 * When evict_accept_path had to truncate `path` (path_len[b] > path_stride) only the path_stride
 * rows that are there are committed, ctx_len_out advances by that many, and EVICT_ST_PATH_TRUNCATED
 * is set. dtype / Hkv / D describe the rows (EVICT_F32 / EVICT_BF16). */
int evict_kv_commit(evict_ctx* ctx, int dtype, int Hkv, int D, const void* k_new, const void* v_new,
                    const int32_t* tree_off, const int32_t* path, int path_stride, const int32_t* path_len,
                    void* k_cache, void* v_cache, int64_t kv_seq_stride, int64_t kv_head_stride,
                    const int32_t* ctx_len, int capacity, int32_t* ctx_len_out, int B, void* stream);

/* The same commit for all layers of a stack in one call (one launch per 64 layers): k_new,
 * v_new, k_caches, v_caches are [host] arrays of n_layers [dev] pointers as in
 * evict_verify_stack; the caches share strides and capacity. */
int evict_kv_commit_stack(evict_ctx* ctx, int dtype, int Hkv, int D, const void* const* k_new,
                          const void* const* v_new, int n_layers, const int32_t* tree_off, const int32_t* path,
                          int path_stride, const int32_t* path_len, void* const* k_caches, void* const* v_caches,
                          int64_t kv_seq_stride, int64_t kv_head_stride, const int32_t* ctx_len, int capacity,
                          int32_t* ctx_len_out, int B, void* stream);

/* Paged KV caches: the block-table layout that serving engines of the kind the method is
 * integrated into (Sec. 3.3) keep their caches in. Every layer has a key pool and a value
 * pool [dev] of n_pages pages; page g of a pool holds page_size consecutive positions of one
 * sequence: position slot r, KV head h, channel c of page g at
 *   pool + g*page_stride + h*kv_head_stride + r*D + c   (strides in elements, multiples of 8,
 *   kv_head_stride >= page_size*D, page_stride >= Hkv*kv_head_stride).
 * block_table [dev] int32[B][table_stride]: entry [b][i] is the page that holds positions
 * i*page_size .. (i+1)*page_size - 1 of sequence b, the same for every layer; entries past a
 * sequence's length are never read. page_size is a power of two in [1, 65536];
 * table_stride*page_size must cover max_ctx_host (verification) or capacity (commit). A table
 * entry outside [0, n_pages) sets a bit of the context's status word; such a key is read from
 * page 0 and such a row is not written.
 *
 * evict_verify_stack_paged: evict_verify_stack with k_pools / v_pools [host] arrays of n_layers
 * [dev] pool pointers in place of the contiguous caches; all other arguments, outputs and
 * results as there (the attention kernels look the page of every key up; nothing is copied).
 * evict_kv_commit_stack_paged: evict_kv_commit_stack writing row ctx_len[b] + j into the page
 * the table names for that position; the caller has put pages for all positions below
 * `capacity` (in positions, per sequence) into the table beforehand. */
int evict_verify_stack_paged(evict_ctx* ctx, const evict_layer_weights* layers, int n_layers, const int32_t* tree_off,
                             const int32_t* parent, int B, int T, const void* const* k_pools, const void* const* v_pools,
                             int64_t page_stride, int64_t kv_head_stride, const int32_t* block_table, int table_stride,
                             int page_size, int n_pages, const int32_t* ctx_len, int max_ctx_host, const void* x_in,
                             void* x_out, void* const* k_new, void* const* v_new, void* stream);
int evict_kv_commit_stack_paged(evict_ctx* ctx, int dtype, int Hkv, int D, const void* const* k_new,
                                const void* const* v_new, int n_layers, const int32_t* tree_off, const int32_t* path,
                                int path_stride, const int32_t* path_len, void* const* k_pools, void* const* v_pools,
                                int64_t page_stride, int64_t kv_head_stride, const int32_t* block_table, int table_stride,
                                int page_size, int n_pages, const int32_t* ctx_len, int capacity, int32_t* ctx_len_out,
                                int B, void* stream);

/* Gather rows of a [T, row_bytes] array by the kept node lists of evict_select_prefix:
 * dst row new_tree_off[b] + r = src row tree_off[b] + keep[new_tree_off[b] + r].
 * row_bytes % 4 == 0. Grid is sized for T rows; rows beyond new_tree_off[B] are untouched. */
int evict_gather_rows(const void* src, void* dst, int row_bytes, const int32_t* tree_off,
                      const int32_t* new_tree_off, const int32_t* keep, int B, int T, void* stream);

/* Host-side structural check of a batch of trees ([host] pointers): EVICT_OK, or
 * EVICT_E_INVALID when some parent[i] is outside [-1, i), a root is not -1, offsets are not
 * increasing, or a tree exceeds max_nodes. */
int evict_validate_trees_host(const int32_t* tree_off, const int32_t* parent, int B, int max_nodes);

/* Device-side status word of a context: 0, or bits set (sticky) when a kernel met an invalid
 * value, which is clamped or skipped, never dereferenced. Synchronises the stream. */
#define EVICT_ST_BAD_PARENT 1      /* parent id outside [0, i) */
#define EVICT_ST_BAD_EXPERT 2      /* expert index outside [0, E) */
#define EVICT_ST_BAD_CTXLEN 4      /* context length outside [0, max_ctx_host] / [0, capacity], or rows past the capacity */
#define EVICT_ST_BAD_TREE_SIZE 8   /* a tree of more than EVICT_MAX_TREE_NODES nodes in evict_verify_layer */
#define EVICT_ST_BAD_PAGE 16       /* block-table entry outside [0, n_pages) */
#define EVICT_ST_PATH_TRUNCATED 32 /* evict_kv_commit*: path_len exceeds path_stride */
#define EVICT_ST_BAD_PROB 64       /* evict_select_prefix*: draft probability outside [0, 1] or NaN */
#define EVICT_ST_BAD_COST 128      /* evict_select_prefix: cost entry not > 0 */
int evict_device_status(evict_ctx* ctx, int32_t* status_host, void* stream);

/* Launch-shape tuning knobs of a context (defaults are chosen in evict_create):
 *   "moe_grid"        workgroups of the grouped expert GEMMs (chunks are dealt round-robin)
 *   "moe_prefetch"    1: weight registers of the streaming GEMMs refilled right behind each MFMA where the
 *                     step count is known at compile time (default); 3: refilled per step (measurement knob)
 *   "moe_chunk_gateup", "moe_chunk_down"  units (16-row strips; strip pairs for gate/up) a
 *                     workgroup takes from the device-side work list at a time
 *   "moe_gateup_kernel" 1: gate/up projections with one (gate, up) strip pair per wavefront and the token
 *                     operand in LDS; 0: contraction split over the wavefronts of a workgroup; 2 = auto
 *                     (the former from 64 tokens on where its chunks line up with the XCDs, else from 128)
 *   "moe_lds_dma"     1 (default): that kernel stages its token operand with direct global-to-LDS loads where
 *                     the shape allows (bf16, 64 contraction blocks); 0: through registers
 *   "moe_down_kernel" 1: down projections with one 16-row strip per wavefront over the whole
 *                     contraction range (token operand staged in LDS); 0: contraction split
 *                     over the wavefronts of a workgroup like the other GEMMs
 *   "dense_nt"        16-token tiles a workgroup of the QKV / output projections takes: 1, 2, or 0 = auto
 *                     (2 from 64 tokens on)
 *   "dense_units"     consecutive 16-row strips a workgroup of the QKV projection takes, 0 = auto
 *   "moe_nt_loads"    expert weights fetched with non-temporal loads: 1, 0 (ordinary loads), 2 = auto;
 *   "dense_nt_loads"  the same for the QKV / output projections and the LM head (auto: always for the
 *                     projections; for the LM head when every strip is read by a single workgroup)
 *   "dense_kernel"    QKV / output projections: 0 contraction split over the wavefronts of a workgroup,
 *                     1 one strip per wavefront with the token operand in LDS (where its shape conditions
 *                     hold), 2 = auto (the latter from 128 or 256 tokens on); "dense_ntw" its token tiles
 *                     per workgroup, 1, 2 or 0 = auto
 *   "lm_units", "lm_nt" LM head: consecutive 16-row strips and 16-token tiles a workgroup takes, 0 = auto
 *   "attn_target_wgs" workgroups the bf16 attention kernel aims for when it cuts the context into splits
 *   "moe_nt"          16-token tiles per work-list slot of the grouped expert GEMMs: 1, 2, or 0 = auto (1)
 *   "attn_waves"      wavefronts per workgroup of that kernel: 4, 8 (two LDS buffers, next chunk fetched
 *                     during the matrix work), or 0 = auto
 *   "attn_row_blocks" workgroups per (KV split, KV head) in the bf16 attention kernel, 0 = auto
 *   "moe_pair_down"   down projection: two consecutive 16-token slots of an expert through one weight stream:
 *                     0 off, 1 on (where the kernel's LDS budget allows), 2 = auto (from 128 tokens on)
 *   "moe_down_ws"     down projection, strip-per-wavefront kernel: strips (wavefronts) per workgroup, 8, 16,
 *                     or 0 = auto (16 from 128 tokens on, from 64 at expert width 1408)
 * Returns EVICT_E_INVALID for an unknown key or a value out of range. */
int evict_tune(evict_ctx* ctx, const char* key, int value);

/* HIP-graph capture of a sequence of calls, for the launch-bound regime (small trees) and for
 * one pre-built graph per verification length as in Sec. 3.3: evict_graph_begin puts `stream`
 * (not the null stream) into capture mode; every entry point called on that stream until
 * evict_graph_end is recorded instead of run (all of them only enqueue kernels and
 * device-to-device copies; evict_device_status, evict_profile_cost and evict_stage_times
 * synchronise and must stay outside, and stage timing must be off). evict_graph_end
 * instantiates the recorded work as *out, which evict_graph_launch replays on any stream of
 * the same device. The graph holds the pointer and size arguments of the recorded calls:
 * the caller keeps those buffers alive and refreshes their contents in place between
 * launches. Launches of graphs recorded from one context share its scratch, so they must not
 * overlap each other or eager calls on that context. The context must outlive its graphs.
 * Errors: EVICT_E_INVALID (null stream, capture already open / not open, timing on),
 * EVICT_E_HIP (the capture was invalidated or could not be instantiated; *out is NULL). */
typedef struct evict_graph evict_graph;
int evict_graph_begin(evict_ctx* ctx, void* stream);
int evict_graph_end(evict_ctx* ctx, void* stream, evict_graph** out);
int evict_graph_launch(evict_graph* graph, void* stream);
int evict_graph_destroy(evict_graph* graph);

/* Measurement helpers: a plain streaming read (every byte of src read once with 16-byte
 * loads, a checksum written to sink [dev] uint32[4]) and a plain copy, used to measure the
 * achievable HBM read bandwidth of the device and to calibrate hardware byte counters against
 * a kernel of known traffic. bytes must be a multiple of 16; pointers [dev], 16-byte aligned. */
int evict_probe_read(const void* src, size_t bytes, void* sink, void* stream);
int evict_probe_copy(const void* src, void* dst, size_t bytes, void* stream);

/* Per-stage timing of evict_verify_layer with HIP events recorded on the call's stream
 * between the stages (for measurement; adds event records to the stream). Stages, in order:
 * 0 tree prep + RMSNorm, 1 QKV projection + rotation, 2 tree attention (partials + merge),
 * 3 output projection + residual, 4 router top-k, 5 expert union / grouping,
 * 6 gate/up grouped GEMM + SiLU gating, 7 down grouped GEMM, 8 shared experts, 9 combine.
 * evict_stage_times waits for the last timed call to finish and writes the milliseconds of
 * each stage of that call to ms_host [host] float[EVICT_N_STAGES]. */
#define EVICT_N_STAGES 10
int evict_stage_timing(evict_ctx* ctx, int enable);
int evict_stage_times(evict_ctx* ctx, float* ms_host);

#ifdef __cplusplus
}
#endif
#endif /* EVICT_H_ */
