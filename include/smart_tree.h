/*
 * smart_tree.h -- C ABI of the tree-verification hot path of SMART speculative
 * decoding on AMD MI355X (gfx950).
 *
 * One speculative-decoding step, as the paper frames it (Sec. 1; Sec. 3.2;
 * Algorithm 1): a draft model proposes candidate continuations, a tree of them
 * is chosen, the target model verifies the whole tree in one forward pass, and
 * the longest accepted path is kept.  This library provides the four
 * data-parallel pieces of that step which do not need model weights:
 *
 *   smart_select_tree      which candidates form each sequence's tree
 *                          (Sec. 3.2, Eqs. "definition" .. "decision_rule",
 *                          Algorithm 1)
 *   smart_cost_tables,     the fitted device cost models of Sec. 3.1 and the cost
 *   smart_fit_cost_models  tables the selection rule consumes
 *   tree_pack              depth / position ids / ancestor bitmasks of the
 *                          chosen trees (what "verify the tree in a single
 *                          forward pass", Sec. 1, needs as mask and positions)
 *   tree_verify_attention  attention of every tree node over its sequence's
 *                          paged KV prefix plus its own ancestors (the
 *                          attention sub-step of that forward pass)
 *   tree_accept            greedy longest accepted path ("accepted" prefix by
 *                          prefix, Sec. 3.1 below Eq. "cum_prob")
 *   tree_rope              rotates the tree's queries and keys by their position
 *                          ids (for rotary-embedding target models)
 *   tree_accept_sample     temperature-1 (sampling) verification, lossless for
 *                          deterministic proposals
 *   kv_cache_write         writes token K/V rows into the paged cache in the
 *                          layout tree_verify_attention streams fastest
 *   tree_commit            appends the accepted path's K/V rows to the cache and
 *                          advances the prefix lengths (closes the step's loop)
 *
 * Conventions
 *   - Every function returns int32_t: SMART_OK (0) or a negative error code.
 *     All argument checks happen on the host before anything is enqueued, so a
 *     non-zero return means no kernel was launched and no output was touched.
 *   - Pointers named d_* are device memory, h_* host memory.  The caller owns
 *     every buffer passed in; the library neither frees nor retains them.
 *   - A smart_ctx owns only internal device workspace (split-KV partial
 *     results and the launch plan).  It is bound to one device.
 *   - Device entry points are asynchronous on the given hipStream_t (passed as
 *     void*; NULL is the default stream) and never synchronise, except that
 *     growing the workspace inside tree_verify_attention synchronises the
 *     stream once (avoid by calling smart_reserve up front).
 *   - Calls that share one smart_ctx must be issued on one stream or otherwise
 *     serialised by the caller: they share its workspace.
 *   - Element types: SMART_F32 (float) or SMART_BF16 (bfloat16, upper half of
 *     an IEEE binary32, round-to-nearest-even on output).
 *   - Trees: local node 0 of every sequence is the root; parent[i] < i
 *     (any topological order); at most SMART_MAX_NODES nodes per sequence.
 */
#ifndef SMART_TREE_H_
#define SMART_TREE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SMART_MAX_NODES 128

enum {
  SMART_OK = 0,
  SMART_EINVAL = -1, /* null pointer, bad shape / stride / dtype / option        */
  SMART_ETREE = -2,  /* malformed candidate forest or tree (host-checked inputs) */
  SMART_ECAP = -3,   /* an output buffer's stated capacity is too small          */
  SMART_EHIP = -4,   /* a HIP runtime call failed; see smart_last_hip_error      */
  SMART_ENOMEM = -5  /* workspace allocation failed                              */
};

enum { SMART_F32 = 0, SMART_BF16 = 1 };
/* tva_params.d_status values */
enum { SMART_TVA_BAD_BLOCK = 1 };
/* Element type of an fp8 KV cache (cache only; q, tree k / v and outputs stay SMART_F32 / SMART_BF16):
 * E4M3 of the OCP 8-bit floating point specification (bias 7, no infinities, largest value 448). */
enum { SMART_FP8_E4M3 = 2 };

/* Paged KV-cache layouts.  A page is the block_size x head_dim elements of one
 * (physical block, kv head); pages are addressed by block_stride / head_stride
 * (in elements).
 *   SMART_KV_PLAIN        element (slot, d) at slot * token_stride + d
 *   SMART_KV_INTERLEAVED  groups of 8 elements are matrix-core operand vectors:
 *                         K: ((d / 8) * block_size + slot) * 8 + d % 8
 *                         V: ((slot / 8) * head_dim + d) * 8 + slot % 8
 *                         (page contiguous; block_size and head_dim multiples of 8)
 * The bf16 matrix-core kernel requires SMART_KV_INTERLEAVED, block_size 16 and
 * head_dim 128; every other combination runs a slower general kernel. */
enum { SMART_KV_PLAIN = 0, SMART_KV_INTERLEAVED = 1 };

/* smart_select_tree modes */
enum { SMART_BEST_FIRST = 0, SMART_LAYERWISE = 1 };
enum { SMART_DILUTION_NONE = 0, SMART_DILUTION_PATH_MEAN = 1 };

/* tree_rope pairings */
enum { SMART_ROPE_HALF_SPLIT = 0, SMART_ROPE_INTERLEAVED = 1 };

/* smart_set_option keys */
enum {
  SMART_OPT_TVA_WORKERS = 1,      /* number of split-KV workers (waves); 0 = automatic   */
  SMART_OPT_TVA_FORCE_GENERAL = 2, /* 1 = always run the general (non matrix-core) kernel */
  SMART_OPT_TVA_PROFILE_STRIDE = 4, /* record every value-th tree_verify_attention call only
                                      (default 1)                                          */
  SMART_OPT_TVA_PROFILE = 3        /* n > 0: keep n pairs of HIP events and record one pair
                                      on the dominant attention kernel of every
                                      tree_verify_attention call (ring; the matrix-core path
                                      attaches the pair to the kernel's dispatch, so it holds
                                      the kernel's own start and end); 0 = off (default)   */
};

typedef struct smart_ctx smart_ctx;

const char* smart_strerror(int32_t code);
/* hipError_t value of the most recent failing HIP call on this thread (0 if none). */
int32_t smart_last_hip_error(void);

/* Creates a context on device `device_id` (must be a gfx950 device for the
 * device entry points to work).  Allocates nothing on the device yet. */
int32_t smart_create(smart_ctx** out_ctx, int32_t device_id);
/* Frees the workspace.  Synchronises the device. */
int32_t smart_destroy(smart_ctx* ctx);
/* Pre-sizes the attention workspace for calls with at most this many sequences,
 * total tree nodes, query heads and kv heads (head_dim <= 128), so that later
 * tree_verify_attention calls do not allocate. */
int32_t smart_reserve(smart_ctx* ctx, int32_t max_batch, int32_t max_total_nodes,
                      int32_t max_q_heads, int32_t max_kv_heads);
int32_t smart_set_option(smart_ctx* ctx, int32_t key, int64_t value);
/* Profiling read-out (see SMART_OPT_TVA_PROFILE).  The caller must have
 * synchronised the stream(s) the recorded calls ran on.  Writes the duration in
 * milliseconds of the dominant attention kernel (the prefix-streaming kernel of
 * the matrix-core path, or the general kernel) of each call recorded since the
 * last read, oldest first, at most `cap` values (only the newest n if the ring
 * wrapped), stores their number in *h_count and clears the record. */
int32_t smart_tva_profile_read(smart_ctx* ctx, float* h_ms, int32_t cap, int32_t* h_count);

/* ---------------------------------------------------------------------------
 * smart_select_tree (host, batched over sequences)
 *
 * Sec. 3.2 of the paper.  Per sequence, a candidate forest (the draft model's
 * top-k expansions with conditional probabilities p(u | path), Sec. 3.2
 * "Sequential Decision Formulation") is reduced to a tree S by the marginal
 * rule of Eq. "decision_rule": candidate u is kept iff
 *        alpha * dL(u) / dC(n)  >  L(S) / cost[n]          (strict, fp64)
 * with n = |S| (root included), cost[n] = C_spec(n) / c_T (Eq. "definition"),
 * dC(n) = h_dcost[n] if given (Eq. "marginal_cost") else cost[n+1] - cost[n],
 * P(u) the cumulative path probability (Eq. "cum_prob"),
 *   dilution NONE:      L = sum_{u in S} P(u),                  dL(u) = P(u)
 *   dilution PATH_MEAN: L = Eq. "expected_acc_length" literally, dL(u) = P(u) / #paths
 *                       (Eq. "marginal_benefit").
 *   schedule BEST_FIRST: node by node; always the unselected candidate with the
 *     largest P whose parent is selected (ties: smaller index); stops at the
 *     first failed test, at |S| = budget, or when nothing is left.
 *   schedule LAYERWISE:  Algorithm 1: per layer the terms L, n, #paths are
 *     frozen, all children of the previous layer's survivors are tested, and
 *     survivors beyond the budget are dropped lowest-P first (ties: larger
 *     index first), so |S| <= budget always (Eq. "optimization").
 * Depth is capped at max_depth.  Arithmetic is IEEE binary64, evaluated as
 * ((alpha * dL) / dC) > (L / cost[n]), no fused multiply-add; L (NONE) is
 * accumulated in selection order starting from 1.0.
 *
 * Inputs (host): h_cand_cu[batch+1] CSR offsets; per candidate, local parent
 * index (-1 only for candidate 0, the root; otherwise < own index),
 * conditional probability in [0,1] (ignored for the root), token id.
 * h_cost[budget+2]; h_dcost[budget+1] or NULL.
 * Outputs (host): tree CSR h_out_cu[batch+1]; per node (node id = selection
 * rank for BEST_FIRST; layer then candidate index for LAYERWISE): local parent
 * node id, token, candidate index, P(u); per sequence L and R = L / cost[|S|].
 * out_cap = capacity (nodes) of the per-node outputs.
 * Errors: SMART_EINVAL (null, batch < 0, budget < 1 or > SMART_MAX_NODES,
 * alpha outside (0,1], max_depth < 0, unknown mode), SMART_ETREE (bad forest),
 * SMART_ECAP (out_cap too small; nothing is written in that case).
 * ------------------------------------------------------------------------- */
int32_t smart_select_tree(
    int32_t batch, const int32_t* h_cand_cu, const int32_t* h_cand_parent,
    const double* h_cand_prob, const int32_t* h_cand_token,
    const double* h_cost, const double* h_dcost,
    double alpha, int32_t max_depth, int32_t budget, int32_t schedule, int32_t dilution,
    int32_t* h_out_cu, int32_t* h_out_parent, int32_t* h_out_token,
    int32_t* h_out_cand_index, double* h_out_pathprob, int64_t out_cap,
    double* h_out_L, double* h_out_R);

/* The same with a budget of its own for every sequence (Sec. 3.2 derives one
 * per-sequence budget B = B_verify / b from the batch; a scheduler that hands
 * sequences unequal shares of B_verify passes them here): h_budgets[batch],
 * each in 1 .. max_budget; the cost tables are sized by max_budget
 * (h_cost[max_budget+2], h_dcost[max_budget+1]).  Errors as above, plus
 * SMART_EINVAL for a missing or out-of-range budget. */
int32_t smart_select_tree_budgets(
    int32_t batch, const int32_t* h_cand_cu, const int32_t* h_cand_parent,
    const double* h_cand_prob, const int32_t* h_cand_token,
    const double* h_cost, const double* h_dcost,
    double alpha, int32_t max_depth, int32_t max_budget, const int32_t* h_budgets,
    int32_t schedule, int32_t dilution,
    int32_t* h_out_cu, int32_t* h_out_parent, int32_t* h_out_token,
    int32_t* h_out_cand_index, double* h_out_pathprob, int64_t out_cap,
    double* h_out_L, double* h_out_R);

/* ---------------------------------------------------------------------------
 * smart_baseline_tree (host, batched over sequences)
 *
 * The likelihood-maximising two-phase policy the paper compares SMART with
 * (Sec. 3.1, first paragraph; Fig. "method-comparison" (a), (b)), over the same
 * candidate forests and with the same outputs as smart_select_tree, so that
 * both policies' trees can be fed to the verification kernels and their
 * modelled speedups R compared under one cost table.
 *   Expansion: layer 1 is the root's children; of every layer the k candidates
 *   with the largest cumulative probability P are expanded, their children (as
 *   the forest lists them) form the next layer; max_depth layers.
 *   Rerank: all generated candidates are ranked by P and the best g kept,
 *   besides the root.  Ties anywhere: smaller candidate index first.
 * Nodes are numbered by layer, then candidate index.  L = sum of P over the
 * kept nodes (root included), R = L / h_cost[n]; h_cost needs g + 2 entries.
 * Errors: SMART_EINVAL (null, k < 1, max_depth < 0, g outside
 * 0 .. SMART_MAX_NODES - 1), SMART_ETREE, SMART_ECAP as for smart_select_tree.
 * ------------------------------------------------------------------------- */
int32_t smart_baseline_tree(
    int32_t batch, const int32_t* h_cand_cu, const int32_t* h_cand_parent,
    const double* h_cand_prob, const int32_t* h_cand_token, const double* h_cost,
    int32_t k, int32_t max_depth, int32_t g,
    int32_t* h_out_cu, int32_t* h_out_parent, int32_t* h_out_token,
    int32_t* h_out_cand_index, double* h_out_pathprob, int64_t out_cap,
    double* h_out_L, double* h_out_R);

/* ---------------------------------------------------------------------------
 * smart_product_forest (host, batched over sequences)
 *
 * Candidate forest of a drafter whose positions are independent (appendix,
 * "Additional Experimental Results": a block-diffusion drafter yields top-k
 * candidates for every position in one pass; the tree is the Cartesian product
 * of the positions' candidates, pruned to the most probable nodes by
 * cumulative probability).  Every index sequence (j_1 .. j_l), l <= depth, is a
 * node whose parent is (j_1 .. j_{l-1}) and whose conditional probability is
 * pos_prob[l-1][j_l]; P = product along the path, multiplied root to leaf in
 * binary64.  Kept per sequence: the `cap` nodes with the largest P, root
 * included (ties: smaller depth, then the lexicographically smaller index
 * sequence), listed in that order, so a parent precedes its children.  The
 * result has the layout smart_select_tree and smart_baseline_tree read; its
 * first g + 1 candidates are the tree cut to its g most probable nodes.
 *
 * Inputs (host): h_pos_prob, h_pos_token [batch][depth][k] (probabilities in
 * [0,1], in any order).  Outputs (host): h_cand_cu[batch+1]; per candidate the
 * local parent index (-1 for the root), conditional probability (1.0 for the
 * root) and token (-1 for the root); out_cap = capacity in candidates.
 * Errors: SMART_EINVAL (null, batch < 0, depth < 0, k < 1, cap < 1, a
 * probability outside [0,1], depth * log2(k) > 62), SMART_ECAP (out_cap below
 * batch * min(cap, nodes of the product); nothing is written).
 * ------------------------------------------------------------------------- */
int32_t smart_product_forest(
    int32_t batch, int32_t depth, int32_t k, const double* h_pos_prob, const int32_t* h_pos_token,
    int32_t cap, int32_t* h_cand_cu, int32_t* h_cand_parent, double* h_cand_prob,
    int32_t* h_cand_token, int64_t out_cap);

/* ---------------------------------------------------------------------------
 * Algorithm 1 one layer at a time: smart_select_begin / smart_select_layer
 * (host) and smart_select_begin_device / smart_select_layer_device (device)
 *
 * With a live draft model the candidates of layer l exist only after the
 * survivors of layer l - 1 are known (Sec. 3.2 "Sequential Decision
 * Formulation": U_l are the expansions of the active set A_{l-1}).  These calls
 * run one iteration of Algorithm 1's loop per call: the caller offers, per
 * sequence, the children of the newest layer's nodes with their conditional
 * draft probabilities; every candidate is tested with the terms L, n, #paths
 * of the tree before this layer (frozen); survivors beyond the budget are
 * dropped lowest-P first (ties: larger index first); survivors are appended in
 * candidate order and become the active set of the next call.  Feeding a
 * forest's layers one by one gives exactly the tree, L and R that
 * smart_select_tree with SMART_LAYERWISE gives for the whole forest.
 * The device form is the same arithmetic in binary64 on the GPU, one wavefront
 * per sequence, for draft probabilities that never leave the device; nothing
 * synchronises.
 *
 * smart_layer_state: the trees under construction, caller-owned arrays (all
 * host pointers for the host calls, all device pointers for the device calls;
 * the struct itself is always read on the host).  Node arrays have `budget`
 * entries per sequence.  path_sum may be NULL with SMART_DILUTION_NONE.
 * smart_select_begin(_device) sets every tree to its root.
 *
 * smart_select_layer: h_cand_cu[batch+1] CSR offsets of this layer's
 * candidates (a sequence may offer none); per candidate the node id (within
 * its sequence's tree) it extends, which must be one of layer_begin .. n-1,
 * its conditional probability in [0,1] and its token.  h_out_node[c] receives
 * the candidate's new node id or -1.  h_cost[budget+2], h_dcost[budget+1] or
 * NULL, alpha and dilution as for smart_select_tree (same dilution on every
 * call of one tree).  After the call n, layer_begin (= the old n), sum_P, the
 * node arrays, L and R = L / cost[n] are current.  A sequence whose tree is
 * full, or whose layer keeps nothing, ends with an empty active set.
 * Errors (host form; nothing is modified): SMART_EINVAL (null pointers, budget
 * outside 1..SMART_MAX_NODES, alpha outside (0,1], unknown dilution, PATH_MEAN
 * without path_sum), SMART_ETREE (offsets not ascending from 0, state
 * inconsistent, a parent outside the newest layer, a probability outside
 * [0,1]).
 * Device form: cand_cap is the capacity (entries) of the candidate arrays and
 * d_out_node; per sequence d_status[b] = SMART_OK, SMART_ETREE (as above; also
 * offsets leaving [0, cand_cap]) or SMART_ECAP (more than
 * SMART_MAX_LAYER_CAND candidates); a sequence with a non-zero status is left
 * as it was and its candidates (where addressable) get -1.
 * ------------------------------------------------------------------------- */
#define SMART_MAX_LAYER_CAND 2048

typedef struct smart_layer_state {
  int32_t batch;
  int32_t budget;       /* nodes a tree may hold, root included (1 .. SMART_MAX_NODES) */
  int32_t* n;           /* [batch] nodes so far                                          */
  int32_t* layer_begin; /* [batch] first node of the newest layer (active set: .. n-1)  */
  double* sum_P;        /* [batch] sum of P over the nodes, in node order                */
  int32_t* parent;      /* [batch * budget] local parent node id, -1 for the root        */
  int32_t* token;       /* [batch * budget]                                              */
  double* pathprob;     /* [batch * budget] P(u), Eq. "cum_prob"                         */
  double* path_sum;     /* [batch * budget] sum of P from the root down to the node      */
  double* L;            /* [batch] expected acceptance length of the current tree        */
  double* R;            /* [batch] L / cost[n]                                           */
} smart_layer_state;

int32_t smart_select_begin(const smart_layer_state* h_state, const int32_t* h_root_token,
                           const double* h_cost);
int32_t smart_select_layer(const smart_layer_state* h_state, const int32_t* h_cand_cu,
                           const int32_t* h_cand_parent_node, const double* h_cand_prob,
                           const int32_t* h_cand_token, const double* h_cost, const double* h_dcost,
                           double alpha, int32_t dilution, int32_t* h_out_node);
int32_t smart_select_begin_device(smart_ctx* ctx, void* stream, const smart_layer_state* d_state,
                                  const int32_t* d_root_token, const double* d_cost);
int32_t smart_select_layer_device(smart_ctx* ctx, void* stream, const smart_layer_state* d_state,
                                  const int32_t* d_cand_cu, const int32_t* d_cand_parent_node,
                                  const double* d_cand_prob, const int32_t* d_cand_token,
                                  int64_t cand_cap, const double* d_cost, const double* d_dcost,
                                  double alpha, int32_t dilution, int32_t* d_out_node,
                                  int32_t* d_status);

/* ---------------------------------------------------------------------------
 * tree_compact_pack (device)
 *
 * Turns the trees of a smart_layer_state (device pointers) into what the rest
 * of the step takes, in one launch and without the host learning the sizes:
 * d_cu_nodes[batch+1] (running sum of n), d_parent and d_token in CSR order,
 * and the outputs of tree_pack.  total_cap, the capacity (nodes) of the
 * per-node outputs, must be at least batch * budget; the number of nodes
 * actually written is d_cu_nodes[batch].  tree_verify_attention
 * may then be called with total_nodes = total_cap (see there).
 * d_status as for tree_pack (a sequence with n outside 1 .. budget counts as
 * malformed and contributes no nodes).
 * Host errors: SMART_EINVAL (null pointers, total_cap < batch * budget).
 * ------------------------------------------------------------------------- */
int32_t tree_compact_pack(smart_ctx* ctx, void* stream, const smart_layer_state* d_state,
                          int32_t total_cap, const int32_t* d_prefix_len, int32_t* d_cu_nodes,
                          int32_t* d_parent, int32_t* d_token, int32_t* d_depth,
                          int32_t* d_position, int32_t* d_node_seq, uint64_t* d_anc_mask,
                          int32_t* d_status);

/* ---------------------------------------------------------------------------
 * smart_cost_tables, smart_fit_cost_models (host)
 *
 * The device cost models of Sec. 3.1 ("Cost Modeling"), biases fixed to zero as
 * the paper does:  C_draft(x) = lambda x  (Eq. "linear_model"),
 * C_verify(x) = gamma (exp(delta x^rho) - 1)  (Eq. "exp_model"), x = tokens
 * drafted into one forward pass.
 *
 * smart_cost_tables fills what smart_select_tree takes, in units of c_T
 * (Eq. "definition"): h_cost[n] = (C_draft + C_verify)(tokens_per_node n) / c_T
 * for n = 0 .. n_max + 1 and, if h_dcost is not NULL, the differentiated
 * marginal cost of Eq. "marginal_cost" per NODE,
 * h_dcost[n] = tokens_per_node (lambda + gamma delta rho x^(rho-1) exp(delta x^rho)) / c_T
 * at x = tokens_per_node n, for n = 0 .. n_max (n = 0 with rho < 1: +inf).
 * tokens_per_node is the batch size when a batch verifies together.
 *
 * smart_fit_cost_models fits the models to n_points timings by least squares:
 * lambda from (h_x, h_t_draft) if h_t_draft is given; gamma, delta, rho from
 * (h_x, h_t_verify) if h_t_verify is given (at least 3 points; the paper uses
 * five forward passes), searched over rho in [0.05, 4] and an exponent
 * delta max(x)^rho in [1e-6, 40]; *h_sse (may be NULL) receives the summed
 * squared residual of the verify fit.
 * Errors: SMART_EINVAL (null outputs, n_points too small, x <= 0, non-finite
 * samples, non-positive c_T / tokens_per_node / rho, negative parameters).
 * ------------------------------------------------------------------------- */
int32_t smart_cost_tables(double lambda, double gamma, double delta, double rho, double c_T,
                          double tokens_per_node, int32_t n_max, double* h_cost, double* h_dcost);
/* The same with the bias terms of Eqs. "linear_model" (beta) and "exp_model" (eta) kept, and with the first
 * undrafted_nodes nodes of a tree (the root, which every verification step carries anyway) left out of the token
 * count:  x(n) = tokens_per_node max(n - undrafted_nodes, 0),
 *   h_cost[n]  = (lambda x + beta + gamma (exp(delta x^rho) - 1) + eta) / c_T,
 *   h_dcost[n] = tokens_per_node (lambda + gamma delta rho x^(rho-1) exp(delta x^rho)) / c_T   (x = 0, rho < 1: +inf).
 * A cost measured as the extra time of a verification step over the plain decoding step c_T is eta = c_T,
 * beta = 0, undrafted_nodes = 1: then h_cost[1] = 1 exactly and h_cost[n] = 1 + model(drafted tokens) / c_T.
 * smart_cost_tables is this with zero biases and undrafted_nodes = 0.
 * Errors: as smart_cost_tables; also negative or non-finite biases, negative undrafted_nodes. */
int32_t smart_cost_tables_biased(double lambda, double beta, double gamma, double delta, double rho, double eta,
                                 double c_T, double tokens_per_node, int32_t undrafted_nodes, int32_t n_max,
                                 double* h_cost, double* h_dcost);
int32_t smart_fit_cost_models(int32_t n_points, const double* h_x, const double* h_t_draft,
                              const double* h_t_verify, double* h_lambda, double* h_gamma,
                              double* h_delta, double* h_rho, double* h_sse);

/* ---------------------------------------------------------------------------
 * tree_upload (pinned host -> device)
 *
 * smart_select_tree runs on the host (Sec. 3.2 builds the tree on the CPU side
 * of the draft/verify loop), tree_pack and the calls after it on the device.
 * This copies n_words 32-bit words of its output from PINNED host memory
 * (hipHostMalloc, or a framework's pinned allocation: memory the device can
 * address) to device memory with a copy kernel on `stream`, so the next kernel
 * on the stream follows without a hand-off between the DMA engine's queue and
 * the compute queue.  The host must leave h_pinned_src untouched until the
 * copy has run (an event recorded after this call tells).
 * Errors: SMART_EINVAL (null pointers, negative size, h_pinned_src not
 * addressable by the device: pageable memory is refused, nothing is launched).
 * ------------------------------------------------------------------------- */
int32_t tree_upload(smart_ctx* ctx, void* stream, const void* h_pinned_src, void* d_dst,
                    int64_t n_words);

/* ---------------------------------------------------------------------------
 * tree_upload_pack (pinned host -> device, then tree_pack, in one launch)
 *
 * What tree_upload of the three arrays smart_select_tree wrote followed by
 * tree_pack would do: d_cu_nodes[batch+1], d_parent[total_nodes] and (if both
 * token pointers are given) d_token[total_nodes] receive copies of the pinned
 * host arrays, and the outputs of tree_pack are produced from them.  One
 * wavefront per sequence fetches that sequence's tree over the host link and
 * packs it from LDS, which saves a kernel launch per verify step.
 * total_nodes must equal h_pinned_cu_nodes[batch] (a sequence whose offsets
 * leave [0, total_nodes] gets status SMART_ETREE and nothing of it is copied).
 * The pinned arrays must be complete when this is called (of a batch of at
 * most 64 sequences the offsets, and with at most 448 nodes in all the trees
 * too, are read by the host during the call and travel with the launch) and
 * stay untouched until the kernel has run.  On a stream that is being
 * captured into a graph nothing travels with the launch: every replay reads
 * the pinned arrays when it runs (batch and total_nodes are the graph's).
 * Errors: as tree_pack, plus SMART_EINVAL for pageable host memory and for
 * token pointers of which only one is NULL.
 * ------------------------------------------------------------------------- */
int32_t tree_upload_pack(smart_ctx* ctx, void* stream, int32_t batch, int32_t total_nodes,
                         const int32_t* h_pinned_cu_nodes, const int32_t* h_pinned_parent,
                         const int32_t* h_pinned_token /* may be NULL */,
                         int32_t* d_cu_nodes, int32_t* d_parent, int32_t* d_token /* may be NULL */,
                         const int32_t* d_prefix_len,
                         int32_t* d_depth, int32_t* d_position, int32_t* d_node_seq,
                         uint64_t* d_anc_mask, int32_t* d_status);

/* ---------------------------------------------------------------------------
 * tree_pack (device)
 *
 * For every node i of every sequence b (local ids):
 *   depth[i]    = 0 for the root, depth[parent[i]] + 1 otherwise
 *   position[i] = prefix_len[b] + depth[i]          (the node's position id)
 *   node_seq[i] = b
 *   anc_mask[i] = 128-bit set {i} U ancestors(i): word 0 holds bits 0..63,
 *                 word 1 bits 64..127; layout [total_nodes][2]
 * d_status[b] = 0, or SMART_ETREE if sequence b's tree is malformed (no node,
 * more than SMART_MAX_NODES nodes, parent[0] != -1, parent[i] outside [0, i));
 * outputs of a malformed sequence are zero-filled.
 * Host errors: SMART_EINVAL (null pointers, negative sizes).
 * ------------------------------------------------------------------------- */
int32_t tree_pack(smart_ctx* ctx, void* stream, int32_t batch, int32_t total_nodes,
                  const int32_t* d_cu_nodes, const int32_t* d_parent, const int32_t* d_prefix_len,
                  int32_t* d_depth, int32_t* d_position, int32_t* d_node_seq,
                  uint64_t* d_anc_mask, int32_t* d_status);

/* ---------------------------------------------------------------------------
 * tree_rope (device)
 *
 * Rotary position embedding of the tree's queries and keys, in place, by the
 * position ids tree_pack wrote (a node at depth d of sequence b is verified at
 * position prefix_len[b] + d: the whole tree passes through the target model
 * at once, Sec. 1).  Pair i (i = 0 .. rotary_dim/2 - 1) of every head of node
 * t is turned by the angle d_position[t] * base^(-2 i / rotary_dim):
 *   (x, y) -> (x cos - y sin, x sin + y cos),
 *   SMART_ROPE_HALF_SPLIT:  (x, y) = (v[i], v[i + rotary_dim/2])
 *   SMART_ROPE_INTERLEAVED: (x, y) = (v[2i], v[2i + 1])
 * Elements from rotary_dim on are left alone.  Angles are formed in binary64,
 * the rotation in binary32; bf16 results are rounded to nearest even.
 * d_q [total_nodes][num_q_heads][head_dim], d_k_tree [total_nodes][num_kv_heads]
 * [head_dim] (either may be NULL if its head count is 0).  Call it before
 * tree_verify_attention and tree_commit, so that the cache only ever holds
 * rotated keys.  total_nodes may be a capacity (rows past the trees are
 * rotated by whatever d_position holds there; nothing reads them).
 * Host errors: SMART_EINVAL (null pointers, head_dim > 128, rotary_dim odd or
 * outside 2 .. head_dim, unknown dtype / pairing, base not positive).
 * ------------------------------------------------------------------------- */
int32_t tree_rope(smart_ctx* ctx, void* stream, int32_t dtype, int32_t total_nodes,
                  int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim, int32_t rotary_dim,
                  int32_t pairing, double base, const int32_t* d_position, void* d_q, void* d_k_tree);

/* ---------------------------------------------------------------------------
 * kv_cache_write (device)
 *
 * Copies n_tokens rows of K and V ([n_tokens][num_kv_heads][head_dim]) into the
 * paged cache: row t goes to physical block d_slot_mapping[t] / block_size,
 * slot d_slot_mapping[t] % block_size, in the given layout (negative mapping
 * entries are skipped).  This is how a prefix is laid down and how accepted
 * tree nodes are committed after tree_accept.
 * ------------------------------------------------------------------------- */
int32_t kv_cache_write(smart_ctx* ctx, void* stream, int32_t dtype, int32_t kv_layout,
                       int32_t n_tokens, int32_t num_kv_heads, int32_t head_dim,
                       int32_t block_size, int32_t num_blocks,
                       const void* d_k_src, const void* d_v_src, const int64_t* d_slot_mapping,
                       void* d_k_cache, void* d_v_cache,
                       int64_t cache_block_stride, int64_t cache_head_stride,
                       int64_t cache_token_stride /* PLAIN only */);

/* ---------------------------------------------------------------------------
 * kv_cache_write_fp8 (device)
 *
 * kv_cache_write into an fp8 cache (SMART_FP8_E4M3, one byte per element, same
 * two layouts, strides in elements): every source element x (src_dtype
 * SMART_F32 or SMART_BF16) is stored as the E4M3 value nearest to x / k_scale
 * (keys) or x / v_scale (values): binary32 division, round to nearest with
 * ties to the even mantissa, saturation at +-448, NaN kept.  Halving the bytes
 * tree_verify_attention streams is the point: the prefix kernel is bound by
 * HBM bandwidth.
 * Errors as kv_cache_write, plus SMART_EINVAL for scales that are not positive
 * and finite.
 * ------------------------------------------------------------------------- */
int32_t kv_cache_write_fp8(smart_ctx* ctx, void* stream, int32_t src_dtype, int32_t kv_layout,
                           int32_t n_tokens, int32_t num_kv_heads, int32_t head_dim,
                           int32_t block_size, int32_t num_blocks,
                           const void* d_k_src, const void* d_v_src, const int64_t* d_slot_mapping,
                           void* d_k_cache, void* d_v_cache,
                           int64_t cache_block_stride, int64_t cache_head_stride,
                           int64_t cache_token_stride /* PLAIN only */, float k_scale, float v_scale);

/* ---------------------------------------------------------------------------
 * tree_verify_attention (device)
 *
 * For every sequence b, node i of its tree, query head h (kv head g = h / G,
 * G = num_q_heads / num_kv_heads):
 *   keys   = cache tokens 0 .. prefix_len[b]-1 of b (token t lives in physical
 *            block d_block_table[b][t / block_size], slot t % block_size)
 *            followed by the tree nodes j of b with bit j set in anc_mask[i]
 *            (i itself and its ancestors)
 *   out[i,h,:] = softmax_keys(softmax_scale * <q[i,h,:], k[g,:]>) . v[g,:]
 *   lse[i,h]   = log sum_keys exp(score)                      (optional)
 * Scores, softmax and accumulation are fp32 (bf16 inputs are multiplied on
 * the matrix cores with fp32 accumulation; softmax weights are rounded to
 * bf16 before the second product).  With an fp8 cache (kv_cache_dtype =
 * SMART_FP8_E4M3) the cached keys and values are k_scale / v_scale times the
 * stored E4M3 values (exact in bf16); everything else is as above.  (The
 * matrix-core kernel then streams every sequence in row groups of 64 rows, so
 * trees with more than 64 rows per kv head re-read their prefix per group.)
 *
 * Shapes: q, out [total_nodes][Hq][D]; k_tree, v_tree [total_nodes][Hkv][D]
 * (tree K/V are not in the cache yet); block_table [batch][max_blocks_per_seq]
 * (entries past a sequence's prefix are never read; read entries are clamped
 * to [0, num_blocks) and reported through d_status); prefix_len is clamped to
 * [0, max_blocks_per_seq * block_size]; anc_mask as written by tree_pack.
 * total_nodes may exceed d_cu_nodes[batch] (a capacity, when only the device
 * knows the trees' sizes: see tree_compact_pack): rows from d_cu_nodes[batch]
 * on are then either left untouched or zero-filled, never read.
 * d_cu_nodes must be a running sum, 0 <= cu[b] <= cu[b+1] <= total_nodes; a
 * batch whose offsets are not (checked on the device) is treated as a batch of
 * empty trees by the matrix-core path (no output row is written); the general
 * kernel zero-fills the rows of a sequence whose range leaves [0, total_nodes].
 * Any group size G = Hq / Hkv is accepted (a tree's rows per kv head, n x G,
 * are served in groups of up to 256).
 * Host errors: SMART_EINVAL for null pointers, Hq % Hkv != 0,
 * total_nodes x Hq >= 2^31, head_dim not in {64, 128}, block_size not a
 * multiple of 8 or > 64, unknown dtype / layout, strides smaller than a page;
 * SMART_ENOMEM / SMART_EHIP.
 * ------------------------------------------------------------------------- */
typedef struct {
  int32_t dtype;     /* SMART_F32 | SMART_BF16: q, k, v, out share it */
  int32_t kv_layout; /* SMART_KV_PLAIN | SMART_KV_INTERLEAVED        */
  int32_t batch, total_nodes, num_q_heads, num_kv_heads, head_dim;
  int32_t block_size, max_blocks_per_seq, num_blocks;
  float softmax_scale;
  int32_t kv_cache_dtype; /* 0: the cache holds `dtype` elements; SMART_FP8_E4M3: one byte per element,
                             key = k_scale * stored value, value = v_scale * stored value (strides still
                             count elements) */
  const void* d_q;
  const void* d_k_tree;
  const void* d_v_tree;
  const void* d_k_cache;
  const void* d_v_cache;
  int64_t cache_block_stride, cache_head_stride, cache_token_stride; /* elements */
  const int32_t* d_block_table;
  const int32_t* d_prefix_len; /* [batch]   */
  const int32_t* d_cu_nodes;   /* [batch+1] */
  const uint64_t* d_anc_mask;  /* [total_nodes][2] */
  void* d_out;
  float* d_lse; /* [total_nodes][Hq] or NULL */
  /* Optional host copy of d_cu_nodes (the host that ran smart_select_tree has it), or NULL.
   * A hint only: results never depend on it and the present kernels plan on the device
   * without it.  If given it must agree with d_cu_nodes. */
  const int32_t* h_cu_nodes;
  float k_scale, v_scale; /* fp8 cache only: positive, finite */
  /* Optional [batch] (device) or NULL: per sequence 0, or SMART_TVA_BAD_BLOCK if one of the block-table entries the
   * call reads for it (the first ceil(prefix_len / block_size) of its row) lies outside [0, num_blocks).  Such an
   * entry is read as the nearest valid block, so the call stays inside the cache, but that sequence's output is
   * then not meaningful.  Written for every sequence by every call that gets the pointer and has work to launch
   * (batch > 0 and total_nodes > 0). */
  int32_t* d_status;
} tva_params;

int32_t tree_verify_attention(smart_ctx* ctx, void* stream, const tva_params* params);

/* ---------------------------------------------------------------------------
 * tree_verify_attention_static (device)
 *
 * For callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and same results as tree_verify_attention, but the
 * split-KV partial results and the launch plan live in a static device array
 * of SMART_STATIC_SCRATCH_BYTES that is part of the library's code object (one
 * copy per GPU the library runs on, held until the process ends; its address
 * on the context's device is resolved once, by smart_create).  The call
 * allocates and frees nothing and never synchronises.
 * Limits: the partial results of the call must fit the array -- SMART_ECAP if
 * they do not (nothing is enqueued then).  Their size is counted from the
 * trees' sizes when params->h_cu_nodes (host copy of d_cu_nodes) is given,
 * which is what makes the usual problem sizes fit (all workloads named in this
 * repository do); without it, from batch and total_nodes alone, assuming the
 * least favourable tree sizes.  If h_cu_nodes is given it must be a running sum
 * inside [0, total_nodes] (SMART_EINVAL otherwise); if it disagrees with
 * d_cu_nodes so that the device counts more partial results than the host left
 * room for, the call writes no output at all.  At most about a thousand
 * sequences per call (the plan's corner of the array; SMART_ECAP beyond).
 * Every call on one GPU shares that GPU's array: calls that overlap in time on
 * one GPU (different streams, different contexts, different threads) race;
 * calls on one stream do not.  The array keeps the previous call's contents;
 * nothing in it needs to start at zero, every word that is read was written
 * by the same call before.
 * The general (non matrix-core) kernel needs no scratch memory and is used as
 * in tree_verify_attention.
 * Errors: as tree_verify_attention, plus SMART_ECAP as above, and SMART_EHIP
 * if the array's address could not be resolved when the context was created.
 * ------------------------------------------------------------------------- */
#define SMART_STATIC_SCRATCH_BYTES (128u << 20)
int32_t tree_verify_attention_static(smart_ctx* ctx, void* stream, const tva_params* params);

/* ---------------------------------------------------------------------------
 * tree_accept (device)
 *
 * Greedy verification walk per sequence.  d_target_next[i] is the target
 * model's own next token after node i.  Start at the root; from node cur move
 * to the child whose drafted token equals d_target_next[cur] (smallest node id
 * among equal siblings); stop when there is none or max_depth drafts are
 * accepted.
 *   d_accept_len[b]   accepted draft nodes (root excluded)
 *   d_accept_path[b][0..max_depth]  visited local node ids, root first, -1 padded
 *   d_bonus_token[b]  d_target_next at the last node reached
 * Sequences with no node or more than SMART_MAX_NODES nodes get accept_len -1.
 * ------------------------------------------------------------------------- */
int32_t tree_accept(smart_ctx* ctx, void* stream, int32_t batch, int32_t max_depth,
                    const int32_t* d_cu_nodes, const int32_t* d_parent, const int32_t* d_token,
                    const int32_t* d_target_next,
                    int32_t* d_accept_len, int32_t* d_accept_path, int32_t* d_bonus_token);

/* ---------------------------------------------------------------------------
 * tree_accept_sample (device)
 *
 * Temperature-1 verification (the paper evaluates at temperatures 0 and 1 and
 * relies on verification being lossless, Sec. 4) for trees whose children are
 * deterministic proposals, as the tree drafters the paper builds on produce
 * them.  d_target_prob[i][0..vocab) is the distribution the target model
 * assigns after node i (binary32, row stride prob_row_stride elements).  Per
 * sequence, from the root: the current node's children are visited in node
 * order; a child proposing token x is accepted with probability
 * p(x) / (mass not yet rejected at this node), a rejected token's mass is
 * removed (a later sibling with the same token, or a token outside the
 * vocabulary, is skipped); the walk descends into an accepted child and stops
 * when no child is accepted or max_depth drafts are.  The bonus token is drawn
 * from what is left of the last node's distribution; every emitted token is
 * then distributed exactly as the target's.
 * Arithmetic is on integers: w(x) = floor(p(x) 2^32) (NaN and negatives count
 * 0, values above 1 count 1), with a 64-bit draw r and remaining weight R a
 * child is accepted iff floor(r R / 2^64) < w(x), and the bonus token is the
 * first index whose running weight sum exceeds floor(r R / 2^64).  Draws are
 * Philox-4x32-10 with counter (draw index within the sequence's step, step
 * low, step high, sequence index) and key (seed low, seed high); a draw is the
 * first two output words, low word first.  Results therefore depend only on
 * (seed, step, sequence index) and the inputs, bit for bit.
 * Outputs as tree_accept; d_bonus_token[b] = -1 if no weight is left.
 * Sequences with no node, more than SMART_MAX_NODES nodes or offsets outside
 * [0, total_nodes] get accept_len -1.
 * Host errors: SMART_EINVAL (null pointers, negative sizes, vocab < 1,
 * prob_row_stride < vocab, max_depth > SMART_MAX_NODES).
 * ------------------------------------------------------------------------- */
int32_t tree_accept_sample(smart_ctx* ctx, void* stream, int32_t batch, int32_t total_nodes,
                           int32_t max_depth, int32_t vocab,
                           const int32_t* d_cu_nodes, const int32_t* d_parent, const int32_t* d_token,
                           const float* d_target_prob, int64_t prob_row_stride,
                           uint64_t seed, uint64_t step,
                           int32_t* d_accept_len, int32_t* d_accept_path, int32_t* d_bonus_token);

/* ---------------------------------------------------------------------------
 * tree_commit (device)
 *
 * Makes the tokens a verify step produced part of their sequences (a draft
 * path is accepted prefix by prefix, Sec. 3.1 below Eq. "cum_prob"; the root is
 * the token every step yields): for i = 0 .. accept_len[b], node
 * accept_path[b][i] (depth i, position id prefix_len[b] + i) has its row of
 * d_k_tree / d_v_tree written to token position prefix_len[b] + i of sequence
 * b's paged cache (block d_block_table[b][pos / block_size], slot
 * pos % block_size, in the given layout), and
 * d_new_prefix_len[b] = prefix_len[b] + accept_len[b] + 1.
 * d_status[b] = 0; SMART_ECAP if the block table has no room for the new
 * tokens; SMART_ETREE if accept_len[b] is outside [0, max_depth], a path entry
 * is not a node of the tree or a block id is outside the cache.  A sequence
 * with a non-zero status keeps its length and nothing of it is written.
 * d_new_prefix_len must not alias d_prefix_len.
 * Host errors: SMART_EINVAL (null pointers, sizes, dtype, layout, strides as for
 * kv_cache_write).
 * ------------------------------------------------------------------------- */
int32_t tree_commit(smart_ctx* ctx, void* stream, int32_t dtype, int32_t kv_layout,
                    int32_t batch, int32_t max_depth, int32_t num_kv_heads, int32_t head_dim,
                    int32_t block_size, int32_t max_blocks_per_seq, int32_t num_blocks,
                    const int32_t* d_cu_nodes, const int32_t* d_accept_len, const int32_t* d_accept_path,
                    const void* d_k_tree, const void* d_v_tree,
                    const int32_t* d_block_table, const int32_t* d_prefix_len,
                    void* d_k_cache, void* d_v_cache,
                    int64_t cache_block_stride, int64_t cache_head_stride,
                    int64_t cache_token_stride /* PLAIN only */,
                    int32_t* d_new_prefix_len, int32_t* d_status);

/* tree_commit into an fp8 cache (SMART_FP8_E4M3): rows are quantised as kv_cache_write_fp8 does
 * (E4M3 of row / scale).  src_dtype is the type of d_k_tree / d_v_tree.  Everything else, errors
 * included, as tree_commit; SMART_EINVAL also for scales that are not positive and finite. */
int32_t tree_commit_fp8(smart_ctx* ctx, void* stream, int32_t src_dtype, int32_t kv_layout,
                        int32_t batch, int32_t max_depth, int32_t num_kv_heads, int32_t head_dim,
                        int32_t block_size, int32_t max_blocks_per_seq, int32_t num_blocks,
                        const int32_t* d_cu_nodes, const int32_t* d_accept_len, const int32_t* d_accept_path,
                        const void* d_k_tree, const void* d_v_tree,
                        const int32_t* d_block_table, const int32_t* d_prefix_len,
                        void* d_k_cache, void* d_v_cache,
                        int64_t cache_block_stride, int64_t cache_head_stride,
                        int64_t cache_token_stride /* PLAIN only */,
                        int32_t* d_new_prefix_len, int32_t* d_status, float k_scale, float v_scale);

#ifdef __cplusplus
}
#endif
#endif /* SMART_TREE_H_ */
