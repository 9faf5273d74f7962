/*
 * CPU oracle for tree-verification attention.  TEST INFRASTRUCTURE ONLY: nothing
 * in the product path may call, link or import this file.
 *
 * What it computes (the plain definition; the paper only names the step --
 * the target model checks a whole draft tree in one forward pass, Sec. 1 -- and
 * leaves the verification mechanism unchanged, Sec. 1, contributions):
 *
 *   for every sequence b, tree node i of b, query head h (kv head g = h / G):
 *     keys(i)  = { cache token t : 0 <= t < prefix_len[b] }
 *              U { tree node j of b : j is i itself or an ancestor of i }
 *     s_x      = scale * <q[i,h,:], k_x[g,:]>
 *     p        = softmax_x(s_x)                  (max-subtracted, two passes)
 *     out[i,h] = sum_x p_x * v_x[g,:]
 *     lse[i,h] = max_x s_x + log sum_x exp(s_x - max)
 *
 * Cache token t of sequence b lives in physical block
 * block_table[b][t / block_size], slot t % block_size, of a cache laid out
 * [block][kv head][slot][dim] through the element strides given.  The ancestor
 * set is obtained by walking the parent array, never from a bitmask.
 *
 * All arithmetic is fp64.  Inputs of type f32 or bf16 are converted exactly.
 * No blocking, no fusion, no reordering beyond the definition above.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { REF_F32 = 0, REF_BF16 = 1, REF_F64 = 2 };

static double load_elem(const void* base, int dtype, int64_t idx) {
  if (dtype == REF_F32) return (double)((const float*)base)[idx];
  if (dtype == REF_F64) return ((const double*)base)[idx];
  /* bf16: the upper 16 bits of an IEEE binary32 */
  uint32_t bits = ((uint32_t)((const uint16_t*)base)[idx]) << 16;
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

int tree_attention_ref_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * n_sel < 0 : compute every (node, head); out is [total_nodes][Hq][D], lse is
 *             [total_nodes][Hq].
 * n_sel >= 0: compute only the pairs (sel_node[s], sel_head[s]); out is
 *             [n_sel][D], lse is [n_sel].
 * Returns 0, or a negative value for malformed input (nothing is written then).
 */
int tree_attention_ref(
    int dtype, int batch, int num_q_heads, int num_kv_heads, int head_dim,
    int block_size, double scale,
    const void* q,        /* [total_nodes][Hq][D]  */
    const void* k_tree,   /* [total_nodes][Hkv][D] */
    const void* v_tree,   /* [total_nodes][Hkv][D] */
    const void* k_cache, const void* v_cache,
    int64_t block_stride, int64_t head_stride, int64_t token_stride,
    const int32_t* block_table, int max_blocks_per_seq,
    const int32_t* prefix_len,  /* [batch]   */
    const int32_t* cu_nodes,    /* [batch+1] */
    const int32_t* parent,      /* [total_nodes], local index, -1 for the root */
    int64_t n_sel, const int32_t* sel_node, const int32_t* sel_head,
    double* out, double* lse) {
  if (batch < 0 || num_kv_heads <= 0 || num_q_heads % num_kv_heads != 0 ||
      head_dim <= 0 || block_size <= 0)
    return -1;
  const int Hq = num_q_heads, Hkv = num_kv_heads, D = head_dim;
  const int G = Hq / Hkv;
  const int total_nodes = cu_nodes[batch];

  /* node -> sequence */
  int32_t* node_seq = (int32_t*)malloc(sizeof(int32_t) * (size_t)(total_nodes > 0 ? total_nodes : 1));
  if (!node_seq) return -2;
  int max_keys = 0;
  for (int b = 0; b < batch; ++b) {
    int n_b = cu_nodes[b + 1] - cu_nodes[b];
    if (n_b < 0 || prefix_len[b] < 0 ||
        (int64_t)prefix_len[b] > (int64_t)max_blocks_per_seq * block_size) {
      free(node_seq);
      return -1;
    }
    for (int i = 0; i < n_b; ++i) {
      int p = parent[cu_nodes[b] + i];
      if (p >= i || p < -1) { free(node_seq); return -3; }
      node_seq[cu_nodes[b] + i] = b;
    }
    if (prefix_len[b] + n_b > max_keys) max_keys = prefix_len[b] + n_b;
  }

  const int64_t n_work = n_sel >= 0 ? n_sel : (int64_t)total_nodes * Hq;
  int failed = 0;

#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)(max_keys + 1));
    /* tree keys, as global node indices, for the current query */
    int32_t* anc = (int32_t*)malloc(sizeof(int32_t) * (size_t)(total_nodes + 1));
    double* acc = (double*)malloc(sizeof(double) * (size_t)D);
    if (!s || !anc || !acc) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp barrier
    if (!failed) {
#pragma omp for schedule(dynamic, 1)
      for (int64_t w = 0; w < n_work; ++w) {
        int node, h;
        if (n_sel >= 0) { node = sel_node[w]; h = sel_head[w]; }
        else            { node = (int)(w / Hq); h = (int)(w % Hq); }
        const int b = node_seq[node];
        const int g = h / G;
        const int len = prefix_len[b];
        const int base = cu_nodes[b];

        /* ancestor-or-self set by walking the parent array */
        int n_anc = 0;
        for (int j = node - base; j >= 0; j = parent[base + j]) anc[n_anc++] = base + j;

        const int64_t q_off = ((int64_t)node * Hq + h) * D;
        int nk = 0;
        /* scores against the cached prefix */
        for (int t = 0; t < len; ++t) {
          const int64_t blk = block_table[(int64_t)b * max_blocks_per_seq + t / block_size];
          const int64_t k_off = blk * block_stride + (int64_t)g * head_stride +
                                (int64_t)(t % block_size) * token_stride;
          double dot = 0.0;
          for (int d = 0; d < D; ++d)
            dot += load_elem(q, dtype, q_off + d) * load_elem(k_cache, dtype, k_off + d);
          s[nk++] = scale * dot;
        }
        /* scores against the node itself and its ancestors */
        for (int a = 0; a < n_anc; ++a) {
          const int64_t k_off = ((int64_t)anc[a] * Hkv + g) * D;
          double dot = 0.0;
          for (int d = 0; d < D; ++d)
            dot += load_elem(q, dtype, q_off + d) * load_elem(k_tree, dtype, k_off + d);
          s[nk++] = scale * dot;
        }
        double m = s[0];
        for (int x = 1; x < nk; ++x) if (s[x] > m) m = s[x];
        double denom = 0.0;
        for (int x = 0; x < nk; ++x) { s[x] = exp(s[x] - m); denom += s[x]; }

        for (int d = 0; d < D; ++d) acc[d] = 0.0;
        for (int t = 0; t < len; ++t) {
          const int64_t blk = block_table[(int64_t)b * max_blocks_per_seq + t / block_size];
          const int64_t v_off = blk * block_stride + (int64_t)g * head_stride +
                                (int64_t)(t % block_size) * token_stride;
          const double p = s[t] / denom;
          for (int d = 0; d < D; ++d) acc[d] += p * load_elem(v_cache, dtype, v_off + d);
        }
        for (int a = 0; a < n_anc; ++a) {
          const int64_t v_off = ((int64_t)anc[a] * Hkv + g) * D;
          const double p = s[len + a] / denom;
          for (int d = 0; d < D; ++d) acc[d] += p * load_elem(v_tree, dtype, v_off + d);
        }
        double* o = out + (n_sel >= 0 ? w * D : ((int64_t)node * Hq + h) * D);
        for (int d = 0; d < D; ++d) o[d] = acc[d];
        if (lse) lse[n_sel >= 0 ? w : (int64_t)node * Hq + h] = m + log(denom);
      }
    }
    free(s); free(anc); free(acc);
  }
  free(node_seq);
  return failed ? -2 : 0;
}
