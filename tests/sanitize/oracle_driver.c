/* Runs the C attention oracle on a small seeded problem (both element types, full output and selected rows,
 * a malformed tree) for a build with -fsanitize=address,undefined.  Values are checked elsewhere. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int tree_attention_ref(int dtype, int batch, int num_q_heads, int num_kv_heads, int head_dim, int block_size,
                       double scale, const void* q, const void* k_tree, const void* v_tree, const void* k_cache,
                       const void* v_cache, int64_t block_stride, int64_t head_stride, int64_t token_stride,
                       const int32_t* block_table, int max_blocks_per_seq, const int32_t* prefix_len,
                       const int32_t* cu_nodes, const int32_t* parent, int64_t n_sel, const int32_t* sel_node,
                       const int32_t* sel_head, double* out, double* lse);

static uint32_t state = 12345u;
static float unit(void) {
  state = state * 1664525u + 1013904223u;
  return (float)((state >> 8) & 0xFFFF) / 65536.0f - 0.5f;
}

int main(void) {
  enum { B = 3, Hq = 4, Hkv = 2, D = 16, BS = 8, MAXB = 5, NB = B * MAXB };
  const int32_t cu[B + 1] = {0, 1, 6, 9};
  int32_t parent[9] = {-1, -1, 0, 0, 1, 2, -1, 0, 0};
  const int32_t len[B] = {0, 17, 40};
  const int N = 9;
  int32_t table[B * MAXB];
  for (int i = 0; i < B * MAXB; ++i) table[i] = (i * 7) % NB;
  int failures = 0;
  for (int dtype = 0; dtype < 2; ++dtype) {
    const size_t es = dtype == 0 ? 4 : 2;
    const size_t nq = (size_t)N * Hq * D, nk = (size_t)N * Hkv * D, nc = (size_t)NB * Hkv * BS * D;
    unsigned char *q = malloc(nq * es), *k = malloc(nk * es), *v = malloc(nk * es), *kc = malloc(nc * es), *vc = malloc(nc * es);
    unsigned char* bufs[5] = {q, k, v, kc, vc};
    const size_t sizes[5] = {nq, nk, nk, nc, nc};
    for (int a = 0; a < 5; ++a)
      for (size_t i = 0; i < sizes[a]; ++i) {
        float f = unit();
        if (dtype == 0) memcpy(bufs[a] + 4 * i, &f, 4);
        else {
          uint32_t bits;
          memcpy(&bits, &f, 4);
          uint16_t h = (uint16_t)(bits >> 16);
          memcpy(bufs[a] + 2 * i, &h, 2);
        }
      }
    double* out = malloc(sizeof(double) * nq);
    double* lse = malloc(sizeof(double) * (size_t)N * Hq);
    int rc = tree_attention_ref(dtype, B, Hq, Hkv, D, BS, 0.25, q, k, v, kc, vc, (int64_t)Hkv * BS * D, (int64_t)BS * D, D,
                                table, MAXB, len, cu, parent, -1, NULL, NULL, out, lse);
    if (rc != 0) ++failures;
    for (size_t i = 0; i < nq; ++i)
      if (!isfinite(out[i])) ++failures;
    const int32_t sel_node[4] = {0, 5, 8, 3}, sel_head[4] = {0, 3, 1, 2};
    rc = tree_attention_ref(dtype, B, Hq, Hkv, D, BS, 0.25, q, k, v, kc, vc, (int64_t)Hkv * BS * D, (int64_t)BS * D, D, table,
                            MAXB, len, cu, parent, 4, sel_node, sel_head, out, lse);
    if (rc != 0) ++failures;
    parent[4] = 7; /* a parent that does not precede its child: rejected, nothing written */
    rc = tree_attention_ref(dtype, B, Hq, Hkv, D, BS, 0.25, q, k, v, kc, vc, (int64_t)Hkv * BS * D, (int64_t)BS * D, D, table,
                            MAXB, len, cu, parent, -1, NULL, NULL, out, lse);
    if (rc == 0) ++failures;
    parent[4] = 1;
    free(q); free(k); free(v); free(kc); free(vc); free(out); free(lse);
  }
  if (failures) {
    fprintf(stderr, "%d check(s) failed\n", failures);
    return 1;
  }
  puts("oracle driver ok");
  return 0;
}
