/*
 * Test hooks of libkge_mi355: entry points that exist so that the GPU tests can look inside a call.
 * They are not part of the boundary of the training step or of the evaluation (include/kge_mi355.h);
 * a product has no reason to call them.
 */
#ifndef KGE_MI355_TESTING_H
#define KGE_MI355_TESTING_H

#include "kge_mi355.h"

#ifdef __cplusplus
extern "C" {
#endif

/* The fp32 scores that kge_eval_rank_all compares (Eq. 4 for every query against every entity), written
 * out: scores DEVICE float [2 n_test][n_entities] from the tile kernel, answer_score DEVICE float
 * [2 n_test] from the per-query kernel (the two kernels must agree bit for bit on the same pair).
 * Arguments as kge_eval_rank_all; workspace of kge_eval_workspace_bytes(2 n_test, d) bytes.  Small inputs
 * only (the score matrix is materialised).  Returns a status code like every other call. */
int kge_eval_debug_scores(const float *H, int64_t n_entities, int32_t d, const float *M, int32_t n_relations,
                          const int32_t *test_h, const int32_t *test_r, const int32_t *test_t, int64_t n_test,
                          void *workspace, size_t ws_bytes, float *scores, float *answer_score, void *stream);

/* Partitions built after this call order the run ranges of the transposed per-run products by slabs of
 * `vertices` destinations and cut a relation's runs at slab borders once it has `min_runs` runs or more (the
 * library's own values: 262,144 vertices, two full ranges of runs; <= 0 restores them).  It lets a small graph
 * take the code path that otherwise only a partition of more than 262,144 vertices takes.  Process-wide, not
 * thread-safe. */
void kge_test_set_rel_slab(int32_t vertices, int32_t min_runs);

#ifdef __cplusplus
}
#endif
#endif /* KGE_MI355_TESTING_H */
