/*
 * CPU ORACLE — TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded, double-precision implementation of one
 * training step of the partitioned RGCN + DistMult trainer of
 * "Scaling Knowledge Graph Embedding Models" (arXiv 2201.02791), written from
 * the paper's definitions.  It shares no code with the GPU library; only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 * The product path never does.
 *
 * What follows which passage:
 *   - message edges, partition, n-hop Neighborhood Expansion  Sec. 3.2.1, 3.2.2
 *   - RGCN layer with basis decomposition                     Eq. 1, Eq. 2
 *   - constraint-based (in-partition) negative sampling       Sec. 2.1, Sec. 3.3.1
 *   - DistMult score and cross-entropy loss                   Eq. 4, Eq. 3
 *   - backward pass: chain rule applied to Eq. 1-4
 *
 * Pin status (see tests/test_oracle_*.py): every function below is pinned by
 * something other than itself — brute force with W_r materialised, the
 * one-basis mean-aggregation special case with hand-computed values, GEMM
 * special cases, central finite differences, the self-sufficiency invariant
 * of expanded partitions, ln 2 loss at zero embeddings, and an independent
 * library Philox4x32-10 engine for the counter-based generator.
 *
 * Conventions: row vectors (h is 1 x d, V_b is d_in x d_out, out = h V);
 * relation ids 0..R-1 are the given direction, R..2R-1 the inverses; the
 * self-loop is the dense W_0 term and is not an edge.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Partitioning (Sec. 3.2.1) and Neighborhood Expansion (Sec. 3.2.2)   */
/* ------------------------------------------------------------------ */

typedef struct orc_partition {
    int64_t n_vert, n_edge, n_seg, n_core, n_cand;
    int32_t *vert_gid;   /* [n_vert] global id of local vertex, ascending            */
    int32_t *core_eid;   /* [n_core] indices of this partition's core triples         */
    int32_t *core_h, *core_r, *core_t; /* [n_core] local head, relation, local tail   */
    int32_t *seg_ptr;    /* [n_seg+1] edge range of each (relation, destination) run  */
    int32_t *seg_rel;    /* [n_seg]                                                   */
    int32_t *seg_dst;    /* [n_seg] local destination                                 */
    float   *inv_c;      /* [n_seg] 1 / c_{i,r} = 1 / run length, rounded to float    */
    int32_t *col_src;    /* [n_edge] local source, in sorted order                    */
    int32_t *edge_id;    /* [n_edge] message-edge id: triple i -> i, its inverse M+i  */
    int32_t *cand;       /* [n_cand] local ids negatives may be drawn from            */
} orc_partition;

/* The vertex-cut of the paper is replaced by a hash of the head entity: the
 * core edge sets stay disjoint and cover every triple, which is the property
 * Sec. 3.2.1 needs.  part = ((uint32 head * 0x9E3779B1) >> 8) mod P. */
uint32_t orc_part_of_head(int32_t head, int32_t n_parts)
{
    uint32_t h = (uint32_t)head * 0x9E3779B1u;
    return (h >> 8) % (uint32_t)n_parts;
}

typedef struct { int32_t rel, dst, src, id; } orc_medge;

static int cmp_medge(const void *pa, const void *pb)
{
    const orc_medge *a = (const orc_medge *)pa, *b = (const orc_medge *)pb;
    if (a->rel != b->rel) return a->rel < b->rel ? -1 : 1;
    if (a->dst != b->dst) return a->dst < b->dst ? -1 : 1;
    if (a->src != b->src) return a->src < b->src ? -1 : 1;
    if (a->id  != b->id)  return a->id  < b->id  ? -1 : 1;
    return 0;
}

void orc_partition_free(orc_partition *p)
{
    if (!p) return;
    free(p->vert_gid); free(p->core_eid); free(p->core_h); free(p->core_r); free(p->core_t);
    free(p->seg_ptr); free(p->seg_rel); free(p->seg_dst); free(p->inv_c);
    free(p->col_src); free(p->edge_id); free(p->cand); free(p);
}

/*
 * Build partition `part_id` of `n_parts`.
 *  1. core edges: triples whose head hashes to this partition (they are the
 *     positives, Sec. 3.2.1).  S_0 = their endpoints.
 *  2. expansion: S_k = S_{k-1} united with the sources of all message edges
 *     whose destination is in S_{k-1}, k = 1..n_hops (Sec. 3.2.2).  A triple
 *     (s,r,t) carries two message edges: s->t under r and t->s under r+R.
 *  3. the partition keeps the vertices S_L and every message edge whose
 *     destination lies in S_{L-1} (the edges message passing needs).
 *  4. edges sorted by (relation, destination, source, message-edge id);
 *     a maximal run of equal (relation, destination) is the neighbour set
 *     N_i^r and c_{i,r} its length, counted with multiplicity.
 *  5. negative candidates: neg_domain 0 = endpoints of core edges (S_0),
 *     neg_domain 1 = every vertex of the partition.
 */
orc_partition *orc_build_partition(const int32_t *head, const int32_t *rel, const int32_t *tail,
                                   int64_t n_triples, int32_t n_entities, int32_t n_relations,
                                   int32_t n_parts, int32_t part_id, int32_t n_hops,
                                   int32_t neg_domain)
{
    orc_partition *p = (orc_partition *)calloc(1, sizeof *p);
    int64_t M = n_triples, i;
    uint8_t *s0 = (uint8_t *)calloc((size_t)n_entities + 1, 1);
    uint8_t *prev = (uint8_t *)calloc((size_t)n_entities + 1, 1);
    uint8_t *cur = (uint8_t *)calloc((size_t)n_entities + 1, 1);
    uint8_t *dstset = (uint8_t *)calloc((size_t)n_entities + 1, 1); /* S_{L-1} */
    int32_t *lid = (int32_t *)malloc(sizeof(int32_t) * ((size_t)n_entities + 1));
    int64_t n_core = 0;

    for (i = 0; i < M; ++i)
        if (orc_part_of_head(head[i], n_parts) == (uint32_t)part_id) {
            ++n_core; s0[head[i]] = 1; s0[tail[i]] = 1;
        }
    memcpy(cur, s0, (size_t)n_entities);
    for (int k = 1; k <= n_hops; ++k) {
        memcpy(prev, cur, (size_t)n_entities);
        for (i = 0; i < M; ++i) {
            if (prev[tail[i]]) cur[head[i]] = 1;   /* s->t : source s joins */
            if (prev[head[i]]) cur[tail[i]] = 1;   /* t->s : source t joins */
        }
    }
    if (n_hops >= 1) memcpy(dstset, prev, (size_t)n_entities);

    int64_t N = 0;
    for (i = 0; i < n_entities; ++i) { lid[i] = cur[i] ? (int32_t)N : -1; N += cur[i]; }
    p->n_vert = N;
    p->vert_gid = (int32_t *)malloc(sizeof(int32_t) * (size_t)(N + 1));
    for (i = 0; i < n_entities; ++i) if (cur[i]) p->vert_gid[lid[i]] = (int32_t)i;

    p->n_core = n_core;
    p->core_eid = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_core + 1));
    p->core_h = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_core + 1));
    p->core_r = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_core + 1));
    p->core_t = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_core + 1));
    n_core = 0;
    for (i = 0; i < M; ++i)
        if (orc_part_of_head(head[i], n_parts) == (uint32_t)part_id) {
            p->core_eid[n_core] = (int32_t)i;
            p->core_h[n_core] = lid[head[i]];
            p->core_r[n_core] = rel[i];
            p->core_t[n_core] = lid[tail[i]];
            ++n_core;
        }

    int64_t E = 0;
    for (i = 0; i < M; ++i) { E += dstset[tail[i]]; E += dstset[head[i]]; }
    orc_medge *me = (orc_medge *)malloc(sizeof(orc_medge) * (size_t)(E + 1));
    E = 0;
    for (i = 0; i < M; ++i) if (dstset[tail[i]]) {
        me[E].rel = rel[i]; me[E].dst = lid[tail[i]]; me[E].src = lid[head[i]]; me[E].id = (int32_t)i; ++E;
    }
    for (i = 0; i < M; ++i) if (dstset[head[i]]) {
        me[E].rel = rel[i] + n_relations; me[E].dst = lid[head[i]]; me[E].src = lid[tail[i]];
        me[E].id = (int32_t)(M + i); ++E;
    }
    qsort(me, (size_t)E, sizeof(orc_medge), cmp_medge);
    p->n_edge = E;
    p->col_src = (int32_t *)malloc(sizeof(int32_t) * (size_t)(E + 1));
    p->edge_id = (int32_t *)malloc(sizeof(int32_t) * (size_t)(E + 1));
    int64_t S = 0;
    for (i = 0; i < E; ++i) {
        p->col_src[i] = me[i].src; p->edge_id[i] = me[i].id;
        if (i == 0 || me[i].rel != me[i - 1].rel || me[i].dst != me[i - 1].dst) ++S;
    }
    p->n_seg = S;
    p->seg_ptr = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S + 2));
    p->seg_rel = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S + 1));
    p->seg_dst = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S + 1));
    p->inv_c = (float *)malloc(sizeof(float) * (size_t)(S + 1));
    S = 0;
    for (i = 0; i < E; ++i)
        if (i == 0 || me[i].rel != me[i - 1].rel || me[i].dst != me[i - 1].dst) {
            p->seg_ptr[S] = (int32_t)i; p->seg_rel[S] = me[i].rel; p->seg_dst[S] = me[i].dst; ++S;
        }
    p->seg_ptr[S] = (int32_t)E;
    for (i = 0; i < S; ++i) p->inv_c[i] = 1.0f / (float)(p->seg_ptr[i + 1] - p->seg_ptr[i]);

    int64_t nc = 0;
    p->cand = (int32_t *)malloc(sizeof(int32_t) * (size_t)(N + 1));
    for (i = 0; i < n_entities; ++i)
        if (cur[i] && (neg_domain == 1 || s0[i])) p->cand[nc++] = lid[i];
    p->n_cand = nc;

    free(me); free(s0); free(prev); free(cur); free(dstset); free(lid);
    return p;
}

void orc_partition_sizes(const orc_partition *p, int64_t out[5])
{
    out[0] = p->n_vert; out[1] = p->n_edge; out[2] = p->n_seg; out[3] = p->n_core; out[4] = p->n_cand;
}

/* which: 0 vert_gid, 1 core_eid, 2 core_h, 3 core_r, 4 core_t, 5 seg_ptr, 6 seg_rel,
 * 7 seg_dst, 8 inv_c, 9 col_src, 10 edge_id, 11 cand.  Copies the array out. */
void orc_partition_copy(const orc_partition *p, int32_t which, void *dst)
{
    const void *src = 0; size_t n = 0;
    switch (which) {
    case 0: src = p->vert_gid; n = (size_t)p->n_vert; break;
    case 1: src = p->core_eid; n = (size_t)p->n_core; break;
    case 2: src = p->core_h; n = (size_t)p->n_core; break;
    case 3: src = p->core_r; n = (size_t)p->n_core; break;
    case 4: src = p->core_t; n = (size_t)p->n_core; break;
    case 5: src = p->seg_ptr; n = (size_t)p->n_seg + 1; break;
    case 6: src = p->seg_rel; n = (size_t)p->n_seg; break;
    case 7: src = p->seg_dst; n = (size_t)p->n_seg; break;
    case 8: src = p->inv_c; n = (size_t)p->n_seg; break;
    case 9: src = p->col_src; n = (size_t)p->n_edge; break;
    case 10: src = p->edge_id; n = (size_t)p->n_edge; break;
    case 11: src = p->cand; n = (size_t)p->n_cand; break;
    default: return;
    }
    memcpy(dst, src, n * 4);
}

/* ------------------------------------------------------------------ */
/* RGCN layer (Eq. 1 with the basis decomposition of Eq. 2)            */
/* ------------------------------------------------------------------ */

static double act_fwd(int act, double x) { return act == 1 ? (x > 0.0 ? x : 0.0) : x; }
static double act_grad(int act, double pre) { return act == 1 ? (pre > 0.0 ? 1.0 : 0.0) : 1.0; }

/* P[j][b][:] = h_j V_b  — the B projections of every vertex (Eq. 2 applied to h_j). */
static void project_all(int64_t N, int32_t d_in, int32_t d_out, int32_t B,
                        const double *V, const double *H, double *P)
{
    memset(P, 0, sizeof(double) * (size_t)N * (size_t)B * (size_t)d_out);
    for (int64_t j = 0; j < N; ++j)
        for (int32_t b = 0; b < B; ++b) {
            double *out = P + ((size_t)j * B + b) * d_out;
            const double *Vb = V + (size_t)b * d_in * d_out;
            for (int32_t k = 0; k < d_in; ++k) {
                double h = H[(size_t)j * d_in + k];
                const double *vrow = Vb + (size_t)k * d_out;
                for (int32_t o = 0; o < d_out; ++o) out[o] += h * vrow[o];
            }
        }
}

/*
 * One layer forward over the whole partition:
 *   pre_i = sum_r sum_{j in N_i^r} (1/c_{i,r}) h_j W_r + h_i W_0,   W_r = sum_b a_rb V_b
 *   h'_i  = act(pre_i)                        act: 0 identity, 1 ReLU
 * P_scratch is [N][B][d_out] doubles.  Everything is exact double arithmetic: workloads that keep
 * messages in bf16 are compared with these values under their wider tolerance.
 */
void orc_rgcn_layer_forward(int64_t N, int64_t S, const int32_t *seg_ptr, const int32_t *seg_rel,
                            const int32_t *seg_dst, const int32_t *col_src,
                            int32_t d_in, int32_t d_out, int32_t B,
                            const double *V, const double *a, const double *W0, int32_t act,
                            const double *H, double *P_scratch, double *pre, double *Hout)
{
    project_all(N, d_in, d_out, B, V, H, P_scratch);
    /* self-loop: h_i W_0 */
    for (int64_t i = 0; i < N; ++i) {
        double *o = pre + (size_t)i * d_out;
        for (int32_t c = 0; c < d_out; ++c) o[c] = 0.0;
        for (int32_t k = 0; k < d_in; ++k) {
            double h = H[(size_t)i * d_in + k];
            const double *w = W0 + (size_t)k * d_out;
            for (int32_t c = 0; c < d_out; ++c) o[c] += h * w[c];
        }
    }
    /* neighbours, one (relation, destination) run at a time */
    for (int64_t s = 0; s < S; ++s) {
        int32_t r = seg_rel[s], i = seg_dst[s];
        double invc = 1.0 / (double)(seg_ptr[s + 1] - seg_ptr[s]);
        double *o = pre + (size_t)i * d_out;
        for (int32_t e = seg_ptr[s]; e < seg_ptr[s + 1]; ++e) {
            int32_t j = col_src[e];
            for (int32_t b = 0; b < B; ++b) {
                double w = a[(size_t)r * B + b] * invc;
                const double *pj = P_scratch + ((size_t)j * B + b) * d_out;
                for (int32_t c = 0; c < d_out; ++c) o[c] += w * pj[c];
            }
        }
    }
    for (size_t q = 0; q < (size_t)N * d_out; ++q) Hout[q] = act_fwd(act, pre[q]);
}

/*
 * The same layer, only for the listed destination rows (used where the whole
 * partition is too large for the oracle).  For row q (local vertex rows[q])
 * its runs are row_seg[row_seg_ptr[q] .. row_seg_ptr[q+1]).  Nothing is
 * precomputed: each neighbour is projected on the spot.
 */
void orc_rgcn_layer_rows(int64_t n_rows, const int32_t *rows, const int64_t *row_seg_ptr,
                         const int64_t *row_seg, const int32_t *seg_ptr, const int32_t *seg_rel,
                         const int32_t *col_src, int32_t d_in, int32_t d_out, int32_t B,
                         const double *V, const double *a, const double *W0, int32_t act,
                         const float *H /* [N][d_in], the layer input as stored */,
                         double *pre_rows, double *out_rows)
{
    double *pj = (double *)malloc(sizeof(double) * (size_t)d_out);
    for (int64_t q = 0; q < n_rows; ++q) {
        int32_t i = rows[q];
        double *o = pre_rows + (size_t)q * d_out;
        for (int32_t c = 0; c < d_out; ++c) o[c] = 0.0;
        for (int32_t k = 0; k < d_in; ++k) {
            double h = (double)H[(size_t)i * d_in + k];
            for (int32_t c = 0; c < d_out; ++c) o[c] += h * W0[(size_t)k * d_out + c];
        }
        for (int64_t t = row_seg_ptr[q]; t < row_seg_ptr[q + 1]; ++t) {
            int64_t s = row_seg[t];
            int32_t r = seg_rel[s];
            double invc = 1.0 / (double)(seg_ptr[s + 1] - seg_ptr[s]);
            for (int32_t e = seg_ptr[s]; e < seg_ptr[s + 1]; ++e) {
                int32_t j = col_src[e];
                for (int32_t b = 0; b < B; ++b) {
                    const double *Vb = V + (size_t)b * d_in * d_out;
                    for (int32_t c = 0; c < d_out; ++c) pj[c] = 0.0;
                    for (int32_t k = 0; k < d_in; ++k) {
                        double h = (double)H[(size_t)j * d_in + k];
                        for (int32_t c = 0; c < d_out; ++c) pj[c] += h * Vb[(size_t)k * d_out + c];
                    }
                    double w = a[(size_t)r * B + b] * invc;
                    for (int32_t c = 0; c < d_out; ++c) o[c] += w * pj[c];
                }
            }
        }
        for (int32_t c = 0; c < d_out; ++c) out_rows[(size_t)q * d_out + c] = act_fwd(act, o[c]);
    }
    free(pj);
}

/*
 * One layer backward (chain rule on Eq. 1-2).  With G = dL/dh' (dHout):
 *   Gpre = G * act'(pre)
 *   dW0 = H^T Gpre,                 dH_i  += Gpre_i W0^T
 *   for every edge j -> i under r, with w = 1/c_{i,r}:
 *       da_rb       += w <h_j V_b, Gpre_i>
 *       dP[j][b][:] += a_rb w Gpre_i
 *   dV_b = H^T dP_b,                dH_j  += sum_b dP[j][b][:] V_b^T
 * P_scratch and dP_scratch are [N][B][d_out]; dH_in may be NULL.
 */
void orc_rgcn_layer_backward(int64_t N, int64_t S, const int32_t *seg_ptr, const int32_t *seg_rel,
                             const int32_t *seg_dst, const int32_t *col_src,
                             int32_t d_in, int32_t d_out, int32_t B, int32_t n_rel2,
                             const double *V, const double *a, const double *W0, int32_t act,
                             const double *H, const double *pre, const double *dHout,
                             double *P_scratch, double *dP_scratch, double *Gpre,
                             double *dV, double *da, double *dW0, double *dH_in)
{
    size_t nd_out = (size_t)N * d_out;
    for (size_t q = 0; q < nd_out; ++q) Gpre[q] = dHout[q] * act_grad(act, pre[q]);
    project_all(N, d_in, d_out, B, V, H, P_scratch);
    memset(dP_scratch, 0, sizeof(double) * (size_t)N * B * d_out);
    memset(dV, 0, sizeof(double) * (size_t)B * d_in * d_out);
    memset(da, 0, sizeof(double) * (size_t)n_rel2 * B);
    memset(dW0, 0, sizeof(double) * (size_t)d_in * d_out);
    if (dH_in) memset(dH_in, 0, sizeof(double) * (size_t)N * d_in);

    for (int64_t i = 0; i < N; ++i) {
        const double *g = Gpre + (size_t)i * d_out;
        for (int32_t k = 0; k < d_in; ++k) {
            double h = H[(size_t)i * d_in + k];
            double acc = 0.0;
            for (int32_t c = 0; c < d_out; ++c) {
                dW0[(size_t)k * d_out + c] += h * g[c];
                acc += g[c] * W0[(size_t)k * d_out + c];
            }
            if (dH_in) dH_in[(size_t)i * d_in + k] += acc;
        }
    }
    for (int64_t s = 0; s < S; ++s) {
        int32_t r = seg_rel[s], i = seg_dst[s];
        double invc = 1.0 / (double)(seg_ptr[s + 1] - seg_ptr[s]);
        const double *g = Gpre + (size_t)i * d_out;
        for (int32_t e = seg_ptr[s]; e < seg_ptr[s + 1]; ++e) {
            int32_t j = col_src[e];
            for (int32_t b = 0; b < B; ++b) {
                const double *pj = P_scratch + ((size_t)j * B + b) * d_out;
                double *dpj = dP_scratch + ((size_t)j * B + b) * d_out;
                double dot = 0.0, w = a[(size_t)r * B + b] * invc;
                for (int32_t c = 0; c < d_out; ++c) { dot += pj[c] * g[c]; dpj[c] += w * g[c]; }
                da[(size_t)r * B + b] += invc * dot;
            }
        }
    }
    for (int64_t j = 0; j < N; ++j)
        for (int32_t b = 0; b < B; ++b) {
            const double *dpj = dP_scratch + ((size_t)j * B + b) * d_out;
            const double *Vb = V + (size_t)b * d_in * d_out;
            double *dVb = dV + (size_t)b * d_in * d_out;
            for (int32_t k = 0; k < d_in; ++k) {
                double h = H[(size_t)j * d_in + k], acc = 0.0;
                for (int32_t c = 0; c < d_out; ++c) {
                    dVb[(size_t)k * d_out + c] += h * dpj[c];
                    acc += dpj[c] * Vb[(size_t)k * d_out + c];
                }
                if (dH_in) dH_in[(size_t)j * d_in + k] += acc;
            }
        }
}

/* ------------------------------------------------------------------ */
/* Counter-based negative sampling (Sec. 2.1 corruption, Sec. 3.3.1)   */
/* ------------------------------------------------------------------ */

/* Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).  One round
 * multiplies counter words 0 and 2 by two fixed odd constants, keeps the low
 * halves, and xors the high halves with the other two words and the round
 * key; the key advances by two Weyl constants between rounds. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * For positive p (index into the partition's core-edge list) and slot k:
 *   x = Philox4x32-10(counter = (p, k, step lo, step hi), key = (seed lo, seed hi))
 *   corrupting entity = cand[(x0 * n_cand) >> 32]      (always inside the partition)
 *   mode 0: the tail is replaced; mode 1: the head if x1 >= 2^31, else the tail.
 * No filtering and no rejection: an accidental true triple is labelled negative.
 * neg_side: 0 tail replaced, 1 head replaced.
 */
void orc_sample_negatives(const int32_t *cand, int64_t n_cand, const int32_t *pos_core_idx,
                          int64_t n_pos, int32_t n_neg, int32_t mode, uint64_t seed, uint64_t step,
                          int32_t *neg_ent, uint8_t *neg_side)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    for (int64_t p = 0; p < n_pos; ++p)
        for (int32_t k = 0; k < n_neg; ++k) {
            uint32_t ctr[4] = { (uint32_t)pos_core_idx[p], (uint32_t)k, (uint32_t)step,
                                (uint32_t)(step >> 32) };
            uint32_t x[4];
            orc_philox4x32_10(ctr, key, x);
            uint64_t idx = ((uint64_t)x[0] * (uint64_t)n_cand) >> 32;
            neg_ent[p * n_neg + k] = cand[idx];
            neg_side[p * n_neg + k] = (uint8_t)((mode == 1 && x[1] >= 0x80000000u) ? 1 : 0);
        }
}

/* ------------------------------------------------------------------ */
/* DistMult score (Eq. 4) and cross-entropy loss (Eq. 3)               */
/* ------------------------------------------------------------------ */

static double softplus(double x) { return x > 0.0 ? x + log1p(exp(-x)) : log1p(exp(x)); }
static double sigmoid(double x) { return x >= 0.0 ? 1.0 / (1.0 + exp(-x)) : exp(x) / (1.0 + exp(x)); }

/*
 * Scored triples are positive-major: row p = [positive, negative 0 .. n_neg-1].
 *   g(s,r,t) = sum_k h_s[k] M_r[k] h_t[k]
 *   L = -(1/|T|) sum_T [ y log l(g) + (1-y) log(1 - l(g)) ],  l = logistic sigmoid
 *     (Eq. 3 is minimised, so it carries the leading minus the print lost)
 *   delta = dL/dg = (l(g) - y)/|T|
 *   dH_s += delta M_r*h_t,  dH_t += delta M_r*h_s,  dM_r += delta h_s*h_t
 * scores [n_pos][1+n_neg], dH [N][d], dM [R][d] are overwritten.
 */
void orc_distmult_score_loss(int64_t N, int32_t d, int32_t n_rel, const double *H, const double *M,
                             int64_t n_pos, int32_t n_neg, const int32_t *pos_h, const int32_t *pos_r,
                             const int32_t *pos_t, const int32_t *neg_ent, const uint8_t *neg_side,
                             double *scores, double *loss, double *dH, double *dM)
{
    int64_t T = n_pos * (1 + (int64_t)n_neg);
    double total = 0.0;
    memset(dH, 0, sizeof(double) * (size_t)N * d);
    memset(dM, 0, sizeof(double) * (size_t)n_rel * d);
    for (int64_t p = 0; p < n_pos; ++p)
        for (int32_t k = 0; k <= n_neg; ++k) {
            int32_t s = pos_h[p], r = pos_r[p], t = pos_t[p];
            double y = 1.0;
            if (k > 0) {
                int64_t q = p * n_neg + (k - 1);
                y = 0.0;
                if (neg_side[q]) s = neg_ent[q]; else t = neg_ent[q];
            }
            const double *hs = H + (size_t)s * d, *ht = H + (size_t)t * d, *mr = M + (size_t)r * d;
            double g = 0.0;
            for (int32_t c = 0; c < d; ++c) g += hs[c] * mr[c] * ht[c];
            scores[p * (1 + n_neg) + k] = g;
            total += (y > 0.5) ? softplus(-g) : softplus(g);
            double delta = (sigmoid(g) - y) / (double)T;
            double *ds = dH + (size_t)s * d, *dt = dH + (size_t)t * d, *dm = dM + (size_t)r * d;
            for (int32_t c = 0; c < d; ++c) {
                double hsc = hs[c], htc = ht[c];
                ds[c] += delta * mr[c] * htc;
                dt[c] += delta * mr[c] * hsc;
                dm[c] += delta * hsc * htc;
            }
        }
    *loss = T > 0 ? total / (double)T : 0.0;
}

/* ------------------------------------------------------------------ */
/* Computational sub-graph of one edge batch (Sec. 3.3, Algorithm 1)   */
/* ------------------------------------------------------------------ */
/*
 * The embeddings of a batch's vertices after layer L depend only on the vertices within L hops
 * along incoming message edges.  active[l][i] = 1 if layer l+1 (l = 0 .. L-1) has to produce an
 * output row for vertex i:
 *   active[L-1] = the batch's vertices (heads and tails of the positives, corrupting entities),
 *   active[l-1] = active[l]  united with  the sources of every message edge whose destination is
 *                 in active[l]   (a vertex also needs its own previous row: the self-loop).
 * `active` is [n_layers][N], overwritten.
 */
void orc_compute_graph(int64_t N, int64_t S, const int32_t *seg_ptr, const int32_t *seg_dst,
                       const int32_t *col_src, int64_t n_batch, const int32_t *batch_vertices,
                       int32_t n_layers, uint8_t *active)
{
    memset(active, 0, (size_t)n_layers * (size_t)N);
    if (n_layers <= 0) return;
    uint8_t *top = active + (size_t)(n_layers - 1) * N;
    for (int64_t k = 0; k < n_batch; ++k) top[batch_vertices[k]] = 1;
    for (int32_t l = n_layers - 1; l >= 1; --l) {
        const uint8_t *cur = active + (size_t)l * N;
        uint8_t *below = active + (size_t)(l - 1) * N;
        for (int64_t i = 0; i < N; ++i) if (cur[i]) below[i] = 1;
        for (int64_t s = 0; s < S; ++s)
            if (cur[seg_dst[s]])
                for (int32_t e = seg_ptr[s]; e < seg_ptr[s + 1]; ++e) below[col_src[e]] = 1;
    }
}

/* ------------------------------------------------------------------ */
/* Optimizer step (Algorithm 1, "optimizer.step()")                    */
/* ------------------------------------------------------------------ */
/*
 * The paper trains with synchronous gradient descent at learning rate 0.01 and does not name the
 * update rule; two are provided.
 *   kind 0, plain gradient descent:  p <- p - lr g
 *   kind 1, Adam (Kingma & Ba 2015), t = 1, 2, ... the number of this step:
 *       m <- b1 m + (1 - b1) g,   v <- b2 v + (1 - b2) g^2
 *       p <- p - lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
 * Row form: the tensor is [n_rows][d] and only rows with row_mask[i] != 0 are touched (an embedding
 * table of which a step reaches few rows; moments of the other rows stay as they are, and the bias
 * correction still uses the global t).  row_mask NULL = every row.
 */
void orc_optimizer_step(int32_t kind, double *p, const double *g, double *m, double *v, int64_t n_rows,
                        int64_t d, const uint8_t *row_mask, double lr, double b1, double b2, double eps,
                        int64_t t)
{
    double c1 = 1.0 - pow(b1, (double)t), c2 = 1.0 - pow(b2, (double)t);
    for (int64_t i = 0; i < n_rows; ++i) {
        if (row_mask && !row_mask[i]) continue;
        for (int64_t k = 0; k < d; ++k) {
            size_t q = (size_t)i * d + k;
            if (kind == 0) { p[q] -= lr * g[q]; continue; }
            m[q] = b1 * m[q] + (1.0 - b1) * g[q];
            v[q] = b2 * v[q] + (1.0 - b2) * g[q] * g[q];
            p[q] -= lr * (m[q] / c1) / (sqrt(v[q] / c2) + eps);
        }
    }
}

/* ------------------------------------------------------------------ */
/* Dropout on a layer's input                                          */
/* ------------------------------------------------------------------ */
/*
 * The paper's large-graph setting uses dropout 0.2 and does not say where; it is applied here to the
 * features a layer reads (neighbour messages and self-loop alike), in the usual inverted form:
 *   out[i][k] = keep ? H[i][k] / (1 - p) : 0
 * The decision for element (i, k) of layer `layer` at training step `step` is counter-based, like the
 * negative sampler:  x = Philox4x32-10(counter = (i, k / 4, step lo, step hi),
 *                                       key = (seed lo, seed hi xor (layer + 1)))
 * keep iff x[k mod 4] >= floor(p * 2^32).  mask (optional) receives 1 for kept elements.
 * p = 0 keeps everything.
 */
void orc_dropout(int64_t N, int32_t d, double p, uint64_t seed, uint64_t step, int32_t layer,
                 const double *H, double *out, uint8_t *mask)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) ^ (uint32_t)(layer + 1) };
    uint32_t thr = (uint32_t)(p * 4294967296.0);
    double scale = 1.0 / (1.0 - p);
    for (int64_t i = 0; i < N; ++i)
        for (int32_t g = 0; g < (d + 3) / 4; ++g) {
            uint32_t ctr[4] = { (uint32_t)i, (uint32_t)g, (uint32_t)step, (uint32_t)(step >> 32) };
            uint32_t x[4];
            orc_philox4x32_10(ctr, key, x);
            for (int32_t q = 0; q < 4 && 4 * g + q < d; ++q) {
                size_t e = (size_t)i * d + 4 * g + q;
                int keep = p <= 0.0 || x[q] >= thr;
                out[e] = keep ? H[e] * scale : 0.0;
                if (mask) mask[e] = (uint8_t)keep;
            }
        }
}
