/*
 * kge_mi355 — C ABI of one training step of a partitioned RGCN + DistMult
 * knowledge-graph-embedding trainer on one AMD MI355X (gfx950).
 *
 * The calls follow the training procedure of "Scaling Knowledge Graph
 * Embedding Models" (arXiv 2201.02791), Algorithm 1, for ONE trainer working
 * on ONE self-sufficient partition:
 *
 *   kge_build_partition      Sec. 3.2.1 (core edges) + Sec. 3.2.2 (n-hop
 *                            Neighborhood Expansion); once per partition
 *   kge_rgcn_forward         Eq. 1 with the basis decomposition of Eq. 2
 *   kge_compute_graph        Sec. 3.3 / Algorithm 1 "getComputeGraph": the
 *                            vertices within n_layers hops of an edge batch
 *   kge_sample_negatives     Sec. 2.1 (corrupt s or t) under the in-partition
 *                            constraint of Sec. 3.3.1
 *   kge_distmult_score_loss  Eq. 4 (DistMult) and Eq. 3 (cross entropy), with
 *                            the gradients with respect to embeddings and M_r
 *   kge_rgcn_backward        chain rule on Eq. 1-2 (Algorithm 1, "backward")
 *   kge_optimizer_step       Algorithm 1, "optimizer.step()"
 *
 * General rules
 *  - Every function returns KGE_OK (0) or a negative kge_status; on error no
 *    output is valid and kge_last_error() holds a message for this thread.
 *  - "device" pointers are HIP device memory on the partition's GPU, owned by
 *    the caller; "host" pointers are ordinary host memory.  The library owns
 *    only kge_partition objects.  The four per-step calls allocate nothing,
 *    never synchronise with the host, and run asynchronously on `stream`
 *    (a hipStream_t passed as void*; NULL = the default stream).
 *  - Row vectors: h is 1 x d, V_b is d_in x d_out, a projection is h V_b.
 *  - Local vertex ids are ranks of global ids inside the partition.
 *    Relation ids 0..R-1 are the given direction, R..2R-1 the inverses; the
 *    self-loop is the dense W_0 term, not an edge.
 *  - All matrices are dense row-major.  Feature widths must be multiples of 4
 *    (of 8 when msg_dtype = KGE_MSG_BF16).  Per layer and order:
 *      project-first     d_in <= 512, d_out <= 256
 *      relation-weight   d_in, d_out <= 256 (512 with bf16 messages)
 *    A wider layer is refused with KGE_EINVAL before anything runs.
 */
#ifndef KGE_MI355_H
#define KGE_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum kge_status {
    KGE_OK = 0,
    KGE_EINVAL = -1,  /* null pointer, bad shape, bad enum value            */
    KGE_ENOMEM = -2,  /* allocation failed, or the workspace is too small    */
    KGE_EHIP = -3,    /* a HIP call failed; see kge_last_error()             */
    KGE_ERANGE = -4   /* an id is out of range, or a size exceeds 2^31-1     */
} kge_status;

enum { KGE_ACT_IDENTITY = 0, KGE_ACT_RELU = 1 };
enum { KGE_MSG_F32 = 0, KGE_MSG_BF16 = 1 };      /* storage type of projected messages        */
enum { KGE_NEG_TAIL = 0, KGE_NEG_HEAD_OR_TAIL = 1 };
enum { KGE_DOMAIN_CORE = 0, KGE_DOMAIN_ALL = 1 };
/* Order in which a layer applies Eq. 1-2 (the results are the same up to rounding):
 *   KGE_ORDER_PROJECT_FIRST    the order the step is usually written in: P[j][b] = h_j V_b for every vertex,
 *                              then the neighbour sum over projected messages.  (B+1) d_out values move
 *                              per edge.
 *   KGE_ORDER_RELATION_WEIGHTS the library's product path (what the benchmark times): run means
 *                              z_{i,r} = (1/c_ir) sum_{j in N_i^r} h_j per (relation, destination) run, then
 *                              Eq. 2 written out, W_r = sum_b a_rb V_b for every relation, and
 *                              pre_i = sum_r z_{i,r} W_r + h_i W_0 as one product per run, grouped by relation
 *                              over the (relation, destination)-sorted runs.  d_in values move per edge and
 *                              S d_in d_out multiply-adds replace N B d_in d_out.
 * (Value 1 belonged to a third order that was removed; it is refused.) */
enum { KGE_ORDER_PROJECT_FIRST = 0, KGE_ORDER_RELATION_WEIGHTS = 2 };

typedef struct kge_partition kge_partition;      /* opaque; device resident; library owned    */
typedef struct kge_cgraph kge_cgraph;            /* opaque; one batch's computational sub-graph */
typedef struct kge_score_index kge_score_index;  /* opaque; scratch of the atomic-free scoring call    */

typedef struct kge_part_info {
    int64_t n_vert;        /* N: vertices after expansion (numerator term of Eq. 7)            */
    int64_t n_edge;        /* E: message edges kept                                             */
    int64_t n_seg;         /* S: distinct (relation, destination) pairs                         */
    int64_t n_core;        /* core edges = positive triples of this partition                   */
    int64_t n_cand;        /* vertices negatives may be drawn from                              */
    int64_t n_triples;     /* triples of the whole graph                                        */
    int32_t n_entities, n_relations, n_parts, part_id, n_hops, neg_domain;
    int32_t max_in_degree; /* largest number of message edges into one vertex                   */
    int32_t max_out_degree;
} kge_part_info;

/* One RGCN layer (Eq. 1-2).  Device pointers, caller owned, never written. */
typedef struct kge_layer {
    int32_t d_in, d_out, n_bases, act;   /* act: KGE_ACT_*                                     */
    int32_t order;     /* KGE_ORDER_*                                                           */
    const float *V;    /* [n_bases][d_in][d_out]   basis matrices V_b                          */
    const float *a;    /* [2R][n_bases]            coefficients a_rb                           */
    const float *W0;   /* [d_in][d_out]            self-loop weight                            */
    /* Dropout on the layer's input (training setting of Sec. 4: 0.2 on the large graphs), inverted
     * form: every element the layer reads - for the neighbour messages, the self-loop and the weight
     * gradients - is zeroed with probability `dropout` and scaled by 1 / (1 - dropout) otherwise.
     * Element (i, k) is kept iff word (k mod 4) of Philox4x32-10(counter = (i, k / 4, step lo, step hi),
     * key = (seed lo, seed hi xor (layer index + 1))) is >= floor(dropout * 2^32).  0 = off (the three
     * fields are then ignored); must be in [0, 1).  kge_rgcn_backward must see the same three values
     * as the forward call it follows; change drop_step between training steps for a fresh mask. */
    float dropout;
    uint64_t drop_seed, drop_step;
} kge_layer;

/* Gradients of one layer; device pointers, caller owned, overwritten. */
typedef struct kge_layer_grad {
    float *dV;   /* [n_bases][d_in][d_out] */
    float *da;   /* [2R][n_bases]          */
    float *dW0;  /* [d_in][d_out]          */
} kge_layer_grad;

/* Arrays kge_partition_export can copy out (all 4-byte elements). */
typedef enum kge_array {
    KGE_ARR_VERT_GID = 0,  /* int32 [N]    global id of each local vertex, ascending           */
    KGE_ARR_CORE_EID = 1,  /* int32 [n_core] index of each core triple in the input lists       */
    KGE_ARR_CORE_H = 2,    /* int32 [n_core] local head                                        */
    KGE_ARR_CORE_R = 3,    /* int32 [n_core] relation (0..R-1)                                 */
    KGE_ARR_CORE_T = 4,    /* int32 [n_core] local tail                                        */
    KGE_ARR_SEG_PTR = 5,   /* int32 [S+1]  edge range of each (relation, destination) run      */
    KGE_ARR_SEG_REL = 6,   /* int32 [S]                                                        */
    KGE_ARR_SEG_DST = 7,   /* int32 [S]    local destination                                   */
    KGE_ARR_INV_C = 8,     /* float [S]    1 / c_{i,r} = 1.0f / run length                     */
    KGE_ARR_COL_SRC = 9,   /* int32 [E]    local source, edges sorted by (rel, dst, src, id)   */
    KGE_ARR_EDGE_ID = 10,  /* int32 [E]    message-edge id: triple i -> i, its inverse -> M+i  */
    KGE_ARR_CAND = 11,     /* int32 [n_cand] local ids, ascending                              */
    KGE_ARR_DM_PTR = 12,   /* int32 [N+1]  destination-major view: edge range per destination  */
    KGE_ARR_DM_SRC = 13,   /* int32 [E]    source of each edge, ordered by (dst, rel, src, id) */
    KGE_ARR_DM_REL = 14,   /* int32 [E]                                                        */
    KGE_ARR_DM_INVC = 15,  /* float [E]    1 / c of the edge's run                             */
    KGE_ARR_SM_PTR = 16,   /* int32 [N+1]  source-major view: edge range per source            */
    KGE_ARR_SM_DST = 17,   /* int32 [E]    destination, ordered by (src, rel, dst, id)         */
    KGE_ARR_SM_REL = 18,   /* int32 [E]                                                        */
    KGE_ARR_SM_INVC = 19,  /* float [E]                                                        */
    KGE_ARR_REL_PTR = 20,  /* int32 [2R+1] run range of each relation                          */
    KGE_ARR_DR_PTR = 21,   /* int32 [N+1]  runs grouped by destination: run range per vertex   */
    KGE_ARR_DR_SEG = 22,   /* int32 [S]    run id, ordered by (dst, rel)                       */
    KGE_ARR_DR_REL = 23,   /* int32 [S]    relation of that run                                */
    KGE_ARR_SM_SEG = 24    /* int32 [E]    run id of each edge in source-major order           */
} kge_array;

/*
 * Build partition `part_id` of `n_parts` (Sec. 3.2).
 *   head, rel, tail : HOST int32 [n_triples], the whole graph's training triples (s, r, t);
 *                     entity ids in [0, n_entities), relation ids in [0, n_relations).
 *   Core edges (the positives, Sec. 3.2.1) are the triples with
 *       ((uint32)head * 0x9E3779B1u >> 8) mod n_parts == part_id
 *   (a hash stands in for the paper's vertex-cut partitioner: disjoint cover of the edges).
 *   Expansion (Sec. 3.2.2): S_0 = endpoints of core edges; S_k = S_{k-1} plus the sources of
 *   all message edges into S_{k-1}; the partition keeps the vertices S_{n_hops} and every
 *   message edge whose destination is in S_{n_hops-1}.  n_hops = number of GNN layers.
 *   neg_domain: KGE_DOMAIN_CORE = negatives drawn from endpoints of core edges (Sec. 3.3.1),
 *               KGE_DOMAIN_ALL  = from every vertex of the partition.
 *   The edges are sorted on the GPU by (relation, destination, source, message-edge id);
 *   c_{i,r} of Eq. 1 is the length of a (relation, destination) run, with multiplicity.
 *   *out receives a new partition living on the current HIP device; free it with
 *   kge_partition_destroy.  Synchronous.  KGE_ERANGE if an id is out of range or the packed
 *   sort key (bits(2R) + 2 bits(N)) exceeds 64 bits.
 */
int kge_build_partition(const int32_t *head, const int32_t *rel, const int32_t *tail,
                        int64_t n_triples, int32_t n_entities, int32_t n_relations,
                        int32_t n_parts, int32_t part_id, int32_t n_hops, int32_t neg_domain,
                        kge_partition **out);

int kge_partition_info(const kge_partition *p, kge_part_info *out);

/* Ids inside device arrays (core-edge indices in pos_core_idx, entities in neg_ent) cannot be checked by the
 * host without a synchronisation, so the kernels of kge_compute_graph and kge_distmult_score_loss check them:
 * an id outside [0, n_core) / [0, N) is counted in the partition and skipped or replaced by 0 - it never becomes
 * an address - and the outputs of that call are meaningless.  This call (it synchronises the device) writes to
 * *host_count how many such ids the partition's calls have met since it was built; a caller that cannot vouch
 * for its ids reads it once per epoch and treats a non-zero count as KGE_ERANGE. */
int kge_partition_bad_ids(const kge_partition *p, int64_t *host_count);

/* Copy one array to HOST memory `host_dst` of `bytes` bytes (must equal 4 * its length).
 * Synchronous. */
int kge_partition_export(const kge_partition *p, int32_t which, void *host_dst, int64_t bytes);

void kge_partition_destroy(kge_partition *p);

/* Bytes of device workspace kge_rgcn_forward / kge_rgcn_backward need for these layers.
 * Returns 0 on invalid arguments (kge_last_error explains). */
size_t kge_workspace_bytes(const kge_partition *p, const kge_layer *layers, int32_t n_layers,
                           int32_t msg_dtype);

/*
 * Computational sub-graph of one edge batch (Sec. 3.3; Algorithm 1, "getComputeGraph").
 * With L layers the batch's final embeddings depend only on vertices within L hops along
 * incoming message edges.  For l = L-1 .. 0 (0-based layer index) the object holds one byte per
 * vertex, active_l[i] = 1 iff layer l has to produce a row for vertex i:
 *   active_{L-1} = heads and tails of the batch's positives and every corrupting entity,
 *   active_{l-1} = active_l united with the sources of all message edges into active_l.
 * A self-sufficient partition (n_hops >= L) contains every such vertex and edge.
 *
 * kge_cgraph_create allocates the flags for a partition and a layer count (once per trainer;
 * synchronous); kge_cgraph_destroy frees them.  kge_compute_graph fills them for one batch:
 * asynchronous on `stream`, no allocation, no host synchronisation.
 *   pos_core_idx : device int32 [n_pos], each in [0, n_core) (checked on the device, see kge_partition_bad_ids)
 *   neg_ent      : device int32 [n_neg_entries] local vertex ids (as written by
 *                  kge_sample_negatives, n_neg_entries = n_pos * n_neg), or NULL with 0
 * kge_cgraph_export (synchronises the device) copies the flags to HOST uint8 [L][N] and/or, per
 * layer, four counts to HOST int64 [L][4]: active vertices, message edges into them,
 * (relation, destination) runs into them, and message edges out of them; either pointer may be NULL.
 */
int kge_cgraph_create(const kge_partition *p, int32_t n_layers, kge_cgraph **out);
void kge_cgraph_destroy(kge_cgraph *cg);
int kge_compute_graph(const kge_partition *p, kge_cgraph *cg, const int32_t *pos_core_idx,
                      int64_t n_pos, const int32_t *neg_ent, int64_t n_neg_entries, void *stream);
int kge_cgraph_export(const kge_cgraph *cg, uint8_t *host_active, int64_t *host_stats);
/* The rows of the first layer's INPUT that the batch filled in by kge_compute_graph reads: active_0 united with
 * the sources of all message edges into active_0 (one hop beyond the first layer's outputs).  With learned
 * entity embeddings as that input these are exactly the rows the step produces a gradient for (Algorithm 1's
 * update touches no other row): pass *device_flags (device uint8 [N], owned by cg, valid until the next
 * kge_compute_graph on it or its destruction) as row_mask to kge_optimizer_step_rows.  host_flags (HOST uint8
 * [N]) and host_count (HOST, number of flagged rows) synchronise the device when given; any of the three may
 * be NULL. */
int kge_cgraph_input_rows(const kge_cgraph *cg, const uint8_t **device_flags, uint8_t *host_flags,
                          int64_t *host_count);

/*
 * Encoder forward (Eq. 1-2), for l = 1..n_layers:
 *   P_l[j][b][:] = h_j V_b (stored as msg_dtype),  pre_i = sum_r sum_{j in N_i^r} (1/c_ir)
 *   sum_b a_rb P_l[j][b][:] + h_i W_0,  h'_i = act(pre_i)   (fp32 accumulation throughout).
 *   layers    : HOST array of n_layers descriptors (their pointers are device memory);
 *               layers[l].d_in must equal layers[l-1].d_out.
 *   H0        : device float [N][layers[0].d_in]
 *   workspace : device, >= kge_workspace_bytes(...), 256-byte aligned; keeps what backward needs
 *   H_out     : device float [N][layers[n_layers-1].d_out]
 *   cg        : NULL = propagate the whole partition.  Otherwise a sub-graph filled by
 *               kge_compute_graph for the batch that will be scored: each layer aggregates only
 *               into its active destinations and writes zero rows elsewhere.  The rows of H_out
 *               on the batch's vertices, the loss and every gradient are the same as with NULL
 *               (rows outside cannot reach the batch); H_out rows of other vertices are zero.
 */
int kge_rgcn_forward(const kge_partition *p, const kge_cgraph *cg, const kge_layer *layers,
                     int32_t n_layers, int32_t msg_dtype, const float *H0, void *workspace,
                     size_t ws_bytes, float *H_out, void *stream);

/*
 * Encoder backward.  Must follow kge_rgcn_forward with the same arguments and the same,
 * unmodified workspace.
 *   dH_out : device float [N][d_out of last layer], dL/dH_out (e.g. from kge_distmult_score_loss);
 *            left unchanged
 *   grads  : HOST array of n_layers kge_layer_grad (device pointers); every array is overwritten
 *   dH0    : device float [N][layers[0].d_in] or NULL (NULL when the layer-1 input is a fixed
 *            feature matrix and needs no gradient)
 *   cg     : the same object (or NULL) the forward call got; dH_out must then be zero outside
 *            the batch's vertices, as kge_distmult_score_loss writes it
 */
int kge_rgcn_backward(const kge_partition *p, const kge_cgraph *cg, const kge_layer *layers,
                      int32_t n_layers, int32_t msg_dtype, const float *H0, void *workspace,
                      size_t ws_bytes, const float *dH_out, const kge_layer_grad *grads, float *dH0,
                      void *stream);

/*
 * Negatives for a batch of positives (Sec. 2.1, Sec. 3.3.1).  For positive q (core-edge index
 * c = pos_core_idx[q]) and slot k:
 *   x = Philox4x32-10(counter = (c, k, step lo32, step hi32), key = (seed lo32, seed hi32))
 *   neg_ent[q][k]  = cand[(x0 * n_cand) >> 32]                    (a local vertex id)
 *   neg_side[q][k] = 1 (head replaced) if mode = KGE_NEG_HEAD_OR_TAIL and x1 >= 2^31,
 *                    else 0 (tail replaced)
 * No filtering against true triples.  pos_core_idx: device int32 [n_pos], values in
 * [0, n_core) (not checked on the device; the draw only uses them as counter words).
 * neg_ent: device int32 [n_pos][n_neg]; neg_side: device uint8 [n_pos][n_neg].
 * KGE_EINVAL if the partition has no candidate vertex and n_pos * n_neg > 0.
 */
int kge_sample_negatives(const kge_partition *p, const int32_t *pos_core_idx, int64_t n_pos,
                         int32_t n_neg, int32_t mode, uint64_t seed, uint64_t step,
                         int32_t *neg_ent, uint8_t *neg_side, void *stream);

/*
 * DistMult score (Eq. 4), cross-entropy loss (Eq. 3, minimised form with the leading minus)
 * and gradients, fused.  Scored triples are positive-major: row q = [positive, negative 0 ..
 * n_neg-1]; |T| = n_pos (1 + n_neg).
 *   g = sum_k h_s[k] M_r[k] h_t[k];  loss = (1/|T|) sum softplus(-g) [y=1] or softplus(g) [y=0]
 *   delta = (sigmoid(g) - y)/|T|;  dH[s] += delta M_r*h_t;  dH[t] += delta M_r*h_s;
 *   dM[r] += delta h_s*h_t
 *   H      : device float [N][d]          M : device float [R][d]
 *   pos_core_idx : device int32 [n_pos], each in [0, n_core)
 *   neg_ent / neg_side : as written by kge_sample_negatives, entries in [0, N)
 *   scores : device float [n_pos][1+n_neg] or NULL
 *   loss   : device float [1]
 *   dH     : device float [N][d], overwritten (every row; rows no triple names become zero)
 *   dM     : device float [R][d], overwritten
 *   index  : NULL, or scratch from kge_score_index_create.
 *     NULL : rows are added into dH with fp32 atomics as the triples are scored; low-order bits of dH can
 *            differ from run to run.
 *     else : the atomic-free form.  The rows every scored triple adds into dH (one per negative, to the
 *            corrupting entity; two per positive, to its head and tail) are sorted by entity with a stable
 *            radix sort inside the call, the triples are scored, and one wavefront per entity adds up its rows
 *            in the order of the batch: every row of dH is written once and the result repeats bit for bit.
 *            H, M and dH must then be 16-byte aligned.
 *   In both forms an id outside [0, n_core) / [0, N) is replaced by 0 and counted (kge_partition_bad_ids).
 *   dM and the loss are accumulated with fp32 atomics in both forms.
 *
 * kge_score_index_create allocates the scratch for batches of at most max_pos positives with at most max_neg
 * negatives each and embedding width d (about (n_neg + 2) x 36 bytes + 8 d bytes per positive, plus 4 N bytes);
 * once per trainer, synchronous; free with kge_score_index_destroy.
 */
int kge_score_index_create(const kge_partition *p, int64_t max_pos, int32_t max_neg, int32_t d,
                           kge_score_index **out);
void kge_score_index_destroy(kge_score_index *index);
int kge_distmult_score_loss(const kge_partition *p, kge_score_index *index, const float *H, const float *M,
                            int32_t d, const int32_t *pos_core_idx, int64_t n_pos, const int32_t *neg_ent,
                            const uint8_t *neg_side, int32_t n_neg, float *scores, float *loss,
                            float *dH, float *dM, void *stream);

/*
 * Optimizer step (Algorithm 1, "optimizer.step()"; learning rate 0.01 in the paper's large-graph
 * setting).  The paper speaks of synchronous gradient descent and does not name the update rule:
 *   KGE_OPT_SGD   p <- p - lr g
 *   KGE_OPT_ADAM  m <- beta1 m + (1 - beta1) g;  v <- beta2 v + (1 - beta2) g^2;
 *                 p <- p - lr (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps),  t = 1, 2, ...
 * kge_optimizer_step updates n elements of one tensor in place; param, grad, m, v are device float
 * arrays (m, v: Adam only, zero before the first step).  kge_optimizer_step_rows treats the tensors as
 * [n_rows][d] (d a multiple of 4, 16-byte aligned) and leaves a row - parameters and moments - as it
 * is when row_mask[row] == 0 (device uint8 [n_rows]) or, with row_mask NULL, when the row's gradient is
 * all zeros: the update for an embedding table of which a step reaches few rows.  The bias correction
 * uses the global t for every row.  Asynchronous on `stream`, no allocation.
 */
enum { KGE_OPT_SGD = 0, KGE_OPT_ADAM = 1 };
typedef struct kge_opt {
    int32_t kind;      /* KGE_OPT_*                                   */
    float lr, beta1, beta2, eps;
    int64_t t;         /* number of this step, starting at 1 (Adam)   */
} kge_opt;
int kge_optimizer_step(const kge_opt *opt, float *param, const float *grad, float *m, float *v,
                       int64_t n, void *stream);
int kge_optimizer_step_rows(const kge_opt *opt, float *param, const float *grad, float *m, float *v,
                            int64_t n_rows, int32_t d, const uint8_t *row_mask, void *stream);

/*
 * Link-prediction evaluation ("Evaluation Metrics" section: filtered setting, MRR Eq. 5, Hits@k Eq. 6).
 *
 * A query fixes one entity and a relation and asks for the other entity of a test triple (h, r, t):
 * the tail query fixes h (answer t), the head query fixes t (answer h).  DistMult (Eq. 4) is symmetric
 * in its entities, so a candidate e scores  sum_k H[fixed][k] M[r][k] H[e][k]  in both directions.
 * Candidates are all entities except the answer; with a filter, also except every entity whose triple
 * with the query's (fixed entity, relation) is among the filter's known triples.  Per query the calls
 * return `higher` = candidates scoring strictly above the answer and `equal` = candidates scoring
 * exactly the same (fp32 scores); the answer's rank in the list sorted by descending score is
 * 1 + higher with ties placed first, 1 + higher + equal with ties placed last.  kge_eval_metrics uses
 * rank = 1 + higher + equal / 2 (the mean position over all orders of the ties; the paper leaves the
 * order of equal scores open).
 *
 * kge_eval_filter_create: head, rel, tail are HOST int32 [n_known] (the triples whose corruptions are
 *   dropped: the training triples in the paper's setting); ids must be in range (KGE_ERANGE).  Sorts
 *   and de-duplicates on the host and keeps two device tables.  Synchronous; free with _destroy.
 * kge_eval_rank_all: H DEVICE float [n_entities][d] (d a multiple of 4, <= 1024, 16-byte aligned),
 *   M DEVICE float [n_relations][d], test_h/r/t DEVICE int32 [n_test]; filter may be NULL (raw setting)
 *   and must have been built for the same n_entities / n_relations.  higher, equal: DEVICE int32
 *   [2 n_test], tail queries first, then head queries.  workspace: DEVICE, 256-byte aligned, at least
 *   kge_eval_workspace_bytes(2 n_test, d) bytes.  Scores are an (2 n_test x d) by (d x n_entities)
 *   product on the fp32 matrix cores that is compared and counted tile by tile, never stored.
 * kge_eval_rank_candidates: every query brings its own list cand[q][0..n_cand) (DEVICE int32; the
 *   setting of the large citation graph, which ships a fixed number of negative targets per test edge);
 *   fixed, rel, answer: DEVICE int32 [n_queries]; an entry equal to the answer is skipped.
 * kge_eval_metrics: out DEVICE double [1 + n_ks] = MRR, Hits@ks[0], ..; ks HOST int32 [n_ks], n_ks <= 8.
 * All three are asynchronous on `stream`, allocate nothing, and return KGE_EINVAL on bad arguments;
 * entity / relation ids inside the device arrays are the caller's responsibility.
 */
typedef struct kge_eval_filter kge_eval_filter;
int kge_eval_filter_create(const int32_t *head, const int32_t *rel, const int32_t *tail, int64_t n_known,
                           int32_t n_entities, int32_t n_relations, kge_eval_filter **out);
void kge_eval_filter_destroy(kge_eval_filter *f);
size_t kge_eval_workspace_bytes(int64_t n_queries, int32_t d);
int kge_eval_rank_all(const kge_eval_filter *filter, const float *H, int64_t n_entities, int32_t d,
                      const float *M, int32_t n_relations, const int32_t *test_h, const int32_t *test_r,
                      const int32_t *test_t, int64_t n_test, void *workspace, size_t ws_bytes,
                      int32_t *higher, int32_t *equal, void *stream);
int kge_eval_rank_candidates(const float *H, int64_t n_entities, int32_t d, const float *M,
                             int32_t n_relations, const int32_t *fixed, const int32_t *rel,
                             const int32_t *answer, int64_t n_queries, const int32_t *cand, int32_t n_cand,
                             void *workspace, size_t ws_bytes, int32_t *higher, int32_t *equal, void *stream);
int kge_eval_metrics(const int32_t *higher, const int32_t *equal, int64_t n_queries, const int32_t *ks,
                     int32_t n_ks, double *out, void *stream);
/*
 * kge_eval_rank_all for callers that cannot allocate device memory and have no workspace to hand over:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * (minus the workspace), same kernels, same results; the scratch (query vectors, answer scores,
 * per-query counters) lives in a static device array of KGE_EVAL_STATIC_BYTES inside the library, one
 * copy per GPU, held until the process ends.  The call allocates nothing and never synchronises.
 *   Limit: kge_eval_workspace_bytes(2 n_test, d) <= KGE_EVAL_STATIC_BYTES (about 15,000 test triples at
 *   d = 256, 28,000 at d = 128); beyond it the call returns KGE_ENOMEM and nothing runs.
 *   All calls on one GPU share that GPU's array: two calls that overlap in time (different streams or
 *   threads) race on it; calls on one stream are ordered and safe.  The counters are cleared by a fill
 *   kernel at the start of every call, so a call never sees the previous call's contents.
 */
#define KGE_EVAL_STATIC_BYTES (32u << 20)
int kge_eval_rank_all_static(const kge_eval_filter *filter, const float *H, int64_t n_entities, int32_t d,
                             const float *M, int32_t n_relations, const int32_t *test_h, const int32_t *test_r,
                             const int32_t *test_t, int64_t n_test, int32_t *higher, int32_t *equal, void *stream);

/*
 * Per-kernel timing for benchmarks (not part of the training path).  While enabled, every
 * kernel launch of the per-step calls is bracketed by two HIP events recorded on the launch
 * stream.  kge_profile_collect waits for the recorded events, sums the elapsed time per
 * kernel name into out[0..*n_entries) (at most max_entries), and clears the records.
 * Not thread safe; enabling allocates events, so keep it off in allocation-free callers.
 */
typedef struct kge_prof_entry {
    char name[32];
    double total_ms;
    int64_t calls;
} kge_prof_entry;
int kge_profile_enable(int32_t on);
int kge_profile_collect(kge_prof_entry *out, int32_t max_entries, int32_t *n_entries);

/*
 * Where the intermediates of a step live inside the caller-owned workspace (for inspection and
 * tests; the layout is fixed by the partition, the layer list and msg_dtype).  Writes the byte
 * offset and size of one slice:
 *   KGE_WS_P    layer l's projected messages P_l [N][B*d_out], msg_dtype (valid after forward)
 *   KGE_WS_H    layer l's output H_l [N][d_out] float (valid after forward; the last layer's
 *               output is the call's H_out, and this copy of it is written only when that
 *               layer has ReLU)
 *   KGE_WS_G    G = dL/d(pre) [N][d_out] float of the last ReLU layer backward has processed
 *               (a layer with identity activation uses its incoming gradient in place)
 *   KGE_WS_DP   dP of the last layer backward has processed: [N][ld] msg_dtype with
 *               ld = B*d_out (fp32 messages) or (B+1)*d_out (bf16 messages: G, rounded to
 *               bf16, is appended behind the B blocks)
 *   KGE_WS_DH   gradient with respect to layer l's INPUT, l >= 1, [N][d_in] float (after backward)
 *   KGE_WS_Z    relation-weight layer l: run means z [S][d_in], one row per (relation,
 *               destination) run in the partition's run order (valid after forward).  A relation-weight
 *               layer with bf16 messages leaves the rows of single-edge runs unwritten: such a run's mean
 *               is its source's row of the layer input, which the layer reads in place
 *   KGE_WS_HD   layer l's input after dropout [N][d_in] float (valid after forward; only for layers
 *               with dropout > 0; with dropout, KGE_WS_DH is the gradient with respect to the
 *               input BEFORE dropout)
 *   KGE_WS_U    relation-weight layers: one buffer shared by all of them, msg_dtype elements.  After
 *               forward it holds u [S][d_out] of the last layer (the per-run products z W_r); after
 *               backward dz [S][d_in] of the last layer that produced an input gradient.  The slice
 *               is sized for the wider of the two.
 * KGE_WS_P exists only for project-first layers; KGE_WS_Z, KGE_WS_U and no KGE_WS_DP contents beyond G for
 * relation-weight layers.
 */
enum { KGE_WS_P = 0, KGE_WS_H = 1, KGE_WS_G = 2, KGE_WS_DP = 3, KGE_WS_DH = 4, KGE_WS_Z = 5, KGE_WS_U = 7, KGE_WS_HD = 8 };
int kge_workspace_slice(const kge_partition *p, const kge_layer *layers, int32_t n_layers,
                        int32_t msg_dtype, int32_t which, int32_t layer, size_t *offset,
                        size_t *bytes);

/* Message of the last failure on the calling thread ("" if none). */
const char *kge_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* KGE_MI355_H */
