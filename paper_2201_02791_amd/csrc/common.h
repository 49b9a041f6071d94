// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "kge_mi355.h"
#include "kge_mi355_testing.h"

void kge_set_error(const char *fmt, ...);

#define KGE_HIP(expr)                                                                         \
    do {                                                                                      \
        hipError_t e__ = (expr);                                                              \
        if (e__ != hipSuccess) {                                                              \
            kge_set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__,   \
                          __LINE__);                                                          \
            return KGE_EHIP;                                                                  \
        }                                                                                     \
    } while (0)

#define KGE_REQUIRE(cond, code, ...)                                                          \
    do {                                                                                      \
        if (!(cond)) {                                                                        \
            kge_set_error(__VA_ARGS__);                                                       \
            return (code);                                                                    \
        }                                                                                     \
    } while (0)

#define KGE_LAUNCH_CHECK() KGE_HIP(hipGetLastError())

// Rows (destinations, sources or runs) with at least KGE_HEAVY edges are cut into units of at most
// KGE_HEAVY edges; each unit is handled by its own wavefront and writes a partial result that a
// small finishing kernel sums in unit order (deterministic).  Power-law graphs put a large share
// of all edges into such rows.
#define KGE_HEAVY 256
struct kge_heavy_index {
    int32_t n_hv, n_units;
    int32_t *hv_row;        // [n_hv]    row id of each heavy row, ascending
    int32_t *hv_unit_ptr;   // [n_hv+1]  first unit of each heavy row
    int32_t *unit_hv;       // [n_units] heavy-row index of each unit
};

struct kge_partition {
    int device;
    int64_t n_vert, n_edge, n_seg, n_core, n_cand, n_triples;
    int32_t n_entities, n_relations, n_parts, part_id, n_hops, neg_domain;
    int32_t max_in_degree, max_out_degree;
    // canonical arrays (bit-exact contract)
    int32_t *vert_gid, *core_eid, *core_h, *core_r, *core_t;
    int32_t *seg_ptr, *seg_rel, *seg_dst;
    float *inv_c;
    int32_t *col_src, *edge_id, *cand;
    // destination-major and source-major views of the same edges
    int32_t *dm_ptr, *dm_src, *dm_rel;
    float *dm_invc;
    int32_t *sm_ptr, *sm_dst, *sm_rel;
    float *sm_invc;
    int32_t *sm_seg;    // [E] run id of each edge in source-major order
    int32_t *rel_ptr;   // [2R+1] run range per relation
    kge_heavy_index hv_dm, hv_sm, hv_seg;   // heavy destinations, sources, runs
    // the runs grouped by destination (order dst, rel): dr_seg = run id, dr_rel = its relation
    int32_t *dr_ptr, *dr_seg, *dr_rel;
    kge_heavy_index hv_dr;
    // each relation's run range cut into chunks of KGE_REL_CHUNK .. 8 KGE_REL_CHUNK runs (about 2048 chunks in all)
    int32_t n_relc;
    int32_t *relc_rel, *relc_beg, *relc_end;
    // and into row tiles of at most KGE_REL_TILE runs
    int32_t n_relt;
    int32_t *relt_rel, *relt_beg, *relt_end;
    // and into ranges of at most KGE_REL_RANGE runs (what one block of the bf16 per-run products takes)
    int32_t n_relr;
    int32_t *relr_rel, *relr_beg, *relr_end;
    // the same kind of ranges ordered by slab of the destination range first (KGE_REL_SLAB vertices), relation
    // second: the order in which the transposed per-run products gather the output-gradient rows
    int32_t n_rels;
    int32_t *rels_rel, *rels_beg, *rels_end;
    // where the mean of run s can be read when the layer input X [N][d] and the run means Z [S][d] are one
    // matrix [X; Z]: a run of a single edge has its source's row of X as its mean (row col_src), any other
    // run row N + s.  NULL if N + S does not fit 31 bits.
    int32_t *seg_zrow;
    // the runs of two or more edges, ascending (the only ones whose mean is computed when single-edge runs
    // are read in place); allocated together with seg_zrow
    int64_t n_mrun;
    int32_t *mrun;
    // [1] how many ids outside the partition (core-edge indices, entities) the per-step kernels have met so far:
    // such an id is counted and replaced or skipped, never used as an address (kge_partition_bad_ids)
    uint32_t *bad_ids;
};
#define KGE_REL_CHUNK 2048
#define KGE_REL_TILE 128
#define KGE_REL_RANGE 4096
// vertices per slab of the destination range by which those ranges are ordered
#define KGE_REL_SLAB 262144

// Optional per-kernel timing with HIP events on the launch stream (kge_profile_enable).
struct KgeProfScope {
    KgeProfScope(const char *name, hipStream_t st);
    ~KgeProfScope();
    int slot;
    hipStream_t st;
};
#define KGE_PROF(name, st) KgeProfScope prof_scope__(name, st)

static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- kernels' host launchers (implemented in the .hip files) ----

// gemm.hip (fp32 messages) -------------------------------------------------
// P[N][B*d_out] and Self[N][d_out] = H[N][d_in] * [V_1 .. V_B | W0]
int launch_project(const float *H, int64_t N, int32_t d_in, int32_t d_out, int32_t B,
                   const float *V, const float *W0, float *P, float *Self, hipStream_t st);
// dV[B][d_in][d_out] = H^T dP_b ; dW0 = H^T G      (outputs zeroed inside, split over N)
int launch_weight_grad(const float *H, int64_t N, int32_t d_in, int32_t d_out, int32_t B,
                       const float *dP, const float *G, float *dV, float *dW0, hipStream_t st);
// dH[N][d_in] = sum_b dP_b V_b^T + G W0^T
int launch_input_grad(const float *dP, const float *G, int64_t N, int32_t d_in, int32_t d_out,
                      int32_t B, const float *V, const float *W0, float *dH, hipStream_t st);

// gemm_bf16.hip (bf16 messages): every operand is a row-major bf16 matrix ----
int launch_cvt_rows_bf16(const float *src, int64_t n, void *dst, hipStream_t st);
int launch_cvt_weights_bf16(const float *V, const float *W0, int32_t d_in, int32_t d_out, int32_t B,
                            void *Wbf /*[d_in][nc]*/, void *WbfT /*[nc][d_in]*/, hipStream_t st);
// G (fp32 [N][d_out]) -> last d_out columns of X (bf16 [N][(B+1) d_out])
int launch_append_g_bf16(const float *G, int64_t N, int32_t d_out, int32_t B, void *X, hipStream_t st);
// G = act'(Hout) * dHout in fp32 and, in the same pass, its bf16 copy behind the B d_out columns of X
int launch_act_backward_append_bf16(const float *dHout, const float *Hout, int act, int64_t N, int32_t d_out, int32_t B,
                                    float *G, void *X, hipStream_t st);
int launch_project_bf16(const void *Hbf, int64_t N, int32_t d_in, int32_t d_out, int32_t B,
                        const void *WbfT, void *P, float *Self, hipStream_t st);
int launch_weight_grad_bf16(const void *Hbf, int64_t N, int32_t d_in, int32_t d_out, int32_t B,
                            const void *X, float *dV, float *dW0, hipStream_t st);
int launch_input_grad_bf16(const void *X, int64_t N, int32_t d_in, int32_t d_out, int32_t B,
                           const void *Wbf, float *dH, hipStream_t st);

// gather.hip -------------------------------------------------------------
// `active` (may be null = every vertex): one byte per vertex, the destinations inside the batch's
// computational sub-graph for this layer.  Rows outside it are written as zeros (forward) and
// edges into them are skipped (backward: their upstream gradient is zero).
// out[i] = act( sum_{e into i} invc_e sum_b a[rel_e][b] P[src_e][b][:] + Self[i] ); out2 optional copy
// `partial`: [hv_dm.n_units][d] floats of scratch
int launch_gather_forward(const kge_partition *p, const void *P, int msg_bf16, const float *a,
                          int32_t B, int32_t d, const float *Self, int act, float *out, float *out2,
                          float *partial, const uint8_t *active, hipStream_t st);
// G = dHout * act'(Hout) (ReLU: Hout > 0)
int launch_act_backward(const float *dHout, const float *Hout, int act, int64_t n, float *G,
                        hipStream_t st);
// dP[j][b][:] = sum_{e out of j} a[rel_e][b] invc_e G[dst_e][:]
// `partial`: [hv_sm.n_units][B*d] floats of scratch
// dP rows are `ld` elements apart (B*d, or (B+1)*d when G is appended behind them)
// rel_outer_bf16.hip: C[r] += sum over relation r's runs of X[xidx ? xidx[s] : s]^T G[seg_dst[s]] (bf16 rows, fp32 C)
bool rel_outer_bf16_supported(int32_t d_in, int32_t d_out);
int launch_rel_outer_rows_bf16(const kge_partition *p, const void *X, int64_t ldx, const int32_t *xidx, const void *G,
                               int64_t ldg, int32_t d_in, int32_t d_out, float *C, hipStream_t st);
// C[g] += X^T Y_g for every d_out-wide column block g of Y's rows; the last block's sum to C_last when non-null
int launch_col_blocks_outer_bf16(const void *X, int64_t rows, const void *Y, int64_t ldy, int32_t n_groups,
                                 int32_t d_in, int32_t d_out, float *C, float *C_last, hipStream_t st);
bool gather_transpose_bf16_supported(int32_t B, int32_t d);
int launch_gather_transpose_bf16(const kge_partition *p, const void *Gbf, int64_t ldg, const float *a, int32_t B,
                                 int32_t d, void *dP, int64_t ld, float *partial, const uint8_t *active, hipStream_t st);
int launch_gather_transpose(const kge_partition *p, const float *G, const float *a, int32_t B,
                            int32_t d, void *dP, int64_t ld, int msg_bf16, float *partial,
                            const uint8_t *active, hipStream_t st);
// da[r][b] = sum_{runs (r,i)} invc sum_{j in run} <P[j][b][:], G[i][:]> ; seg_scratch [S][B] floats
// seg_scratch [S][B] floats; `partial`: [hv_seg.n_units][B] floats
int launch_coeff_grad(const kge_partition *p, const void *P, int msg_bf16, const float *G,
                      int32_t B, int32_t d, float *seg_scratch, float *partial, float *da,
                      const uint8_t *active, hipStream_t st);

// cgraph.hip: per-batch computational sub-graph ------------------------------
// flag row of layer `layer` (device pointer; -1: the first layer's input rows the batch reads), or null when cg is null
const uint8_t *kge_cgraph_layer(const kge_cgraph *cg, int32_t layer);
int kge_cgraph_check(const kge_partition *p, const kge_cgraph *cg, int32_t n_layers);

// gather.hip, run means (relation-weight order) -----------------------------
// Z[s][:] = invc_s sum_{j in run s} H[j][:]  ([S][d]; H and Z both fp32 or, with bf16 != 0, both bf16;
// sums in fp32); runs into inactive destinations get zeros; `partial`: [hv_seg.n_units][d] floats
// skip_single: runs of one edge are left unwritten (their mean is their source's row of H, see seg_zrow)
int launch_run_mean(const kge_partition *p, const void *H, int32_t d, void *Z, int bf16, float *partial,
                    const uint8_t *active, int skip_single, hipStream_t st);
// gather.hip, relation-weight order ------------------------------------------
// out[i] = act( sum over the runs (r, i) of destination i of U[run][:] + Self[i] ); U [S][d] fp32 or bf16;
// zero rows where active[i] == 0; out_bf16 (optional): a bf16 copy of the same rows; `partial`: [hv_dr.n_units][d] floats
int launch_sum_runs(const kge_partition *p, const void *U, int u_bf16, int32_t d, const float *Self, int act,
                    float *out, float *out2, void *out_bf16, float *partial, const uint8_t *active, hipStream_t st);
// out[j] = sum over the edges e out of j of (1/c_e) dZ[run(e)][:] + Self[j]; `partial`: [hv_sm.n_units][d] floats
int launch_sum_edges_out(const kge_partition *p, const void *dZ, int z_bf16, int32_t d, const float *Self,
                         float *out, float *partial, const uint8_t *active, hipStream_t st);

// gemm.hip / gemm_bf16.hip, relation-weight order -----------------------------
// Wrel[r] = sum_b a[r][b] V_b ([2R][d_in*d_out] floats)
int launch_relation_weights(const float *a, int32_t R2, int32_t B, const float *V, int64_t dd, float *Wrel,
                            hipStream_t st);
// dV[b] = sum_r a[r][b] C[r]   (overwrites dV)
// the same matrices summed in fp32 and stored as bf16 only: Wb [2R][d_in][d_out] and WbT [2R][d_out][d_in]
int launch_relation_weights_bf16(const float *a, int32_t R2, int32_t B, const float *V, int32_t d_in, int32_t d_out,
                                 void *Wb, void *WbT, hipStream_t st);
int launch_basis_grad_from_relations(const float *a, int32_t R2, int32_t B, const float *C, int64_t dd, float *dV,
                                     hipStream_t st);
// U[s] = Z[s] Wrel[rel(s)]  and  dZ[s] = G[dst(s)] Wrel[rel(s)]^T   (fp32)
int launch_apply_relation_weights(const kge_partition *p, const float *Z, const float *Wrel, int32_t d_in,
                                  int32_t d_out, float *U, hipStream_t st);
int launch_apply_relation_weights_t(const kge_partition *p, const float *G, const float *Wrel, int32_t d_in,
                                    int32_t d_out, float *dZ, hipStream_t st);
// the same two products from bf16 operands, bf16 results; Gbf rows are ldg elements apart.  zrow (may be
// NULL): Zbf is then the matrix [X; Z] and run s reads its row zrow[s]
bool rel_rows_bf16_supported(int32_t K, int32_t N);
int launch_rel_rows_bf16(const kge_partition *p, const void *A, int64_t lda, const int32_t *aidx, const void *Wk,
                         int32_t K, int32_t N, void *out, hipStream_t st, bool by_dst_slab = false);
int launch_all_rows_bf16(const void *A, int64_t rows, const void *Wk, int32_t n_groups, int32_t K, int32_t N,
                         void *out, hipStream_t st);
int launch_apply_relation_weights_bf16(const kge_partition *p, const void *Zbf, const int32_t *zrow, const void *WbT,
                                       int32_t d_in, int32_t d_out, void *U, hipStream_t st);
int launch_apply_relation_weights_t_bf16(const kge_partition *p, const void *Gbf, int64_t ldg, const void *Wb,
                                         int32_t d_in, int32_t d_out, void *dZ, hipStream_t st);

// gemm.hip, relation-weight order (coefficient gradient) ---------------------
// C[r] (d_in x d_out; [2R][d_in*d_out] floats, zeroed inside) = sum_{runs s of relation r} Z[s]^T G[seg_dst[s]]
int launch_rel_outer(const kge_partition *p, const float *Z, const float *G, int32_t d_in, int32_t d_out,
                     float *C, hipStream_t st);
// da[r][b] = <C[r], V_b>   (fp32)
int launch_coeff_contract(const kge_partition *p, const float *C, const float *V, int32_t d_in, int32_t d_out,
                          int32_t B, float *da, hipStream_t st);

// gemm_bf16.hip ----------------------------------------------------------------
// the same C from bf16 operands: Zbf [S][d_in] (or, with zrow, the matrix [X; Z] read through zrow); Gbf rows
// of d_out elements, ldg elements apart
int launch_rel_outer_bf16(const kge_partition *p, const void *Zbf, const int32_t *zrow, const void *Gbf, int64_t ldg,
                          int32_t d_in, int32_t d_out, float *C, hipStream_t st);

// sampler_score.hip --------------------------------------------------------
int launch_sample_negatives(const kge_partition *p, const int32_t *pos, int64_t n_pos, int32_t n_neg,
                            int32_t mode, uint64_t seed, uint64_t step, int32_t *neg_ent,
                            uint8_t *neg_side, hipStream_t st);
int launch_distmult(const kge_partition *p, const float *H, const float *M, int32_t d,
                    const int32_t *pos, int64_t n_pos, const int32_t *neg_ent,
                    const uint8_t *neg_side, int32_t n_neg, float *scores, float *loss, float *dH,
                    float *dM, hipStream_t st);
int launch_distmult_indexed(const kge_partition *p, kge_score_index *x, const float *H, const float *M, int32_t d,
                            const int32_t *pos, int64_t n_pos, const int32_t *neg_ent, const uint8_t *neg_side,
                            int32_t n_neg, float *scores, float *loss, float *dH, float *dM, hipStream_t st);
int launch_fill_zero(void *ptr, size_t bytes, hipStream_t st);

// dst = dropout(src) on [n_rows][d] floats (d a multiple of 4), inverted scaling, Philox mask keyed by
// (seed, step, layer, row, column); src == dst is allowed.  p == 0 copies.
int launch_dropout(const float *src, int64_t n_rows, int32_t d, float p, uint64_t seed, uint64_t step, int32_t layer,
                   float *dst, hipStream_t st);
