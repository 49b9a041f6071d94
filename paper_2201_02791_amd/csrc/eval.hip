// Link-prediction evaluation ("Evaluation Metrics" section): filtered ranks of DistMult scores (Eq. 4),
// MRR (Eq. 5) and Hits@k (Eq. 6).
//
// A query (fixed entity f, relation r, answer a) scores every entity e as  sum_k (H[f][k] M[r][k]) H[e][k]:
// with the query vectors Q = H[f] * M[r] gathered once, all scores are the product Q H^T.  That
// (queries x entities) matrix is never stored: k_eval_count computes it tile by tile on the fp32
// matrix cores and keeps, per query, only how many entries lie above / exactly at the answer's score.
// What the filtered setting removes - the known answers of the same (f, r), a handful per query - is
// scored again, one wavefront per query, by k_eval_pairs and subtracted.  Both kernels build a score
// from the same sequence of v_mfma_f32_32x32x2_f32 steps (k ascending, two k per step, fp32
// accumulator starting at zero), so a pair gets the same bits in both and the subtraction is exact.
// The same per-query kernel ranks against explicit candidate lists.
#include "common.h"

#include <algorithm>
#include <cmath>
#include <mutex>
#include <vector>

// Scratch of kge_eval_rank_all_static: device memory that lives in the library's code object, one copy
// per GPU, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the address kernels and fills may use is static_scratch_ptr()'s result.
static __device__ __align__(256) unsigned char scratch[KGE_EVAL_STATIC_BYTES];

struct kge_eval_filter {
    int device;
    int32_t n_entities, n_relations;
    // table 0: known tails of (head, rel); table 1: known heads of (tail, rel).
    // key = (fixed * R + rel) * N + other, ascending, unique; val = other
    int64_t n[2];
    int64_t *key[2];
    int32_t *val[2];
};

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// tail queries of all test triples first, then the head queries
__global__ void k_eval_queries(const int32_t *__restrict__ th, const int32_t *__restrict__ tr,
                               const int32_t *__restrict__ tt, int64_t n_test, int32_t *__restrict__ fixed,
                               int32_t *__restrict__ rel, int32_t *__restrict__ answer)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= 2 * n_test) return;
    const bool head_query = i >= n_test;
    const int64_t j = head_query ? i - n_test : i;
    fixed[i] = head_query ? tt[j] : th[j];
    rel[i] = tr[j];
    answer[i] = head_query ? th[j] : tt[j];
}

// Q[q][:] = H[fixed[q]][:] * M[rel[q]][:], one thread per 4 columns
__global__ void k_eval_qvec(const float4 *__restrict__ H, const float4 *__restrict__ M,
                            const int32_t *__restrict__ fixed, const int32_t *__restrict__ rel, int64_t nq,
                            int32_t d4, float4 *__restrict__ Q)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nq * d4) return;
    const int64_t q = t / d4;
    const int32_t c = (int32_t)(t - q * d4);
    const float4 h = H[(int64_t)fixed[q] * d4 + c], m = M[(int64_t)rel[q] * d4 + c];
    Q[t] = make_float4(h.x * m.x, h.y * m.y, h.z * m.z, h.w * m.w);
}

// Scores of one query row against one entity per column lane % 32 (ent < 0: no entity, score 0).  Every
// row of the matrix-core tile carries the same query, so each lane ends up with its column's score.
// Step s multiplies k = 2 s (lanes 0..31) and k = 2 s + 1 (lanes 32..63), as k_eval_count does.
__device__ __forceinline__ float pair_scores(const float *__restrict__ qrow, const float *__restrict__ H,
                                             int32_t ent, int32_t d, int lane)
{
    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const bool odd = (lane >> 5) != 0;
    const float *hb = H + (int64_t)(ent < 0 ? 0 : ent) * d;
    for (int32_t k0 = 0; k0 < d; k0 += 4) {
        const float4 qa = *reinterpret_cast<const float4 *>(qrow + k0);
        const float4 ba = ent >= 0 ? *reinterpret_cast<const float4 *>(hb + k0) : make_float4(0.f, 0.f, 0.f, 0.f);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(odd ? qa.y : qa.x, odd ? ba.y : ba.x, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(odd ? qa.w : qa.z, odd ? ba.w : ba.z, acc, 0, 0, 0);
    }
    return acc[0];
}

__device__ __forceinline__ int64_t lower_bound_i64(const int64_t *__restrict__ a, int64_t n, int64_t x)
{
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

struct FilterTables {
    const int64_t *key[2]; const int32_t *val[2]; int64_t n[2]; int64_t N; int32_t R;
};

// One wavefront per query: the answer's score, then the known answers of the query's (fixed entity,
// relation) 32 entities at a time.  Counts those other than the answer that score above / exactly at it.
__global__ __launch_bounds__(256) void k_eval_pairs(const float *__restrict__ Q, const float *__restrict__ H,
                                                    int32_t d, int64_t nq, int64_t n_test,
                                                    const int32_t *__restrict__ fixed, const int32_t *__restrict__ rel,
                                                    const int32_t *__restrict__ answer, FilterTables ft,
                                                    float *__restrict__ s_answer, int32_t *__restrict__ out_gt,
                                                    int32_t *__restrict__ out_eq)
{
    const int lane = threadIdx.x & 63;
    const int64_t q = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (q >= nq) return;                                    // whole wavefronts leave
    const float *qrow = Q + q * d;
    const int32_t ans = answer[q];
    float st = pair_scores(qrow, H, (lane & 31) == 0 ? ans : -1, d, lane);
    st = __shfl(st, 0, 64);
    const int side = q >= n_test ? 1 : 0;
    const int64_t base = ((int64_t)fixed[q] * ft.R + rel[q]) * ft.N;
    const int64_t lo = lower_bound_i64(ft.key[side], ft.n[side], base);
    const int64_t hi = lower_bound_i64(ft.key[side], ft.n[side], base + ft.N);
    const int32_t *list = ft.val[side];
    int gt = 0, eq = 0;
    for (int64_t b = lo; b < hi; b += 32) {                 // bounds are the same in every lane
        const int64_t i = b + (lane & 31);
        int32_t e = i < hi ? list[i] : -1;
        if (e == ans) e = -1;
        const float s = pair_scores(qrow, H, e, d, lane);
        const unsigned long long mg = __ballot(e >= 0 && s > st), me = __ballot(e >= 0 && s == st);
        gt += __popc((unsigned)mg);                         // lanes 32..63 repeat lanes 0..31
        eq += __popc((unsigned)me);
    }
    if (lane == 0) {
        s_answer[q] = st;
        out_gt[q] = gt; out_eq[q] = eq;
    }
}

// Candidate lists: one wavefront per query, LPR lanes per entity row (LPR * 4 >= min(d, 256) columns at a
// time), 64 / LPR rows side by side and UN such groups in flight.  A score is the row's fp32 dot product
// with the query vector summed in a fixed order (per lane over its column pieces, then a butterfly over the
// row's lanes), the answer's score included, so equal rows give equal scores.
template <int LPR, int NP>
__device__ __forceinline__ float row_dot(const float4 *__restrict__ hrow, const float4 (&q4)[NP], int32_t d4, int sub)
{
    float4 h[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) h[j] = sub + j * LPR < d4 ? hrow[sub + j * LPR] : make_float4(0.f, 0.f, 0.f, 0.f);
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        s = fmaf(h[j].x, q4[j].x, s); s = fmaf(h[j].y, q4[j].y, s); s = fmaf(h[j].z, q4[j].z, s); s = fmaf(h[j].w, q4[j].w, s);
    }
    return s;
}

// NP: column pieces per lane, LPR * NP * 4 >= d
template <int LPR, int NP>
__global__ __launch_bounds__(256) void k_eval_candidates(const float4 *__restrict__ Q, const float4 *__restrict__ H,
                                                         int32_t d4, int64_t nq, const int32_t *__restrict__ answer,
                                                         const int32_t *__restrict__ cand, int32_t n_cand,
                                                         int32_t *__restrict__ out_gt, int32_t *__restrict__ out_eq)
{
    constexpr int RPP = 64 / LPR, UN = NP > 2 ? 2 : 4;         // rows per pass, passes in flight
    const int lane = threadIdx.x & 63, sub = lane % LPR, grp = lane / LPR;
    const int64_t q = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (q >= nq) return;                                    // whole wavefronts leave
    float4 q4[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) q4[j] = sub + j * LPR < d4 ? Q[q * d4 + sub + j * LPR] : make_float4(0.f, 0.f, 0.f, 0.f);
    const int32_t ans = answer[q];
    auto reduce = [&](float s) {
#pragma unroll
        for (int off = LPR / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
        return s;
    };
    const float st = reduce(row_dot<LPR, NP>(H + (int64_t)ans * d4, q4, d4, sub));
    const int32_t *list = cand + q * n_cand;
    int gt = 0, eq = 0;
    for (int32_t b = 0; b < n_cand; b += RPP * UN) {         // bounds are the same in every lane
        int32_t e[UN];
        float s[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int32_t i = b + u * RPP + grp;
            e[u] = i < n_cand ? list[i] : -1;
            if (e[u] == ans) e[u] = -1;
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) s[u] = row_dot<LPR, NP>(H + (int64_t)(e[u] < 0 ? 0 : e[u]) * d4, q4, d4, sub);
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const float r = reduce(s[u]);
            if (sub == 0 && e[u] >= 0) { gt += r > st ? 1 : 0; eq += r == st ? 1 : 0; }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { gt += __shfl_xor(gt, off, 64); eq += __shfl_xor(eq, off, 64); }
    if (lane == 0) { out_gt[q] = gt; out_eq[q] = eq; }
}

// ---- all entities: 128 queries x 128 entities per tile, 4 wavefronts in a 2 x 2 grid, each with 2 x 2
// 32x32x2 accumulators; 16-deep k chunks staged through LDS k-major.  A block walks `tiles_per_block`
// consecutive entity tiles and keeps its counts in registers: one packed word per accumulator row
// (low half: entries above the answer, high half: entries equal to it).
constexpr int EBM = 128, EBN = 128, EBK = 16, EPAD = 4;
constexpr int ETR = EBK / 4, ERP = 256 / ETR, ENP = EBM / ERP;      // threads per row piece, rows per pass, passes

template <bool DUMP>
__global__ __launch_bounds__(256, 2) void k_eval_count(const float *__restrict__ Q, int64_t nq,
                                                    const float *__restrict__ H, int64_t N, int32_t d,
                                                    const float *__restrict__ s_answer, int32_t tiles_per_block,
                                                    int32_t n_col_tiles, int32_t n_row_tiles, int32_t n_col_chunks,
                                                    unsigned *__restrict__ cnt_gt,
                                                    unsigned *__restrict__ cnt_eq, float *__restrict__ dump)
{
    __shared__ __attribute__((aligned(16))) float As[EBK][EBM + EPAD];
    __shared__ __attribute__((aligned(16))) float Bs[EBK][EBN + EPAD];
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int wm = w >> 1, wn = w & 1, half = lane >> 5;
    // block id -> (query tile, chunk of entity tiles).  Workgroup i runs on XCD i % 8, each with its own L2.
    // The (query tile, chunk) space is cut into 8 x 8 patches; a patch goes to one XCD and is what that XCD
    // runs at a time (64 blocks), so its L2 holds 8 query tiles, re-read at every entity tile, and 8 streams
    // of entity tiles, each shared by 8 blocks - instead of 64 unrelated query tiles that do not fit.
    const int64_t slot = blockIdx.x / 8, xcd = blockIdx.x % 8;
    const int64_t patch = (slot / 64) * 8 + xcd;
    const int r64 = (int)(slot % 64);
    const int64_t patches_r = (n_row_tiles + 7) / 8;
    const int64_t row_tile = (patch % patches_r) * 8 + r64 % 8;
    const int64_t chunk = (patch / patches_r) * 8 + r64 / 8;
    if (row_tile >= n_row_tiles || chunk >= n_col_chunks) return;      // padding blocks of the edge patches
    const int64_t m0 = row_tile * EBM;

    // D register v of lane l of accumulator (i, j): row 32 i + 8 (v / 4) + 4 (l / 32) + v % 4, column 32 j + l % 32
    // the answers' scores of the tile's queries wait in LDS for the comparisons (rows past the end: +inf)
    __shared__ float thr_s[EBM];
    if (t < EBM) thr_s[t] = m0 + t < nq ? s_answer[m0 + t] : INFINITY;
    unsigned cnt[2][16];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) cnt[i][v] = 0u;

    const int32_t ct_beg = (int32_t)chunk * tiles_per_block;
    const int32_t ct_end = ct_beg + tiles_per_block < n_col_tiles ? ct_beg + tiles_per_block : n_col_tiles;
    const int32_t nk = (d + EBK - 1) / EBK;
    const int64_t n_it = (int64_t)(ct_end - ct_beg) * nk;      // k chunks of all tiles, in one sequence

    // operand pieces of this thread: rows r_ld + ERP * pass of the tile, 4 consecutive k from k_ld
    const int r_ld = t / ETR, k_ld = (t % ETR) * 4;
    float4 ra[ENP], rb[ENP];
    auto fetch = [&](int32_t ct, int32_t kc) {
        const int32_t k = kc * EBK + k_ld;
        const int64_t n0 = (int64_t)ct * EBN;
#pragma unroll
        for (int ps = 0; ps < ENP; ++ps) {
            const int64_t m = m0 + r_ld + ps * ERP, n = n0 + r_ld + ps * ERP;
            ra[ps] = (m < nq && k < d) ? *reinterpret_cast<const float4 *>(Q + m * d + k) : make_float4(0.f, 0.f, 0.f, 0.f);
            rb[ps] = (n < N && k < d) ? *reinterpret_cast<const float4 *>(H + n * d + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };

    floatx16 acc[2][2];
    if (n_it > 0) fetch(ct_beg, 0);
    int32_t ct = ct_beg, kc = 0;          // the chunk being multiplied
    for (int64_t it = 0; it < n_it; ++it) {
        if (kc == 0) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        }
        __syncthreads();                  // the previous chunk has been consumed
#pragma unroll
        for (int ps = 0; ps < ENP; ++ps) {
            const int r = r_ld + ps * ERP;
            As[k_ld + 0][r] = ra[ps].x; As[k_ld + 1][r] = ra[ps].y; As[k_ld + 2][r] = ra[ps].z; As[k_ld + 3][r] = ra[ps].w;
            Bs[k_ld + 0][r] = rb[ps].x; Bs[k_ld + 1][r] = rb[ps].y; Bs[k_ld + 2][r] = rb[ps].z; Bs[k_ld + 3][r] = rb[ps].w;
        }
        __syncthreads();
        const int32_t kc_next = kc + 1 < nk ? kc + 1 : 0, ct_next = kc + 1 < nk ? ct : ct + 1;
        if (it + 1 < n_it) fetch(ct_next, kc_next);      // in flight while the matrix cores work
#pragma unroll
        for (int kk = 0; kk < EBK; kk += 2) {
            const int ka = kk + half;
            const float a0 = As[ka][wm * 64 + (lane & 31)], a1 = As[ka][wm * 64 + 32 + (lane & 31)];
            const float b0 = Bs[ka][wn * 64 + (lane & 31)], b1 = Bs[ka][wn * 64 + 32 + (lane & 31)];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
        if (kc == nk - 1) {               // the tile's scores are complete: compare and count
            const int64_t n0 = (int64_t)ct * EBN;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int64_t col = n0 + wn * 64 + j * 32 + (lane & 31);
                if (col < N) {
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const float s = acc[i][j][v];
                            const float th = thr_s[wm * 64 + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3)];
                            cnt[i][v] += s > th ? 1u : (s == th ? 65536u : 0u);
                            if (DUMP) {
                                const int64_t row = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                                if (row < nq) dump[row * N + col] = s;
                            }
                        }
                }
            }
        }
        kc = kc_next; ct = ct_next;
    }
    // sum each row's packed word over the 32 lanes that share it (at most 64 entries per tile and
    // tiles_per_block <= 512: neither half overflows), then one atomic per row, wavefront and field
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            unsigned x = cnt[i][v];
#pragma unroll
            for (int off = 16; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
            const int64_t row = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
            if ((lane & 31) == 0 && row < nq) {
                if (x & 0xFFFFu) atomicAdd(cnt_gt + row, x & 0xFFFFu);
                if (x >> 16) atomicAdd(cnt_eq + row, x >> 16);
            }
        }
}

// higher = above - above among the filtered; equal = equal - equal among the filtered - the answer itself
__global__ void k_eval_finish(const unsigned *__restrict__ cnt_gt, const unsigned *__restrict__ cnt_eq,
                              const int32_t *__restrict__ sub_gt, const int32_t *__restrict__ sub_eq, int64_t nq,
                              int32_t *__restrict__ higher, int32_t *__restrict__ equal)
{
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= nq) return;
    const int64_t g = (int64_t)cnt_gt[q] - sub_gt[q], e = (int64_t)cnt_eq[q] - sub_eq[q] - 1;
    higher[q] = (int32_t)(g > 0 ? g : 0);
    equal[q] = (int32_t)(e > 0 ? e : 0);
}

struct Ks { int32_t k[8]; int32_t n; };

// one block: sums of 1 / rank and of [rank <= k] in double, fixed order
__global__ __launch_bounds__(256) void k_eval_metrics(const int32_t *__restrict__ higher,
                                                       const int32_t *__restrict__ equal, int64_t nq, Ks ks,
                                                       double *__restrict__ out)
{
    __shared__ double red[9][256];
    double s[9];
    for (int j = 0; j < 9; ++j) s[j] = 0.0;
    for (int64_t q = threadIdx.x; q < nq; q += 256) {
        const double r = 1.0 + (double)higher[q] + 0.5 * (double)equal[q];
        s[0] += 1.0 / r;
        for (int j = 0; j < ks.n; ++j) s[1 + j] += r <= (double)ks.k[j] ? 1.0 : 0.0;
    }
    for (int j = 0; j <= ks.n; ++j) red[j][threadIdx.x] = s[j];
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off)
            for (int j = 0; j <= ks.n; ++j) red[j][threadIdx.x] += red[j][threadIdx.x + off];
        __syncthreads();
    }
    if ((int)threadIdx.x <= ks.n) out[threadIdx.x] = nq > 0 ? red[threadIdx.x][0] / (double)nq : 0.0;
}

struct EvalWs {
    size_t off_fixed, off_rel, off_answer, off_Q, off_s, off_sub_gt, off_sub_eq, off_cnt_gt, off_cnt_eq, total;
};

EvalWs eval_layout(int64_t nq, int32_t d)
{
    EvalWs w;
    size_t cur = 0;
    const size_t n = (size_t)(nq > 0 ? nq : 1);
    auto take = [&](size_t bytes) { size_t o = cur; cur = align_up(cur + bytes, 256); return o; };
    w.off_fixed = take(n * 4); w.off_rel = take(n * 4); w.off_answer = take(n * 4);
    w.off_Q = take(n * (size_t)d * 4); w.off_s = take(n * 4);
    w.off_sub_gt = take(n * 4); w.off_sub_eq = take(n * 4);
    w.off_cnt_gt = take(n * 4); w.off_cnt_eq = take(n * 4);
    w.total = cur;
    return w;
}

int check_model(const float *H, int64_t n_entities, int32_t d, const float *M, int32_t n_relations)
{
    KGE_REQUIRE(H && M, KGE_EINVAL, "H or M is NULL");
    KGE_REQUIRE(n_entities > 0 && n_entities <= 0x7FFFFFFFll && n_relations > 0, KGE_EINVAL,
                "n_entities must be in [1, 2^31) and n_relations positive");
    KGE_REQUIRE(d > 0 && d % 4 == 0 && d <= 1024, KGE_EINVAL, "d must be a multiple of 4 in [4, 1024]");
    KGE_REQUIRE(((uintptr_t)H % 16) == 0 && ((uintptr_t)M % 16) == 0, KGE_EINVAL, "H and M must be 16-byte aligned");
    return KGE_OK;
}

int check_ws(void *workspace, size_t ws_bytes, int64_t nq, int32_t d, EvalWs *w)
{
    *w = eval_layout(nq, d);
    KGE_REQUIRE(workspace && ((uintptr_t)workspace % 256) == 0, KGE_EINVAL, "workspace must be 256-byte aligned");
    KGE_REQUIRE(ws_bytes >= w->total, KGE_ENOMEM, "workspace has %zu bytes, %zu needed", ws_bytes, w->total);
    return KGE_OK;
}

int launch_count(const float *Q, int64_t nq, const float *H, int64_t N, int32_t d, const float *s_answer,
                 unsigned *cnt_gt, unsigned *cnt_eq, float *dump, hipStream_t st)
{
    const int64_t row_tiles = cdiv(nq, EBM), col_tiles = cdiv(N, EBN);
    // about 4096 blocks (16 per compute unit) when there is that much work, the chunk count a multiple of
    // the patch width when it exceeds it; a block's packed counters hold 512 tiles
    int64_t col_chunks = cdiv(4096, row_tiles);
    if (col_chunks > 8) col_chunks = cdiv(col_chunks, 8) * 8;
    if (col_chunks > col_tiles) col_chunks = col_tiles;
    int64_t tpb = cdiv(col_tiles, col_chunks);
    if (tpb > 512) tpb = 512;
    col_chunks = cdiv(col_tiles, tpb);
    const int64_t patches = cdiv(row_tiles, 8) * cdiv(col_chunks, 8);
    const int64_t blocks = cdiv(patches, 8) * 8 * 64;        // whole rounds of 8 patches, 64 blocks each
    KGE_REQUIRE(blocks <= 0x7FFFFFFFll, KGE_ERANGE, "evaluation grid too large");
    if (dump)
        k_eval_count<true><<<(unsigned)blocks, 256, 0, st>>>(Q, nq, H, N, d, s_answer, (int32_t)tpb, (int32_t)col_tiles,
                                                            (int32_t)row_tiles, (int32_t)col_chunks, cnt_gt, cnt_eq, dump);
    else
        k_eval_count<false><<<(unsigned)blocks, 256, 0, st>>>(Q, nq, H, N, d, s_answer, (int32_t)tpb, (int32_t)col_tiles,
                                                             (int32_t)row_tiles, (int32_t)col_chunks, cnt_gt, cnt_eq, nullptr);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

int rank_all(const kge_eval_filter *f, const float *H, int64_t N, int32_t d, const float *M, int32_t R,
             const int32_t *test_h, const int32_t *test_r, const int32_t *test_t, int64_t n_test, void *workspace,
             size_t ws_bytes, int32_t *higher, int32_t *equal, float *dump, float *dump_answer, hipStream_t st)
{
    int rc = check_model(H, N, d, M, R);
    if (rc != KGE_OK) return rc;
    KGE_REQUIRE(n_test >= 0 && n_test <= 0x3FFFFFFFll, KGE_EINVAL, "n_test out of range");
    KGE_REQUIRE(!f || (f->n_entities == N && f->n_relations == R), KGE_EINVAL,
                "the filter was built for other entity / relation counts");
    const int64_t nq = 2 * n_test;
    EvalWs w;
    rc = check_ws(workspace, ws_bytes, nq, d, &w);
    if (rc != KGE_OK) return rc;
    if (n_test == 0) return KGE_OK;
    KGE_REQUIRE(test_h && test_r && test_t && (dump || (higher && equal)), KGE_EINVAL, "NULL array");
    char *ws = (char *)workspace;
    int32_t *fixed = (int32_t *)(ws + w.off_fixed), *rel = (int32_t *)(ws + w.off_rel), *answer = (int32_t *)(ws + w.off_answer);
    float *Q = (float *)(ws + w.off_Q), *s = (float *)(ws + w.off_s);
    int32_t *sub_gt = (int32_t *)(ws + w.off_sub_gt), *sub_eq = (int32_t *)(ws + w.off_sub_eq);
    unsigned *cnt_gt = (unsigned *)(ws + w.off_cnt_gt), *cnt_eq = (unsigned *)(ws + w.off_cnt_eq);
    {
        KGE_PROF("eval_queries", st);
        k_eval_queries<<<(unsigned)cdiv(nq, 256), 256, 0, st>>>(test_h, test_r, test_t, n_test, fixed, rel, answer);
        KGE_LAUNCH_CHECK();
        k_eval_qvec<<<(unsigned)cdiv(nq * (d / 4), 256), 256, 0, st>>>((const float4 *)H, (const float4 *)M, fixed, rel, nq,
                                                                      d / 4, (float4 *)Q);
        KGE_LAUNCH_CHECK();
    }
    rc = launch_fill_zero(cnt_gt, (size_t)nq * 4, st);
    if (rc != KGE_OK) return rc;
    rc = launch_fill_zero(cnt_eq, (size_t)nq * 4, st);
    if (rc != KGE_OK) return rc;
    {
        KGE_PROF("eval_pairs", st);
        FilterTables ft;
        for (int sde = 0; sde < 2; ++sde) {
            ft.key[sde] = f ? f->key[sde] : nullptr; ft.val[sde] = f ? f->val[sde] : nullptr; ft.n[sde] = f ? f->n[sde] : 0;
        }
        ft.N = N; ft.R = R;
        k_eval_pairs<<<(unsigned)cdiv(nq, 4), 256, 0, st>>>(Q, H, d, nq, n_test, fixed, rel, answer, ft,
                                                           dump_answer ? dump_answer : s, sub_gt, sub_eq);
        KGE_LAUNCH_CHECK();
    }
    {
        KGE_PROF("eval_count", st);
        rc = launch_count(Q, nq, H, N, d, dump_answer ? dump_answer : s, cnt_gt, cnt_eq, dump, st);
        if (rc != KGE_OK) return rc;
    }
    if (higher && equal) {
        k_eval_finish<<<(unsigned)cdiv(nq, 256), 256, 0, st>>>(cnt_gt, cnt_eq, sub_gt, sub_eq, nq, higher, equal);
        KGE_LAUNCH_CHECK();
    }
    return KGE_OK;
}

}  // namespace

extern "C" int kge_eval_filter_create(const int32_t *head, const int32_t *rel, const int32_t *tail, int64_t n_known,
                                      int32_t n_entities, int32_t n_relations, kge_eval_filter **out)
{
    KGE_REQUIRE(out, KGE_EINVAL, "NULL argument");
    *out = nullptr;
    KGE_REQUIRE(n_known >= 0 && (n_known == 0 || (head && rel && tail)), KGE_EINVAL, "NULL triple arrays");
    KGE_REQUIRE(n_entities > 0 && n_relations > 0, KGE_EINVAL, "n_entities and n_relations must be positive");
    KGE_REQUIRE((double)n_entities * (double)n_relations * (double)n_entities < 9.0e18, KGE_ERANGE,
                "entity and relation counts too large for a 64-bit key");
    for (int64_t i = 0; i < n_known; ++i)
        KGE_REQUIRE(head[i] >= 0 && head[i] < n_entities && tail[i] >= 0 && tail[i] < n_entities && rel[i] >= 0 &&
                        rel[i] < n_relations, KGE_ERANGE, "known triple %lld has an id out of range", (long long)i);
    kge_eval_filter *f = new kge_eval_filter();
    f->n_entities = n_entities; f->n_relations = n_relations;
    for (int sde = 0; sde < 2; ++sde) { f->key[sde] = nullptr; f->val[sde] = nullptr; f->n[sde] = 0; }
    hipError_t e = hipGetDevice(&f->device);
    std::vector<int64_t> keys((size_t)n_known);
    std::vector<int32_t> vals;
    for (int sde = 0; sde < 2 && e == hipSuccess; ++sde) {
        const int32_t *fx = sde ? tail : head, *ot = sde ? head : tail;
        for (int64_t i = 0; i < n_known; ++i)
            keys[(size_t)i] = ((int64_t)fx[i] * n_relations + rel[i]) * n_entities + ot[i];
        std::sort(keys.begin(), keys.end());
        const size_t n = (size_t)(std::unique(keys.begin(), keys.end()) - keys.begin());
        vals.resize(n);
        for (size_t i = 0; i < n; ++i) vals[i] = (int32_t)(keys[i] % n_entities);
        f->n[sde] = (int64_t)n;
        e = hipMalloc((void **)&f->key[sde], (n ? n : 1) * sizeof(int64_t));
        if (e == hipSuccess) e = hipMalloc((void **)&f->val[sde], (n ? n : 1) * sizeof(int32_t));
        if (e == hipSuccess && n) e = hipMemcpy(f->key[sde], keys.data(), n * sizeof(int64_t), hipMemcpyHostToDevice);
        if (e == hipSuccess && n) e = hipMemcpy(f->val[sde], vals.data(), n * sizeof(int32_t), hipMemcpyHostToDevice);
        keys.resize((size_t)n_known);
    }
    if (e != hipSuccess) {
        kge_set_error("building the evaluation filter failed: %s", hipGetErrorString(e));
        kge_eval_filter_destroy(f);
        return KGE_EHIP;
    }
    *out = f;
    return KGE_OK;
}

extern "C" void kge_eval_filter_destroy(kge_eval_filter *f)
{
    if (!f) return;
    for (int sde = 0; sde < 2; ++sde) {
        if (f->key[sde]) (void)hipFree(f->key[sde]);
        if (f->val[sde]) (void)hipFree(f->val[sde]);
    }
    delete f;
}

extern "C" size_t kge_eval_workspace_bytes(int64_t n_queries, int32_t d)
{
    if (n_queries < 0 || d <= 0) { kge_set_error("negative query count or bad d"); return 0; }
    return eval_layout(n_queries, d).total;
}

extern "C" int kge_eval_rank_all(const kge_eval_filter *filter, const float *H, int64_t n_entities, int32_t d,
                                 const float *M, int32_t n_relations, const int32_t *test_h, const int32_t *test_r,
                                 const int32_t *test_t, int64_t n_test, void *workspace, size_t ws_bytes,
                                 int32_t *higher, int32_t *equal, void *stream)
{
    KGE_REQUIRE(n_test <= 0 || (higher && equal), KGE_EINVAL, "higher or equal is NULL");
    return rank_all(filter, H, n_entities, d, M, n_relations, test_h, test_r, test_t, n_test, workspace, ws_bytes,
                    higher, equal, nullptr, nullptr, (hipStream_t)stream);
}

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices];      // per device: where that GPU's copy of `scratch` lives

// Address of the current device's copy of `scratch`, looked up once per device with that device current.
int static_scratch_ptr(void **out)
{
    int dev = -1;
    KGE_HIP(hipGetDevice(&dev));
    KGE_REQUIRE(dev >= 0 && dev < kMaxDevices, KGE_EINVAL, "device index %d is outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        KGE_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        KGE_REQUIRE(ptr && ((uintptr_t)ptr % 256) == 0, KGE_EHIP, "the static scratch array has no usable device address");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return KGE_OK;
}
}  // namespace

extern "C" int kge_eval_rank_all_static(const kge_eval_filter *filter, const float *H, int64_t n_entities, int32_t d,
                                        const float *M, int32_t n_relations, const int32_t *test_h,
                                        const int32_t *test_r, const int32_t *test_t, int64_t n_test,
                                        int32_t *higher, int32_t *equal, void *stream)
{
    KGE_REQUIRE(n_test <= 0 || (higher && equal), KGE_EINVAL, "higher or equal is NULL");
    KGE_REQUIRE(n_test >= 0 && n_test <= 0x3FFFFFFFll && d > 0, KGE_EINVAL, "n_test or d out of range");
    const size_t need = eval_layout(2 * n_test, d).total;
    KGE_REQUIRE(need <= (size_t)KGE_EVAL_STATIC_BYTES, KGE_ENOMEM,
                "%lld test triples of width %d need %zu bytes of scratch; the static buffer holds %zu "
                "(use kge_eval_rank_all with a workspace)", (long long)n_test, d, need, (size_t)KGE_EVAL_STATIC_BYTES);
    void *ptr = nullptr;
    int rc = static_scratch_ptr(&ptr);
    if (rc != KGE_OK) return rc;
    return rank_all(filter, H, n_entities, d, M, n_relations, test_h, test_r, test_t, n_test, ptr,
                    (size_t)KGE_EVAL_STATIC_BYTES, higher, equal, nullptr, nullptr, (hipStream_t)stream);
}

extern "C" int kge_eval_debug_scores(const float *H, int64_t n_entities, int32_t d, const float *M, int32_t n_relations,
                                     const int32_t *test_h, const int32_t *test_r, const int32_t *test_t, int64_t n_test,
                                     void *workspace, size_t ws_bytes, float *scores, float *answer_score, void *stream)
{
    KGE_REQUIRE(scores && answer_score, KGE_EINVAL, "scores or answer_score is NULL");
    return rank_all(nullptr, H, n_entities, d, M, n_relations, test_h, test_r, test_t, n_test, workspace, ws_bytes,
                    nullptr, nullptr, scores, answer_score, (hipStream_t)stream);
}

extern "C" int kge_eval_rank_candidates(const float *H, int64_t n_entities, int32_t d, const float *M,
                                        int32_t n_relations, const int32_t *fixed, const int32_t *rel,
                                        const int32_t *answer, int64_t n_queries, const int32_t *cand, int32_t n_cand,
                                        void *workspace, size_t ws_bytes, int32_t *higher, int32_t *equal, void *stream)
{
    int rc = check_model(H, n_entities, d, M, n_relations);
    if (rc != KGE_OK) return rc;
    KGE_REQUIRE(n_queries >= 0 && n_queries <= 0x7FFFFFFFll && n_cand >= 0, KGE_EINVAL, "negative count");
    EvalWs w;
    rc = check_ws(workspace, ws_bytes, n_queries, d, &w);
    if (rc != KGE_OK) return rc;
    if (n_queries == 0) return KGE_OK;
    KGE_REQUIRE(fixed && rel && answer && higher && equal && (n_cand == 0 || cand), KGE_EINVAL, "NULL array");
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    float *Q = (float *)(ws + w.off_Q);
    {
        KGE_PROF("eval_queries", st);
        k_eval_qvec<<<(unsigned)cdiv(n_queries * (d / 4), 256), 256, 0, st>>>((const float4 *)H, (const float4 *)M, fixed, rel,
                                                                             n_queries, d / 4, (float4 *)Q);
        KGE_LAUNCH_CHECK();
    }
    KGE_PROF("eval_cand", st);
    const unsigned grid = (unsigned)cdiv(n_queries, 4);
    const int32_t d4 = d / 4;
    const float4 *Q4 = (const float4 *)Q, *H4 = (const float4 *)H;
    if (d4 <= 8) k_eval_candidates<8, 1><<<grid, 256, 0, st>>>(Q4, H4, d4, n_queries, answer, cand, n_cand, higher, equal);
    else if (d4 <= 16) k_eval_candidates<16, 1><<<grid, 256, 0, st>>>(Q4, H4, d4, n_queries, answer, cand, n_cand, higher, equal);
    else if (d4 <= 32) k_eval_candidates<32, 1><<<grid, 256, 0, st>>>(Q4, H4, d4, n_queries, answer, cand, n_cand, higher, equal);
    else if (d4 <= 64) k_eval_candidates<64, 1><<<grid, 256, 0, st>>>(Q4, H4, d4, n_queries, answer, cand, n_cand, higher, equal);
    else if (d4 <= 128) k_eval_candidates<64, 2><<<grid, 256, 0, st>>>(Q4, H4, d4, n_queries, answer, cand, n_cand, higher, equal);
    else k_eval_candidates<64, 4><<<grid, 256, 0, st>>>(Q4, H4, d4, n_queries, answer, cand, n_cand, higher, equal);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

extern "C" int kge_eval_metrics(const int32_t *higher, const int32_t *equal, int64_t n_queries, const int32_t *ks,
                                int32_t n_ks, double *out, void *stream)
{
    KGE_REQUIRE(out && n_queries >= 0 && (n_queries == 0 || (higher && equal)), KGE_EINVAL, "NULL array or negative count");
    KGE_REQUIRE(n_ks >= 0 && n_ks <= 8 && (n_ks == 0 || ks), KGE_EINVAL, "n_ks must be in [0, 8]");
    KGE_REQUIRE(((uintptr_t)out % 8) == 0, KGE_EINVAL, "out must be 8-byte aligned");
    Ks k;
    k.n = n_ks;
    for (int j = 0; j < 8; ++j) k.k[j] = j < n_ks ? ks[j] : 0;
    k_eval_metrics<<<1, 256, 0, (hipStream_t)stream>>>(higher, equal, n_queries, k, out);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}
