// In-partition negative sampling (Sec. 2.1 corruption under the constraint of Sec. 3.3.1)
// with a counter-based generator, and the fused DistMult score (Eq. 4) + cross-entropy loss
// (Eq. 3) + gradient kernel.
#include <string.h>

#include "common.h"
#include "sort_scan.h"

// Scratch of the atomic-free form of the scoring call, allocated once per trainer for a largest batch.
// An "occurrence" is one row that a scored triple adds into the embedding gradient: for positive q (of
// n_pos) slot k < n_neg is its k-th negative (the row goes to the corrupting entity), slot n_neg its head
// and slot n_neg + 1 its tail (rows summed over the positive's own triples); occurrence id = q (n_neg + 2) + slot.
struct kge_score_index {
    int device;
    int64_t n_vert, max_pos, max_occ;
    int32_t max_neg, d;
    uint32_t *keys[2], *vals[2];   // [max_occ] entity of each occurrence / occurrence id; ping-pong buffers of the sort
    uint32_t *sort_ws;             // radix_scratch_words(max_occ)
    int32_t *ent_ptr;              // [N + 1] range of each entity in the sorted occurrence list
    uint32_t *slot_of;             // [max_occ] position of each occurrence in the list sorted by entity
    int4 *recs;                    // [max_occ] in sorted order, what the occurrence adds: x = the positive's entity on the
                                   // other side (a negative: its row of H, times M_r, is what the delta multiplies) or
                                   // -1 - (row of rows[]) for a positive's own end; y = relation; z = bits of delta
    uint32_t *pkeys[2], *pvals[2]; // [max_pos] the batch's positives sorted by relation (ping-pong buffers)
    float *rows;                   // [2 max_pos][d] per positive q: the summed rows for its head (2q) and its tail (2q+1)
    float *dm_part;                // [KGE_SCORE_MAX_BLOCKS][d] one partial relation-gradient row per scoring block,
    int32_t *dm_rel;               // [KGE_SCORE_MAX_BLOCKS] its relation (-1: none, the block used atomics),
    float *loss_part;              // [KGE_SCORE_MAX_BLOCKS] and the block's loss terms
};

namespace {

// Philox4x32 with 10 rounds (Salmon et al., SC'11): a keyed bijection of a 128-bit counter.
// Each round multiplies words 0 and 2 by fixed odd constants; the low halves pass through,
// the high halves are xored with the other words and the round key; the key is bumped by
// two Weyl constants after every round.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t &x0, uint32_t &x1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    x0 = c0; x1 = c1;
}

// One thread per (positive, slot).
__global__ void k_sample_negatives(const int32_t *__restrict__ cand, uint32_t n_cand,
                                   const int32_t *__restrict__ pos, int64_t n_pos, int32_t n_neg,
                                   int32_t mode, uint32_t seed_lo, uint32_t seed_hi, uint32_t step_lo,
                                   uint32_t step_hi, int32_t *__restrict__ neg_ent,
                                   uint8_t *__restrict__ neg_side)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_pos * n_neg) return;
    const int64_t q = idx / n_neg;
    const uint32_t k = (uint32_t)(idx - q * n_neg);
    uint32_t x0, x1;
    philox4x32_10((uint32_t)pos[q], k, step_lo, step_hi, seed_lo, seed_hi, x0, x1);
    neg_ent[idx] = cand[__umulhi(x0, n_cand)];
    neg_side[idx] = (uint8_t)((mode == KGE_NEG_HEAD_OR_TAIL && x1 >= 0x80000000u) ? 1 : 0);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ float softplus_f(float x) { return x > 0.f ? x + log1pf(expf(-x)) : log1pf(expf(x)); }
__device__ __forceinline__ float sigmoid_f(float x)
{
    return x >= 0.f ? 1.f / (1.f + expf(-x)) : expf(x) / (1.f + expf(x));
}

constexpr int KGE_SCORE_MAX_BLOCKS = 4096;   // the scoring kernel runs at most 16384 wavefronts, four per block
constexpr int DM_WAVES = 16;     // wavefronts per block of the scoring kernel

// Each wavefront takes a contiguous chunk of positives; for each, lane l holds elements
// l, l+64, ... of a row (NCH per lane).  The positive's h_s, h_t and M_r stay in registers;
// every negative costs one row read and one atomic row update; the gradients of the shared
// rows are accumulated in registers and flushed once per positive.  The relation-diagonal
// gradient and the loss stay in registers across the chunk (flushed when the relation changes)
// and are combined across the block's wavefronts in LDS when they all end on the same relation,
// so that few relations (down to one) do not serialise on the same atomics.
template <int NCH>
__global__ __launch_bounds__(64 * DM_WAVES) void k_distmult(
    const float *__restrict__ H, const float *__restrict__ M, int32_t d,
    const int32_t *__restrict__ core_h, const int32_t *__restrict__ core_r,
    const int32_t *__restrict__ core_t, const int32_t *__restrict__ pos, int64_t n_pos, int32_t per_wave,
    const int32_t *__restrict__ neg_ent, const uint8_t *__restrict__ neg_side, int32_t n_neg,
    uint32_t n_vert, uint32_t n_core, uint32_t *__restrict__ bad,
    float inv_T, float *__restrict__ scores, float *__restrict__ loss, float *__restrict__ dH,
    float *__restrict__ dM)
{
    __shared__ float red[DM_WAVES][64 * NCH];
    __shared__ int32_t rel_of_wave[DM_WAVES];
    __shared__ float loss_of_wave[DM_WAVES];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t wave_id = (int64_t)blockIdx.x * DM_WAVES + w;
    const int64_t q_beg = wave_id * per_wave;
    const int64_t q_end = q_beg + per_wave < n_pos ? q_beg + per_wave : n_pos;

    float aM[NCH];
#pragma unroll
    for (int u = 0; u < NCH; ++u) aM[u] = 0.f;
    int32_t r_cur = -1;
    float lsum = 0.f;

    for (int64_t q = q_beg; q < q_end; ++q) {
        uint32_t c = (uint32_t)pos[q];
        if (c >= n_core) {                // an index outside the partition never becomes an address: counted, replaced
            c = 0;
            if (lane == 0) atomicAdd(bad, 1u);
        }
        const int32_t s = core_h[c], r = core_r[c], t = core_t[c];
        if (r != r_cur) {                 // uniform: flush the relation gradient of the finished run
            if (r_cur >= 0) {
#pragma unroll
                for (int u = 0; u < NCH; ++u) {
                    const int k = lane + 64 * u;
                    if (k < d) unsafeAtomicAdd(&dM[(int64_t)r_cur * d + k], aM[u]);
                    aM[u] = 0.f;
                }
            }
            r_cur = r;
        }
        float hs[NCH], ht[NCH], mr[NCH], aS[NCH], aT[NCH];
#pragma unroll
        for (int u = 0; u < NCH; ++u) {
            const int k = lane + 64 * u;
            const bool ok = k < d;
            hs[u] = ok ? H[(int64_t)s * d + k] : 0.f;
            ht[u] = ok ? H[(int64_t)t * d + k] : 0.f;
            mr[u] = ok ? M[(int64_t)r * d + k] : 0.f;
            aS[u] = aT[u] = 0.f;
        }
        {   // the positive
            float g = 0.f;
#pragma unroll
            for (int u = 0; u < NCH; ++u) g = fmaf(hs[u] * mr[u], ht[u], g);
            g = wave_sum(g);
            if (scores && lane == 0) scores[q * (1 + n_neg)] = g;
            lsum += softplus_f(-g);
            const float delta = (sigmoid_f(g) - 1.f) * inv_T;
#pragma unroll
            for (int u = 0; u < NCH; ++u) {
                aS[u] = fmaf(delta * mr[u], ht[u], aS[u]);
                aT[u] = fmaf(delta * mr[u], hs[u], aT[u]);
                aM[u] = fmaf(delta * hs[u], ht[u], aM[u]);
            }
        }
        // negatives, four rows in flight
        for (int32_t k0 = 0; k0 < n_neg; k0 += 4) {
            int32_t ent[4]; int side[4]; float hx[4][NCH];
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                const bool ok = k0 + z < n_neg;
                ent[z] = ok ? neg_ent[q * n_neg + k0 + z] : 0;
                if ((uint32_t)ent[z] >= n_vert) {
                    ent[z] = 0;
                    if (lane == 0) atomicAdd(bad, 1u);
                }
                side[z] = ok ? (int)neg_side[q * n_neg + k0 + z] : 0;
#pragma unroll
                for (int u = 0; u < NCH; ++u) {
                    const int k = lane + 64 * u;
                    hx[z][u] = (ok && k < d) ? H[(int64_t)ent[z] * d + k] : 0.f;
                }
            }
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                if (k0 + z >= n_neg) break;
                // the corrupted entity is scored against M_r * h_t (head replaced) or M_r * h_s
                float g = 0.f;
#pragma unroll
                for (int u = 0; u < NCH; ++u) g = fmaf(hx[z][u] * mr[u], side[z] ? ht[u] : hs[u], g);
                g = wave_sum(g);
                if (scores && lane == 0) scores[q * (1 + n_neg) + 1 + k0 + z] = g;
                lsum += softplus_f(g);
                const float delta = sigmoid_f(g) * inv_T;
#pragma unroll
                for (int u = 0; u < NCH; ++u) {
                    const int k = lane + 64 * u;
                    const float other = side[z] ? ht[u] : hs[u];
                    if (k < d) unsafeAtomicAdd(&dH[(int64_t)ent[z] * d + k], delta * mr[u] * other);
                    if (side[z]) aT[u] = fmaf(delta * mr[u], hx[z][u], aT[u]);
                    else aS[u] = fmaf(delta * mr[u], hx[z][u], aS[u]);
                    aM[u] = fmaf(delta * hx[z][u], other, aM[u]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < NCH; ++u) {
            const int k = lane + 64 * u;
            if (k < d) {
                unsafeAtomicAdd(&dH[(int64_t)s * d + k], aS[u]);
                unsafeAtomicAdd(&dH[(int64_t)t * d + k], aT[u]);
            }
        }
    }
    // combine across the block
    if (lane == 0) { rel_of_wave[w] = r_cur; loss_of_wave[w] = lsum; }
#pragma unroll
    for (int u = 0; u < NCH; ++u) red[w][lane + 64 * u] = aM[u];
    __syncthreads();
    bool same = true;
    int32_t r_any = -1;
#pragma unroll
    for (int k = 0; k < DM_WAVES; ++k) {
        const int32_t rk = rel_of_wave[k];
        if (rk >= 0) { if (r_any < 0) r_any = rk; else if (rk != r_any) same = false; }
    }
    if (same) {
        if (r_any >= 0 && w == 0) {
#pragma unroll
            for (int u = 0; u < NCH; ++u) {
                const int k = lane + 64 * u;
                float t = 0.f;
#pragma unroll
                for (int x = 0; x < DM_WAVES; ++x) t += red[x][k];
                if (k < d) unsafeAtomicAdd(&dM[(int64_t)r_any * d + k], t);
            }
        }
    } else if (r_cur >= 0) {
#pragma unroll
        for (int u = 0; u < NCH; ++u) {
            const int k = lane + 64 * u;
            if (k < d) unsafeAtomicAdd(&dM[(int64_t)r_cur * d + k], aM[u]);
        }
    }
    if (threadIdx.x == 0) {
        float t = 0.f;
#pragma unroll
        for (int x = 0; x < DM_WAVES; ++x) t += loss_of_wave[x];
        unsafeAtomicAdd(loss, t * inv_T);
    }
}

// ---------------------------------------------------------------- atomic-free form
// keys[o] = the entity whose gradient row occurrence o adds to; vals[o] = o
__global__ void k_score_keys(const int32_t *__restrict__ core_h, const int32_t *__restrict__ core_t,
                             const int32_t *__restrict__ pos, int64_t n_pos, const int32_t *__restrict__ neg_ent,
                             int32_t n_neg, uint32_t n_vert, uint32_t n_core, uint32_t *__restrict__ keys,
                             uint32_t *__restrict__ vals, uint32_t *__restrict__ bad)
{
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int32_t per = n_neg + 2;
    if (o >= n_pos * per) return;
    const int64_t q = o / per;
    const int32_t slot = (int32_t)(o - q * per);
    uint32_t e;
    if (slot < n_neg) {
        e = (uint32_t)neg_ent[q * n_neg + slot];
    } else {
        uint32_t c = (uint32_t)pos[q];
        if (c >= n_core) { c = 0; if (slot == n_neg) atomicAdd(bad, 1u); }
        e = (uint32_t)(slot == n_neg ? core_h[c] : core_t[c]);
    }
    // an id outside the partition never becomes an address: it is counted and replaced by vertex 0
    if (e >= n_vert) { e = 0; atomicAdd(bad, 1u); }
    keys[o] = e;
    vals[o] = (uint32_t)o;
}

// keys[q] = relation of positive q, vals[q] = q
__global__ void k_score_rel_keys(const int32_t *__restrict__ core_r, const int32_t *__restrict__ pos, int64_t n_pos,
                                 uint32_t n_core, uint32_t *__restrict__ keys, uint32_t *__restrict__ vals)
{
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= n_pos) return;
    uint32_t c = (uint32_t)pos[q];
    if (c >= n_core) c = 0;
    keys[q] = (uint32_t)core_r[c];
    vals[q] = (uint32_t)q;
}

// slot_of[sorted[i]] = i
__global__ void k_invert_permutation(const uint32_t *__restrict__ sorted, int64_t n, uint32_t *__restrict__ slot_of)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) slot_of[sorted[i]] = (uint32_t)i;
}

__device__ __forceinline__ float dot4(const float4 a, const float4 b, const float4 c)
{
    return fmaf(a.x * b.x, c.x, fmaf(a.y * b.y, c.y, fmaf(a.z * b.z, c.z, a.w * b.w * c.w)));
}

// Sums of eight per-lane values over the 64 lanes at once: the halves of the wavefront trade the four values
// each does not keep, then quarters two, then eighths one (7 exchanges), and three more steps finish the sum
// inside every group of 8 lanes - 10 exchanges instead of 48.  Returns the total of v[z] in the lanes whose bits
// 5, 4, 3 spell z (lane8_of(z) is the first of them).
__device__ __forceinline__ float reduce8(const float v[8], int lane)
{
    float a[4], b[2];
    bool up = (lane & 32) != 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = (up ? v[i + 4] : v[i]) + __shfl_xor(up ? v[i] : v[i + 4], 32, 64);
    up = (lane & 16) != 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) b[i] = (up ? a[i + 2] : a[i]) + __shfl_xor(up ? a[i] : a[i + 2], 16, 64);
    up = (lane & 8) != 0;
    float c = (up ? b[1] : b[0]) + __shfl_xor(up ? b[0] : b[1], 8, 64);
    c += __shfl_xor(c, 4, 64);
    c += __shfl_xor(c, 2, 64);
    c += __shfl_xor(c, 1, 64);
    return c;
}
__device__ __forceinline__ constexpr int lane8_of(int z) { return ((z & 4) ? 32 : 0) + ((z & 2) ? 16 : 0) + ((z & 1) ? 8 : 0); }
__device__ __forceinline__ float lane_value(float x, int src_lane)      // src_lane: a compile-time constant
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), src_lane));
}

// softplus(g) and sigmoid(g) from one exponential: e = exp(-|g|)
__device__ __forceinline__ void softplus_sigmoid(float g, float &sp, float &sg)
{
    const float e = expf(-fabsf(g));
    sp = fmaxf(g, 0.f) + log1pf(e);
    sg = (g >= 0.f ? 1.f : e) / (1.f + e);
}

constexpr int DS_WAVES = 4;      // wavefronts per block of the scoring kernel below

// Scores, loss, relation gradient, and per triple what the gather below needs: delta and the row it multiplies.
// One wavefront per chunk of positives; lane l holds columns 4l .. 4l+3 (and 256 + 4l .. for NV = 2) of every
// row as one 16-byte load.  The positive's h_s, h_t and M_r stay in registers.  The corrupting entities of a
// positive are fetched by one coalesced load (a lane each) and handed out with readlane, so no row address
// waits on a second memory access; the negatives' rows arrive eight at a time in two register buffers - the
// next eight are in flight while the current eight are scored.  Their eight scores are summed across the lanes
// together (reduce8), and the loss terms and deltas of the eight are computed once, each in its own lanes.
// Nothing is added into dH here.  The wavefront walks the positives in the order `perm` gives (sorted by relation:
// the relation gradient then stays in registers over runs of positives and few atomics meet on one row), and
// writes each triple's record where the entity-sorted list has it (slot_of).
template <int NV>
__global__ __launch_bounds__(64 * DS_WAVES) void k_distmult_score(
    const float4 *__restrict__ H, const float4 *__restrict__ M, int32_t d4,
    const int32_t *__restrict__ core_h, const int32_t *__restrict__ core_r,
    const int32_t *__restrict__ core_t, const int32_t *__restrict__ pos, const uint32_t *__restrict__ perm,
    int64_t n_pos, int32_t per_wave,
    const int32_t *__restrict__ neg_ent, const uint8_t *__restrict__ neg_side, int32_t n_neg,
    uint32_t n_vert, uint32_t n_core,
    float inv_T, float *__restrict__ scores, float *__restrict__ dM,
    const uint32_t *__restrict__ slot_of, int4 *__restrict__ recs, float4 *__restrict__ rows,
    float4 *__restrict__ dm_part, int32_t *__restrict__ dm_rel, float *__restrict__ loss_part)
{
    __shared__ float loss_of_wave[DS_WAVES];
    __shared__ int32_t rel_of_wave[DS_WAVES];
    __shared__ float4 part_of_wave[DS_WAVES][64 * NV];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t wave_id = (int64_t)blockIdx.x * DS_WAVES + w;
    const int64_t q_beg = wave_id * per_wave;
    const int64_t q_end = q_beg + per_wave < n_pos ? q_beg + per_wave : n_pos;
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    const int my_z = ((lane >> 5) & 1) * 4 + ((lane >> 4) & 1) * 2 + ((lane >> 3) & 1);   // the row reduce8 leaves here
    bool ok[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) ok[u] = lane + 64 * u < d4;

    float4 aM[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) aM[u] = zero4;
    int32_t r_cur = -1;
    float lsum = 0.f;          // loss terms, each counted in one lane
    const int32_t per = n_neg + 2;

    auto flush_rel = [&](int32_t r) {
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            if (ok[u]) {
                float *dst = dM + ((int64_t)r * d4 + lane + 64 * u) * 4;
                unsafeAtomicAdd(dst + 0, aM[u].x); unsafeAtomicAdd(dst + 1, aM[u].y);
                unsafeAtomicAdd(dst + 2, aM[u].z); unsafeAtomicAdd(dst + 3, aM[u].w);
            }
            aM[u] = zero4;
        }
    };

    for (int64_t i = q_beg; i < q_end; ++i) {
        const int64_t q = (int64_t)perm[i];
        uint32_t c = (uint32_t)pos[q];
        if (c >= n_core) c = 0;           // counted by k_score_keys
        const int32_t s = core_h[c], r = core_r[c], t = core_t[c];
        if (r != r_cur) {                 // uniform: flush the relation gradient of the finished run
            if (r_cur >= 0) flush_rel(r_cur);
            r_cur = r;
        }
        float4 hs[NV], ht[NV], mr[NV], aS[NV], aT[NV];
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int k = lane + 64 * u;
            hs[u] = ok[u] ? H[(int64_t)s * d4 + k] : zero4;
            ht[u] = ok[u] ? H[(int64_t)t * d4 + k] : zero4;
            mr[u] = ok[u] ? M[(int64_t)r * d4 + k] : zero4;
        }
        {   // the positive
            float g = 0.f;
#pragma unroll
            for (int u = 0; u < NV; ++u) g += dot4(hs[u], mr[u], ht[u]);
            g = wave_sum(g);
            float sp, sg;
            softplus_sigmoid(-g, sp, sg);            // softplus(-g); sigmoid(g) - 1 = -sigmoid(-g)
            if (lane == 0) {
                lsum += sp;
                if (scores) scores[q * (1 + n_neg)] = g;
                recs[slot_of[q * per + n_neg]] = make_int4(-1 - (int32_t)(2 * q), r, 0, 0);
                recs[slot_of[q * per + n_neg + 1]] = make_int4(-1 - (int32_t)(2 * q + 1), r, 0, 0);
            }
            const float delta = -sg * inv_T;
#pragma unroll
            for (int u = 0; u < NV; ++u) {
                aS[u].x = delta * mr[u].x * ht[u].x; aS[u].y = delta * mr[u].y * ht[u].y;
                aS[u].z = delta * mr[u].z * ht[u].z; aS[u].w = delta * mr[u].w * ht[u].w;
                aT[u].x = delta * mr[u].x * hs[u].x; aT[u].y = delta * mr[u].y * hs[u].y;
                aT[u].z = delta * mr[u].z * hs[u].z; aT[u].w = delta * mr[u].w * hs[u].w;
                aM[u].x = fmaf(delta * hs[u].x, ht[u].x, aM[u].x); aM[u].y = fmaf(delta * hs[u].y, ht[u].y, aM[u].y);
                aM[u].z = fmaf(delta * hs[u].z, ht[u].z, aM[u].z); aM[u].w = fmaf(delta * hs[u].w, ht[u].w, aM[u].w);
            }
        }
        // negatives: 64 at a time, a lane per corrupting entity; within those, groups of eight rows
        for (int32_t kb = 0; kb < n_neg; kb += 64) {
            const int32_t cnt = n_neg - kb < 64 ? n_neg - kb : 64;
            int32_t my_ent = 0, my_side = 0;
            if (lane < cnt) {
                my_ent = neg_ent[q * n_neg + kb + lane];
                if ((uint32_t)my_ent >= n_vert) my_ent = 0;
                my_side = (int32_t)neg_side[q * n_neg + kb + lane];
            }
            const int32_t n_grp = (cnt + 7) >> 3;
            // fetch the eight rows of group g (rows past the end: zeros)
            auto fetch = [&](float4 (&hx)[8][NV], int32_t g) {
#pragma unroll
                for (int z = 0; z < 8; ++z) {
                    const int j = 8 * g + z;
                    const int32_t e = __shfl(my_ent, j < cnt ? j : 0, 64);
#pragma unroll
                    for (int u = 0; u < NV; ++u)
                        hx[z][u] = (j < cnt && ok[u]) ? H[(int64_t)e * d4 + lane + 64 * u] : zero4;
                }
            };
            // score the eight rows of group g and add what they contribute to the positive's own rows and to dM_r
            auto score = [&](const float4 (&hx)[8][NV], int32_t g) {
                const int32_t k0 = kb + 8 * g;
                int side[8];
                float part[8];
#pragma unroll
                for (int z = 0; z < 8; ++z) {
                    side[z] = __shfl(my_side, 8 * g + z < cnt ? 8 * g + z : 0, 64);
                    // the corrupted entity is scored against M_r * h_t (head replaced) or M_r * h_s
                    float gz = 0.f;
#pragma unroll
                    for (int u = 0; u < NV; ++u) gz += dot4(hx[z][u], mr[u], side[z] ? ht[u] : hs[u]);
                    part[z] = gz;
                }
                const float g_mine = reduce8(part, lane);          // score of row my_z, in its 8 lanes
                float sp, sg;
                softplus_sigmoid(g_mine, sp, sg);
                const float d_mine = sg * inv_T;
                if ((lane & 7) == 0 && k0 + my_z < n_neg) {         // one lane per row writes what the row produced
                    lsum += sp;
                    if (scores) scores[q * (1 + n_neg) + 1 + k0 + my_z] = g_mine;
                    const int64_t o = q * per + k0 + my_z;
                    int32_t oth = s;
#pragma unroll
                    for (int z = 0; z < 8; ++z) if (z == my_z && side[z]) oth = t;
                    recs[slot_of[o]] = make_int4(oth, r, __float_as_int(d_mine), 0);
                }
#pragma unroll
                for (int z = 0; z < 8; ++z) {
                    if (k0 + z >= n_neg) break;
                    const float delta = lane_value(d_mine, lane8_of(z));
#pragma unroll
                    for (int u = 0; u < NV; ++u) {
                        const float4 other = side[z] ? ht[u] : hs[u];
                        const float4 x = hx[z][u];
                        if (side[z]) {
                            aT[u].x = fmaf(delta * mr[u].x, x.x, aT[u].x); aT[u].y = fmaf(delta * mr[u].y, x.y, aT[u].y);
                            aT[u].z = fmaf(delta * mr[u].z, x.z, aT[u].z); aT[u].w = fmaf(delta * mr[u].w, x.w, aT[u].w);
                        } else {
                            aS[u].x = fmaf(delta * mr[u].x, x.x, aS[u].x); aS[u].y = fmaf(delta * mr[u].y, x.y, aS[u].y);
                            aS[u].z = fmaf(delta * mr[u].z, x.z, aS[u].z); aS[u].w = fmaf(delta * mr[u].w, x.w, aS[u].w);
                        }
                        aM[u].x = fmaf(delta * x.x, other.x, aM[u].x); aM[u].y = fmaf(delta * x.y, other.y, aM[u].y);
                        aM[u].z = fmaf(delta * x.z, other.z, aM[u].z); aM[u].w = fmaf(delta * x.w, other.w, aM[u].w);
                    }
                }
            };
            float4 bufA[8][NV], bufB[8][NV];
            fetch(bufA, 0);
            for (int32_t g = 0; g < n_grp; g += 2) {
                if (g + 1 < n_grp) fetch(bufB, g + 1);
                score(bufA, g);
                if (g + 1 < n_grp) {
                    if (g + 2 < n_grp) fetch(bufA, g + 2);
                    score(bufB, g + 1);
                }
            }
        }
        // the two rows this positive adds to its own head and tail
#pragma unroll
        for (int u = 0; u < NV; ++u)
            if (ok[u]) {
                rows[(2 * q) * d4 + lane + 64 * u] = aS[u];
                rows[(2 * q + 1) * d4 + lane + 64 * u] = aT[u];
            }
    }
    // What is still in registers - the relation gradient of the wavefront's last relation and its loss terms -
    // leaves as one partial per BLOCK when the block's wavefronts ended on the same relation (the usual case:
    // the positives are walked in relation order), and k_score_finish adds the partials up.  Thousands of
    // wavefronts adding to the same few rows of dM (one relation, or a few) would otherwise queue up on the
    // same addresses.
    lsum = wave_sum(lsum);
    if (lane == 0) { loss_of_wave[w] = lsum; rel_of_wave[w] = r_cur; }
#pragma unroll
    for (int u = 0; u < NV; ++u) part_of_wave[w][lane + 64 * u] = aM[u];
    __syncthreads();
    int32_t r0 = -1;
    bool same = true;
#pragma unroll
    for (int x = 0; x < DS_WAVES; ++x) {
        const int32_t r = rel_of_wave[x];
        if (r >= 0) {
            if (r0 < 0) r0 = r;
            else if (r != r0) same = false;
        }
    }
    if (same) {
        if (w == 0) {
#pragma unroll
            for (int u = 0; u < NV; ++u) {
                if (!ok[u]) continue;
                float4 t4 = part_of_wave[0][lane + 64 * u];
#pragma unroll
                for (int x = 1; x < DS_WAVES; ++x) {      // a wavefront without positives holds zeros
                    const float4 y = part_of_wave[x][lane + 64 * u];
                    t4.x += y.x; t4.y += y.y; t4.z += y.z; t4.w += y.w;
                }
                dm_part[(int64_t)blockIdx.x * d4 + lane + 64 * u] = t4;
            }
        }
    } else if (r_cur >= 0) {
        flush_rel(r_cur);
    }
    if (threadIdx.x == 0) {
        dm_rel[blockIdx.x] = same ? r0 : -1;
        float t = 0.f;
#pragma unroll
        for (int x = 0; x < DS_WAVES; ++x) t += loss_of_wave[x];
        loss_part[blockIdx.x] = t;
    }
}

// loss = (sum of the blocks' loss terms) / T, in a fixed order; dM[r] += the blocks' partial rows of relation r.
// Block c walks the c-th range of the scoring blocks (they are in relation order, so a relation's partials are
// consecutive) and adds a run of equal relations in registers before it touches dM.
__global__ __launch_bounds__(256) void k_score_finish(const float *__restrict__ dm_part, const int32_t *__restrict__ dm_rel,
                                                      const float *__restrict__ loss_part, int32_t n_blocks, int32_t len,
                                                      int32_t d, float inv_T, float *__restrict__ dM, float *__restrict__ loss)
{
    __shared__ float red[256];
    const int32_t b0 = blockIdx.x * len, b1 = b0 + len < n_blocks ? b0 + len : n_blocks;
    for (int32_t k = threadIdx.x; k < d; k += 256) {
        float acc = 0.f;
        int32_t r_acc = -1;
        for (int32_t b = b0; b < b1; ++b) {
            const int32_t r = dm_rel[b];
            if (r < 0) continue;
            if (r != r_acc) {
                if (r_acc >= 0) unsafeAtomicAdd(dM + (int64_t)r_acc * d + k, acc);
                acc = 0.f;
                r_acc = r;
            }
            acc += dm_part[(int64_t)b * d + k];
        }
        if (r_acc >= 0) unsafeAtomicAdd(dM + (int64_t)r_acc * d + k, acc);
    }
    if (blockIdx.x == 0) {
        float t = 0.f;
        for (int32_t b = threadIdx.x; b < n_blocks; b += 256) t += loss_part[b];
        red[threadIdx.x] = t;
        __syncthreads();
        for (int off = 128; off > 0; off >>= 1) {
            if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
            __syncthreads();
        }
        if (threadIdx.x == 0) loss[0] = red[0] * inv_T;
    }
}

// dH[e] = sum over the occurrences of entity e, in ascending occurrence id, of
//   delta (M_r * h_other)   for a negative that put e into a triple, or the stored row of a positive's own end.
// The rows h_other are those of the batch's positives (a few hundred MB at most, re-read many times: they stay in
// the last-level cache).  A wavefront owns DG_ENT consecutive entities and streams their occurrences - contiguous
// in the entity-sorted list - four at a time (eight rows in flight) straight across the entity boundaries: when
// the next occurrence belongs to a later entity the finished sum is stored and the accumulator cleared.  Every
// row of dH is written exactly once (zeros for entities no triple names), in a fixed order of additions: the
// result repeats bit for bit.
constexpr int DG_ENT = 16;
template <int NV>
__global__ __launch_bounds__(256) void k_distmult_gather(
    const float4 *__restrict__ H, const float4 *__restrict__ M, int32_t d4, int64_t N,
    const int32_t *__restrict__ ent_ptr, const int4 *__restrict__ recs, const float4 *__restrict__ rows,
    float4 *__restrict__ dH)
{
    const int lane = threadIdx.x & 63;
    const int64_t e0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * DG_ENT;
    if (e0 >= N) return;
    const int n_ent = N - e0 < DG_ENT ? (int)(N - e0) : DG_ENT;
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f), one4 = make_float4(1.f, 1.f, 1.f, 1.f);
    bool ok[NV];
    float4 acc[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) { ok[u] = lane + 64 * u < d4; acc[u] = zero4; }
    const int32_t my_ptr = lane <= n_ent ? ent_ptr[e0 + lane] : 0x7fffffff;      // lane l: where entity e0 + l starts
    const int32_t lo = __shfl(my_ptr, 0, 64), hi = __shfl(my_ptr, n_ent, 64);
    int cur = 0;                                   // the entity being summed
    int32_t boundary = __shfl(my_ptr, 1, 64);      // where the next one starts
    auto close_entity = [&]() {
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            if (ok[u]) dH[(e0 + cur) * d4 + lane + 64 * u] = acc[u];
            acc[u] = zero4;
        }
        ++cur;
        boundary = __shfl(my_ptr, cur + 1, 64);
    };
    for (int32_t base = lo; base < hi; base += 64) {
        const int32_t cnt = hi - base < 64 ? hi - base : 64;
        int32_t other = 0, rel = 0;
        float wgt = 0.f;
        if (lane < cnt) {
            const int4 rec = recs[base + lane];
            other = rec.x; rel = rec.y;
            wgt = other >= 0 ? __int_as_float(rec.z) : 1.f;
        }
        for (int32_t j0 = 0; j0 < cnt; j0 += 4) {
            float4 a[4][NV], b[4][NV];
            float wj[4];
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                const int j = j0 + z < cnt ? j0 + z : cnt - 1;          // past the end: the last one again, unused
                const int32_t oj = __shfl(other, j, 64), rj = __shfl(rel, j, 64);
                wj[z] = __shfl(wgt, j, 64);
#pragma unroll
                for (int u = 0; u < NV; ++u) {
                    const int k = lane + 64 * u;
                    if (!ok[u]) { a[z][u] = zero4; b[z][u] = zero4; }
                    else if (oj < 0) { a[z][u] = rows[(int64_t)(-1 - oj) * d4 + k]; b[z][u] = one4; }
                    else { a[z][u] = H[(int64_t)oj * d4 + k]; b[z][u] = M[(int64_t)rj * d4 + k]; }
                }
            }
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                if (j0 + z >= cnt) break;
                while (base + j0 + z >= boundary) close_entity();       // uniform: entities without occurrences too
#pragma unroll
                for (int u = 0; u < NV; ++u) {
                    acc[u].x = fmaf(wj[z] * b[z][u].x, a[z][u].x, acc[u].x);
                    acc[u].y = fmaf(wj[z] * b[z][u].y, a[z][u].y, acc[u].y);
                    acc[u].z = fmaf(wj[z] * b[z][u].z, a[z][u].z, acc[u].z);
                    acc[u].w = fmaf(wj[z] * b[z][u].w, a[z][u].w, acc[u].w);
                }
            }
        }
    }
    while (cur < n_ent) close_entity();
}

}  // namespace

int launch_sample_negatives(const kge_partition *p, const int32_t *pos, int64_t n_pos, int32_t n_neg,
                            int32_t mode, uint64_t seed, uint64_t step, int32_t *neg_ent,
                            uint8_t *neg_side, hipStream_t st)
{
    const int64_t total = n_pos * n_neg;
    if (total == 0) return KGE_OK;
    KGE_REQUIRE(p->n_cand > 0, KGE_EINVAL, "the partition has no vertex to draw negatives from");
    KGE_REQUIRE(cdiv(total, 256) < 0x7fffffffLL, KGE_ERANGE, "too many negatives for one launch");
    KGE_PROF("sample_neg", st);
    k_sample_negatives<<<(unsigned)cdiv(total, 256), 256, 0, st>>>(
        p->cand, (uint32_t)p->n_cand, pos, n_pos, n_neg, mode, (uint32_t)seed, (uint32_t)(seed >> 32),
        (uint32_t)step, (uint32_t)(step >> 32), neg_ent, neg_side);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

extern "C" int kge_score_index_create(const kge_partition *p, int64_t max_pos, int32_t max_neg, int32_t d,
                                      kge_score_index **out)
{
    KGE_REQUIRE(p && out, KGE_EINVAL, "NULL argument");
    *out = nullptr;
    KGE_REQUIRE(max_pos >= 1 && max_neg >= 0 && d > 0 && d % 4 == 0 && d <= 512, KGE_EINVAL,
                "max_pos must be positive, max_neg non-negative, d a multiple of 4 in [4, 512]");
    const int64_t max_occ = max_pos * ((int64_t)max_neg + 2);
    KGE_REQUIRE(max_pos < (1ll << 29) && max_occ < 0x7fffffffll, KGE_ERANGE, "batch too large for 32-bit occurrence ids");
    kge_score_index *x = new kge_score_index();
    memset(x, 0, sizeof *x);
    x->device = p->device; x->n_vert = p->n_vert; x->max_pos = max_pos; x->max_occ = max_occ; x->max_neg = max_neg; x->d = d;
    hipError_t e = hipSuccess;
    auto take = [&](void **q, size_t bytes) { if (e == hipSuccess) e = hipMalloc(q, bytes ? bytes : 4); };
    for (int k = 0; k < 2; ++k) { take((void **)&x->keys[k], 4 * (size_t)max_occ); take((void **)&x->vals[k], 4 * (size_t)max_occ); }
    take((void **)&x->sort_ws, 4 * radix_scratch_words(max_occ));
    take((void **)&x->ent_ptr, 4 * ((size_t)p->n_vert + 1));
    take((void **)&x->slot_of, 4 * (size_t)max_occ);
    take((void **)&x->recs, 16 * (size_t)max_occ);
    for (int k = 0; k < 2; ++k) { take((void **)&x->pkeys[k], 4 * (size_t)max_pos); take((void **)&x->pvals[k], 4 * (size_t)max_pos); }
    take((void **)&x->rows, 4 * (size_t)2 * max_pos * d);
    take((void **)&x->dm_part, 4 * (size_t)KGE_SCORE_MAX_BLOCKS * d);
    take((void **)&x->dm_rel, 4 * (size_t)KGE_SCORE_MAX_BLOCKS);
    take((void **)&x->loss_part, 4 * (size_t)KGE_SCORE_MAX_BLOCKS);
    if (e != hipSuccess) {
        kge_set_error("allocating the scoring index failed: %s", hipGetErrorString(e));
        kge_score_index_destroy(x);
        return KGE_ENOMEM;
    }
    *out = x;
    return KGE_OK;
}

extern "C" void kge_score_index_destroy(kge_score_index *x)
{
    if (!x) return;
    void *all[] = {x->keys[0], x->keys[1], x->vals[0], x->vals[1], x->sort_ws, x->ent_ptr, x->slot_of, x->recs,
                   x->pkeys[0], x->pkeys[1], x->pvals[0], x->pvals[1], x->rows, x->dm_part, x->dm_rel, x->loss_part};
    for (void *q : all) if (q) (void)hipFree(q);
    delete x;
}

// The atomic-free form: sort the batch's occurrences by entity (stable, so ties keep occurrence order), score
// every triple, then let one wavefront per entity add up its rows.
int launch_distmult_indexed(const kge_partition *p, kge_score_index *x, const float *H, const float *M, int32_t d,
                            const int32_t *pos, int64_t n_pos, const int32_t *neg_ent, const uint8_t *neg_side,
                            int32_t n_neg, float *scores, float *loss, float *dH, float *dM, hipStream_t st)
{
    KGE_REQUIRE(x->n_vert == p->n_vert && x->device == p->device, KGE_EINVAL, "the scoring index was created for another partition");
    KGE_REQUIRE(n_pos <= x->max_pos && n_neg <= x->max_neg && d == x->d, KGE_EINVAL,
                "the scoring index was created for at most %lld positives x %d negatives of width %d",
                (long long)x->max_pos, x->max_neg, x->d);
    KGE_REQUIRE(((uintptr_t)H % 16) == 0 && ((uintptr_t)M % 16) == 0 && ((uintptr_t)dH % 16) == 0, KGE_EINVAL,
                "H, M and dH must be 16-byte aligned");
    int rc = launch_fill_zero(dM, sizeof(float) * (size_t)p->n_relations * d, st);
    if (rc != KGE_OK) return rc;
    rc = launch_fill_zero(loss, sizeof(float), st);
    if (rc != KGE_OK) return rc;
    if (n_pos == 0 || p->n_vert == 0) return launch_fill_zero(dH, sizeof(float) * (size_t)p->n_vert * d, st);
    const int64_t n_occ = n_pos * ((int64_t)n_neg + 2);
    const float inv_T = (float)(1.0 / ((double)n_pos * (1.0 + (double)n_neg)));
    const int32_t d4 = d / 4;
    uint32_t *keys = x->keys[0], *keys_alt = x->keys[1], *vals = x->vals[0], *vals_alt = x->vals[1];
    uint32_t *pkeys = x->pkeys[0], *pkeys_alt = x->pkeys[1], *pvals = x->pvals[0], *pvals_alt = x->pvals[1];
    {
        KGE_PROF("score_index", st);
        k_score_keys<<<(unsigned)cdiv(n_occ, 256), 256, 0, st>>>(p->core_h, p->core_t, pos, n_pos, neg_ent, n_neg,
                                                                (uint32_t)p->n_vert, (uint32_t)p->n_core, keys, vals, p->bad_ids);
        KGE_LAUNCH_CHECK();
        int bits = 1;
        while (bits < 32 && ((int64_t)1 << bits) < p->n_vert) ++bits;
        rc = radix_sort_ws<uint32_t>(&keys, &vals, &keys_alt, &vals_alt, n_occ, bits, x->sort_ws, st);
        if (rc != KGE_OK) return rc;
        k_ptr_from_sorted<uint32_t><<<(unsigned)cdiv(n_occ + 1, 256), 256, 0, st>>>(keys, n_occ, p->n_vert, x->ent_ptr);
        KGE_LAUNCH_CHECK();
        k_invert_permutation<<<(unsigned)cdiv(n_occ, 256), 256, 0, st>>>(vals, n_occ, x->slot_of);
        KGE_LAUNCH_CHECK();
        // the positives in relation order (stable), for the walk of the scoring kernel
        k_score_rel_keys<<<(unsigned)cdiv(n_pos, 256), 256, 0, st>>>(p->core_r, pos, n_pos, (uint32_t)p->n_core, pkeys, pvals);
        KGE_LAUNCH_CHECK();
        int rbits = 1;
        while (rbits < 32 && ((int64_t)1 << rbits) < p->n_relations) ++rbits;
        rc = radix_sort_ws<uint32_t>(&pkeys, &pvals, &pkeys_alt, &pvals_alt, n_pos, rbits, x->sort_ws, st);
        if (rc != KGE_OK) return rc;
    }
    int64_t per_wave = cdiv(n_pos, 16384);
    if (per_wave < 4) per_wave = n_pos >= 4 * 1024 ? 4 : 1;
    const int64_t waves = cdiv(n_pos, per_wave);
    const unsigned grid = (unsigned)cdiv(waves, DS_WAVES);
    {
        KGE_PROF("distmult", st);
#define DMS_CALL(NVV)                                                                                               \
        k_distmult_score<NVV><<<grid, 64 * DS_WAVES, 0, st>>>((const float4 *)H, (const float4 *)M, d4, p->core_h,  \
            p->core_r, p->core_t, pos, pvals, n_pos, (int32_t)per_wave, neg_ent, neg_side, n_neg,                  \
            (uint32_t)p->n_vert, (uint32_t)p->n_core, inv_T, scores, dM, x->slot_of, x->recs, (float4 *)x->rows,  \
            (float4 *)x->dm_part, x->dm_rel, x->loss_part)
        KGE_REQUIRE(grid <= KGE_SCORE_MAX_BLOCKS, KGE_ERANGE, "scoring: more blocks than the index has partial rows for");
        if (d4 <= 64) DMS_CALL(1); else DMS_CALL(2);
#undef DMS_CALL
        KGE_LAUNCH_CHECK();
        const int32_t n_chunks = grid < 64 ? (int32_t)grid : 64, len = (int32_t)cdiv(grid, n_chunks);
        k_score_finish<<<(unsigned)cdiv(grid, len), 256, 0, st>>>(x->dm_part, x->dm_rel, x->loss_part, (int32_t)grid, len, d,
                                                                   inv_T, dM, loss);
        KGE_LAUNCH_CHECK();
    }
    {
        KGE_PROF("distmult_gather", st);
        const unsigned g2 = (unsigned)cdiv(cdiv(p->n_vert, DG_ENT), 4);
        if (d4 <= 64)
            k_distmult_gather<1><<<g2, 256, 0, st>>>((const float4 *)H, (const float4 *)M, d4, p->n_vert, x->ent_ptr,
                                                     x->recs, (const float4 *)x->rows, (float4 *)dH);
        else
            k_distmult_gather<2><<<g2, 256, 0, st>>>((const float4 *)H, (const float4 *)M, d4, p->n_vert, x->ent_ptr,
                                                     x->recs, (const float4 *)x->rows, (float4 *)dH);
        KGE_LAUNCH_CHECK();
    }
    return KGE_OK;
}

int launch_distmult(const kge_partition *p, const float *H, const float *M, int32_t d,
                    const int32_t *pos, int64_t n_pos, const int32_t *neg_ent, const uint8_t *neg_side,
                    int32_t n_neg, float *scores, float *loss, float *dH, float *dM, hipStream_t st)
{
    int rc = launch_fill_zero(dH, sizeof(float) * (size_t)p->n_vert * d, st);
    if (rc != KGE_OK) return rc;
    rc = launch_fill_zero(dM, sizeof(float) * (size_t)p->n_relations * d, st);
    if (rc != KGE_OK) return rc;
    rc = launch_fill_zero(loss, sizeof(float), st);
    if (rc != KGE_OK) return rc;
    if (n_pos == 0) return KGE_OK;
    const float inv_T = (float)(1.0 / ((double)n_pos * (1.0 + (double)n_neg)));
    // about 16k wavefronts, at least 4 positives each when there are enough of them
    int64_t per_wave = cdiv(n_pos, 16384);
    if (per_wave < 4) per_wave = n_pos >= 4 * 1024 ? 4 : 1;
    const int64_t waves = cdiv(n_pos, per_wave);
    const unsigned grid = (unsigned)cdiv(waves, DM_WAVES);
    KGE_PROF("distmult", st);
#define DM_CALL(NCHV)                                                                                \
    k_distmult<NCHV><<<grid, 64 * DM_WAVES, 0, st>>>(H, M, d, p->core_h, p->core_r, p->core_t, pos,  \
                                                    n_pos, (int32_t)per_wave, neg_ent, neg_side,     \
                                                    n_neg, (uint32_t)p->n_vert, (uint32_t)p->n_core, \
                                                    p->bad_ids, inv_T, scores, loss, dH, dM)
    if (d <= 64) DM_CALL(1);
    else if (d <= 128) DM_CALL(2);
    else if (d <= 256) DM_CALL(4);
    else if (d <= 512) DM_CALL(8);
    else KGE_REQUIRE(false, KGE_EINVAL, "embedding width %d > 512 is not supported by the scoring kernel", d);
#undef DM_CALL
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}
