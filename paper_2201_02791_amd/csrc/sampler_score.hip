// In-partition negative sampling (Sec. 2.1 corruption under the constraint of Sec. 3.3.1)
// with a counter-based generator, and the fused DistMult score (Eq. 4) + cross-entropy loss
// (Eq. 3) + gradient kernel.
#include "common.h"

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
        const int32_t c = pos[q];
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
                                                    n_neg, inv_T, scores, loss, dH, dM)
    if (d <= 64) DM_CALL(1);
    else if (d <= 128) DM_CALL(2);
    else if (d <= 256) DM_CALL(4);
    else if (d <= 512) DM_CALL(8);
    else KGE_REQUIRE(false, KGE_EINVAL, "embedding width %d > 512 is not supported by the scoring kernel", d);
#undef DM_CALL
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}
