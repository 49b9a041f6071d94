// Dropout on the features a layer reads (training setting of Sec. 4, rate 0.2 on the large graphs).
//
// Inverted form: out = keep ? h / (1 - p) : 0, applied to the layer input that the neighbour
// messages, the self-loop and the weight gradients all read.  The keep decision of element (i, k)
// is a pure function of (seed, step, layer, i, k): word (k mod 4) of
//     Philox4x32-10(counter = (i, k / 4, step lo, step hi), key = (seed lo, seed hi xor (layer + 1)))
// compared with floor(p * 2^32) (kept when not below).  Backward regenerates it, so no mask is stored:
// one launch costs a read and a write of the matrix and 10 Philox rounds per four elements.
#include "common.h"

namespace {

__device__ __forceinline__ void philox4(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                                        uint32_t x[4])
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0; c1 = lo1; c2 = hi0 ^ c3 ^ k1; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    x[0] = c0; x[1] = c1; x[2] = c2; x[3] = c3;
}

// One thread per four consecutive columns of one row.  src == dst is allowed (backward runs in place).
__global__ __launch_bounds__(256) void k_dropout(const float4 *src, int64_t n_groups, int32_t groups_per_row,
                                                 uint32_t thr, float scale, uint32_t k0, uint32_t k1,
                                                 uint32_t step_lo, uint32_t step_hi, float4 *dst)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n_groups) return;
    const uint32_t row = (uint32_t)(t / groups_per_row), g = (uint32_t)(t - (int64_t)row * groups_per_row);
    uint32_t x[4];
    philox4(row, g, step_lo, step_hi, k0, k1, x);
    float4 v = src[t];
    v.x = x[0] >= thr ? v.x * scale : 0.0f;
    v.y = x[1] >= thr ? v.y * scale : 0.0f;
    v.z = x[2] >= thr ? v.z * scale : 0.0f;
    v.w = x[3] >= thr ? v.w * scale : 0.0f;
    dst[t] = v;
}

}  // namespace

int launch_dropout(const float *src, int64_t n_rows, int32_t d, float p, uint64_t seed, uint64_t step, int32_t layer,
                   float *dst, hipStream_t st)
{
    KGE_REQUIRE(d > 0 && d % 4 == 0, KGE_EINVAL, "dropout: the row width must be a positive multiple of 4");
    KGE_REQUIRE(p >= 0.0f && p < 1.0f, KGE_EINVAL, "dropout: the rate must be in [0, 1)");
    KGE_REQUIRE(n_rows >= 0 && n_rows <= 0xFFFFFFFFll, KGE_EINVAL, "dropout: row count out of range");
    const int64_t n_groups = n_rows * (d / 4);
    if (n_groups == 0) return KGE_OK;
    KGE_REQUIRE(cdiv(n_groups, 256) <= 0x7FFFFFFFll, KGE_ERANGE, "dropout: matrix too large for one launch");
    KGE_PROF("dropout", st);
    // threshold and scale in double on the host, so that both are the correctly rounded values of p
    const uint32_t thr = (uint32_t)((double)p * 4294967296.0);
    const float scale = (float)(1.0 / (1.0 - (double)p));
    k_dropout<<<(unsigned)cdiv(n_groups, 256), 256, 0, st>>>((const float4 *)src, n_groups, d / 4, thr, scale,
                                                            (uint32_t)seed, (uint32_t)(seed >> 32) ^ (uint32_t)(layer + 1),
                                                            (uint32_t)step, (uint32_t)(step >> 32), (float4 *)dst);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}
