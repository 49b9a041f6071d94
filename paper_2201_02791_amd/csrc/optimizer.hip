// Optimizer step (Algorithm 1, "optimizer.step()"): plain gradient descent or Adam (Kingma & Ba 2015),
// one fused pass over a parameter tensor, its gradient and (Adam) its two moment tensors.
//
//   SGD   p <- p - lr g
//   Adam  m <- b1 m + (1 - b1) g;  v <- b2 v + (1 - b2) g^2;
//         p <- p - lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
//
// The row form serves embedding tables of which a step reaches few rows: a wavefront owns a row and
// leaves it (parameters and moments) untouched when the row's mask byte is zero or, without a
// mask, when every element of its gradient is zero.  Bandwidth bound: 16 bytes read and 12 written
// per Adam element.
#include "common.h"

namespace {

struct OptArgs {
    int kind;
    float lr, b1, b2, eps, omb1, omb2, inv_c1, inv_c2;   // omb = 1 - b, inv_c = 1 / (1 - b^t): computed in double on the host
};

__device__ __forceinline__ void opt_update(const OptArgs &o, float &p, float g, float &m, float &v)
{
    if (o.kind == KGE_OPT_SGD) { p -= o.lr * g; return; }
    m = o.b1 * m + o.omb1 * g;
    v = o.b2 * v + o.omb2 * g * g;
    p -= o.lr * (m * o.inv_c1) / (sqrtf(v * o.inv_c2) + o.eps);
}

__global__ void k_opt_dense(OptArgs o, float *__restrict__ p, const float *__restrict__ g, float *__restrict__ m,
                            float *__restrict__ v, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float pi = p[i], mi = 0.f, vi = 0.f;
        if (o.kind == KGE_OPT_ADAM) { mi = m[i]; vi = v[i]; }
        opt_update(o, pi, g[i], mi, vi);
        p[i] = pi;
        if (o.kind == KGE_OPT_ADAM) { m[i] = mi; v[i] = vi; }
    }
}

// one wavefront per row of d elements (d a multiple of 4)
__global__ __launch_bounds__(256) void k_opt_rows(OptArgs o, float *__restrict__ p, const float *__restrict__ g,
                                                  float *__restrict__ m, float *__restrict__ v, int64_t n_rows,
                                                  int32_t d, const uint8_t *__restrict__ row_mask)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    const int d4 = d >> 2;
    const float4 *g4 = reinterpret_cast<const float4 *>(g + row * d);
    if (row_mask) {
        if (!row_mask[row]) return;
    } else {
        bool any = false;
        for (int k = lane; k < d4; k += 64) {
            const float4 x = g4[k];
            any |= (x.x != 0.f) | (x.y != 0.f) | (x.z != 0.f) | (x.w != 0.f);
        }
        if (__ballot(any) == 0ull) return;
    }
    float4 *p4 = reinterpret_cast<float4 *>(p + row * d);
    float4 *m4 = reinterpret_cast<float4 *>(m ? m + row * d : nullptr);
    float4 *v4 = reinterpret_cast<float4 *>(v ? v + row * d : nullptr);
    for (int k = lane; k < d4; k += 64) {
        float4 pp = p4[k];
        const float4 gg = g4[k];
        float4 mm = make_float4(0.f, 0.f, 0.f, 0.f), vv = mm;
        if (o.kind == KGE_OPT_ADAM) { mm = m4[k]; vv = v4[k]; }
        opt_update(o, pp.x, gg.x, mm.x, vv.x); opt_update(o, pp.y, gg.y, mm.y, vv.y);
        opt_update(o, pp.z, gg.z, mm.z, vv.z); opt_update(o, pp.w, gg.w, mm.w, vv.w);
        p4[k] = pp;
        if (o.kind == KGE_OPT_ADAM) { m4[k] = mm; v4[k] = vv; }
    }
}

int make_args(const kge_opt *opt, const float *param, const float *grad, const float *m, const float *v, OptArgs *o)
{
    KGE_REQUIRE(opt && param && grad, KGE_EINVAL, "NULL argument");
    KGE_REQUIRE(opt->kind == KGE_OPT_SGD || opt->kind == KGE_OPT_ADAM, KGE_EINVAL, "bad optimizer kind");
    o->kind = opt->kind; o->lr = opt->lr; o->b1 = opt->beta1; o->b2 = opt->beta2; o->eps = opt->eps;
    o->inv_c1 = o->inv_c2 = 1.f;
    o->omb1 = (float)(1.0 - (double)opt->beta1); o->omb2 = (float)(1.0 - (double)opt->beta2);
    if (opt->kind == KGE_OPT_ADAM) {
        KGE_REQUIRE(m && v, KGE_EINVAL, "Adam needs both moment tensors");
        KGE_REQUIRE(opt->t >= 1, KGE_EINVAL, "Adam's step number t starts at 1");
        KGE_REQUIRE(opt->beta1 >= 0.f && opt->beta1 < 1.f && opt->beta2 >= 0.f && opt->beta2 < 1.f, KGE_EINVAL,
                    "beta1 and beta2 must be in [0, 1)");
        o->inv_c1 = (float)(1.0 / (1.0 - pow((double)opt->beta1, (double)opt->t)));
        o->inv_c2 = (float)(1.0 / (1.0 - pow((double)opt->beta2, (double)opt->t)));
    }
    return KGE_OK;
}

}  // namespace

extern "C" int kge_optimizer_step(const kge_opt *opt, float *param, const float *grad, float *m, float *v,
                                  int64_t n, void *stream)
{
    OptArgs o;
    int rc = make_args(opt, param, grad, m, v, &o);
    if (rc != KGE_OK) return rc;
    KGE_REQUIRE(n >= 0, KGE_EINVAL, "negative size");
    if (n == 0) return KGE_OK;
    hipStream_t st = (hipStream_t)stream;
    int64_t blocks = cdiv(n, 256);
    if (blocks > 65536) blocks = 65536;
    KGE_PROF("optimizer", st);
    k_opt_dense<<<(unsigned)blocks, 256, 0, st>>>(o, param, grad, m, v, n);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

extern "C" int kge_optimizer_step_rows(const kge_opt *opt, float *param, const float *grad, float *m, float *v,
                                       int64_t n_rows, int32_t d, const uint8_t *row_mask, void *stream)
{
    OptArgs o;
    int rc = make_args(opt, param, grad, m, v, &o);
    if (rc != KGE_OK) return rc;
    KGE_REQUIRE(n_rows >= 0 && d > 0 && d % 4 == 0, KGE_EINVAL, "d must be a positive multiple of 4");
    KGE_REQUIRE(((uintptr_t)param % 16) == 0 && ((uintptr_t)grad % 16) == 0 && ((uintptr_t)m % 16) == 0 &&
                    ((uintptr_t)v % 16) == 0, KGE_EINVAL, "row tensors must be 16-byte aligned");
    if (n_rows == 0) return KGE_OK;
    KGE_REQUIRE(cdiv(n_rows, 4) < 0x7fffffffLL, KGE_ERANGE, "too many rows");
    hipStream_t st = (hipStream_t)stream;
    KGE_PROF("optimizer_rows", st);
    k_opt_rows<<<(unsigned)cdiv(n_rows, 4), 256, 0, st>>>(o, param, grad, m, v, n_rows, d, row_mask);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}
