// Dense contractions of the encoder (Eq. 2 applied to every vertex, and its two
// transposes for the backward pass) on the gfx950 matrix cores.
//
//   project      P = H [V_1 .. V_B | W_0]                      (N x d_in) (d_in x (B+1)d_out)
//   weight_grad  d[V_1 .. V_B | W_0] = H^T [dP | G]            (d_in x N) (N x (B+1)d_out)
//   input_grad   dH = [dP | G] [V_1 .. V_B | W_0]^T            (N x (B+1)d_out) ((B+1)d_out x d_in)
//
// and, for layers that apply W_r per (relation, destination) run,
//
//   rel_outer    C_r = sum_{runs s of r} Z_s^T G_{dst(s)}        grouped over relations, (d_in x d_out) each
//   coeff        da = C Vflat^T                                  (2R x d_in d_out) (d_in d_out x B)
//
// One kernel template: 128x128 block tile, 4 wavefronts in a 2x2 grid, each wavefront owns a
// 64x64 sub-tile as 2x2 v_mfma_f32_32x32x2_f32 accumulators.  Operands are staged through LDS
// K-major (As[k][m], Bs[k][n]) so that the MFMA operand reads are 32 consecutive floats.
// Operand loaders and the epilogue are small functors, so the concatenated operands
// ([V|W0], [dP|G]) are never materialised.  This file is the fp32 path; workloads with bf16
// messages use the bf16 matrix-core kernels of gemm_bf16.hip.
#include "common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 16, PADL = 4, GT = 256;

// ---- operand sources: load4(row, col) returns 4 consecutive elements along the contiguous
// dimension starting at (row, col); out-of-range -> zeros.  Contiguous extents are multiples of 4.

// Hooks every source and epilogue has: limit_rows(e) hides rows >= e (a row tile that ends inside the
// block), bind(g) selects group g's matrix or output.  No-ops where they mean nothing.
struct SrcRowMajorF32 {          // X[r][c], c contiguous
    const float *p; int64_t rows; int32_t cols;
    __device__ __forceinline__ void limit_rows(int64_t e) { if (e < rows) rows = e; }
    __device__ __forceinline__ void bind(int32_t) {}
    __device__ __forceinline__ float4 load4(int64_t r, int32_t c) const
    {
        if (r >= rows || c >= cols) return make_float4(0.f, 0.f, 0.f, 0.f);
        return *reinterpret_cast<const float4 *>(p + r * cols + c);
    }
};

// [V_1 .. V_B | W0] viewed as a (d_in x (B+1) d_out) matrix, column index contiguous inside a block
struct SrcWcat {
    const float *V, *W0; int32_t d_in, d_out, B;
    __device__ __forceinline__ void limit_rows(int64_t) {}
    __device__ __forceinline__ void bind(int32_t) {}
    __device__ __forceinline__ float4 load4(int64_t k, int32_t c) const
    {
        int32_t nc = (B + 1) * d_out;
        if (k >= d_in || c >= nc) return make_float4(0.f, 0.f, 0.f, 0.f);
        int32_t b = c / d_out, cc = c - b * d_out;
        const float *base = b < B ? V + ((int64_t)b * d_in + k) * d_out : W0 + k * d_out;
        return *reinterpret_cast<const float4 *>(base + cc);
    }
};

// [dP | G] viewed as an (N x (B+1) d_out) matrix, both fp32
struct SrcXcat {
    const float *dP; const float *G; int64_t rows; int32_t d_out, B;
    __device__ __forceinline__ void limit_rows(int64_t) {}
    __device__ __forceinline__ void bind(int32_t) {}
    __device__ __forceinline__ float4 load4(int64_t r, int32_t c) const
    {
        int32_t bd = B * d_out;
        if (r >= rows || c >= bd + d_out) return make_float4(0.f, 0.f, 0.f, 0.f);
        if (c >= bd) return *reinterpret_cast<const float4 *>(G + r * d_out + (c - bd));
        return *reinterpret_cast<const float4 *>(dP + r * bd + c);
    }
};

// rows of X picked through an index list: row k is X[idx[k]]
struct SrcGatherRows {
    const float *X; const int32_t *idx; int64_t n_idx; int32_t cols;
    __device__ __forceinline__ void limit_rows(int64_t e) { if (e < n_idx) n_idx = e; }
    __device__ __forceinline__ void bind(int32_t) {}
    __device__ __forceinline__ float4 load4(int64_t k, int32_t c) const
    {
        if (k >= n_idx || c >= cols) return make_float4(0.f, 0.f, 0.f, 0.f);
        return *reinterpret_cast<const float4 *>(X + (int64_t)idx[k] * cols + c);
    }
};

// one (rows x cols) matrix per group, W[g][r][c]
struct SrcGroupMat {
    const float *W; int32_t rows, cols;
    __device__ __forceinline__ void limit_rows(int64_t) {}
    __device__ __forceinline__ void bind(int32_t g) { W += (int64_t)g * rows * cols; }
    __device__ __forceinline__ float4 load4(int64_t r, int32_t c) const
    {
        if (r >= rows || c >= cols) return make_float4(0.f, 0.f, 0.f, 0.f);
        return *reinterpret_cast<const float4 *>(W + r * cols + c);
    }
};

// ---- epilogues: store(m, n, value); bind(g) tells a grouped launch which group the block works on
struct EpiProject {             // columns < B*d_out go to P, the rest to Self
    float *P; float *Self; int64_t rows; int32_t d_out, B;
    __device__ __forceinline__ void bind(int32_t) {}
    __device__ __forceinline__ void limit_rows(int64_t) {}
    __device__ __forceinline__ void store(int64_t m, int32_t n, float v) const
    {
        int32_t bd = B * d_out;
        if (m >= rows || n >= bd + d_out) return;
        if (n >= bd) Self[m * d_out + (n - bd)] = v;
        else P[m * bd + n] = v;
    }
};

struct EpiWeightGrad {          // atomic accumulation of split-K partial tiles
    float *dV, *dW0; int32_t d_in, d_out, B;
    __device__ __forceinline__ void bind(int32_t) {}
    __device__ __forceinline__ void limit_rows(int64_t) {}
    __device__ __forceinline__ void store(int64_t m, int32_t n, float v) const
    {
        int32_t bd = B * d_out;
        if (m >= d_in || n >= bd + d_out) return;
        int32_t b = n / d_out, c = n - b * d_out;
        float *dst = b < B ? dV + ((int64_t)b * d_in + m) * d_out + c : dW0 + m * d_out + c;
        unsafeAtomicAdd(dst, v);
    }
};

struct EpiRowMajor {
    float *out; int64_t rows; int32_t cols;
    __device__ __forceinline__ void bind(int32_t) {}
    __device__ __forceinline__ void limit_rows(int64_t e) { if (e < rows) rows = e; }
    __device__ __forceinline__ void store(int64_t m, int32_t n, float v) const
    {
        if (m < rows && n < cols) __builtin_nontemporal_store(v, out + m * cols + n);
    }
};

struct EpiRowMajorAtomic {      // split-K partial tiles
    float *out; int64_t rows; int32_t cols;
    __device__ __forceinline__ void bind(int32_t) {}
    __device__ __forceinline__ void limit_rows(int64_t) {}
    __device__ __forceinline__ void store(int64_t m, int32_t n, float v) const
    {
        if (m < rows && n < cols) unsafeAtomicAdd(out + m * cols + n, v);
    }
};

struct EpiRelOuter {            // C[group] (d_in x d_out) accumulates the chunks of one relation
    float *C; int32_t d_in, d_out; int32_t group;
    __device__ __forceinline__ void bind(int32_t g) { group = g; }
    __device__ __forceinline__ void limit_rows(int64_t) {}
    __device__ __forceinline__ void store(int64_t m, int32_t n, float v) const
    {
        if (m < d_in && n < d_out) unsafeAtomicAdd(C + ((int64_t)group * d_in + m) * d_out + n, v);
    }
};

// A(m,k): A_KCONTIG ? srcA.load4(m, k) along k : srcA.load4(k, m) along m
// B(k,n): B_KCONTIG ? srcB.load4(n, k) along k : srcB.load4(k, n) along n
// The contraction range of block z is [z*kchunk, min((z+1)*kchunk, K)), or, in a grouped launch
// (g_beg non-null), [g_beg[z], g_end[z]) with the epilogue bound to group g_id[z].
template <class SA, bool A_KCONTIG, class SB, bool B_KCONTIG, class EPI>
__global__ __launch_bounds__(GT) void k_gemm(SA srcA, SB srcB, EPI epi, int64_t K, int64_t kchunk,
                                             const int32_t *__restrict__ g_id = nullptr,
                                             const int32_t *__restrict__ g_beg = nullptr,
                                             const int32_t *__restrict__ g_end = nullptr,
                                             const int32_t *__restrict__ mt_id = nullptr,
                                             const int32_t *__restrict__ mt_beg = nullptr,
                                             const int32_t *__restrict__ mt_end = nullptr)
{
    __shared__ __attribute__((aligned(16))) float As[BK][BM + PADL];
    __shared__ __attribute__((aligned(16))) float Bs[BK][BN + PADL];

    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int wm = w >> 1, wn = w & 1;
    // row tiles: blockIdx.x * BM, or, with a tile list (mt_beg non-null), rows [mt_beg[x], mt_end[x]) of
    // group mt_id[x] (at most BM rows): A and the output are cut at the tile's end, B is the group's matrix
    int64_t m0 = (int64_t)blockIdx.x * BM;
    if (mt_beg) {
        m0 = mt_beg[blockIdx.x];
        const int64_t me = mt_end[blockIdx.x];
        srcA.limit_rows(me); epi.limit_rows(me); srcB.bind(mt_id[blockIdx.x]);
    }
    const int32_t n0 = blockIdx.y * BN;
    int64_t kbeg = (int64_t)blockIdx.z * kchunk;
    int64_t kend = (kbeg + kchunk < K) ? kbeg + kchunk : K;
    if (g_beg) { kbeg = g_beg[blockIdx.z]; kend = g_end[blockIdx.z]; epi.bind(g_id[blockIdx.z]); }

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // ---- global -> registers: the chunk after the one being multiplied is always in flight
    float4 ra[2], rb[2];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int ps = 0; ps < 2; ++ps) {
            if (A_KCONTIG) {
                int m = (t >> 2) + ps * 64, k4 = (t & 3) * 4;
                ra[ps] = (k0 + k4 < kend) ? srcA.load4(m0 + m, (int32_t)(k0 + k4)) : make_float4(0.f, 0.f, 0.f, 0.f);
            } else {
                int k = (t >> 5) + ps * 8, m4 = (t & 31) * 4;
                ra[ps] = (k0 + k < kend) ? srcA.load4(k0 + k, (int32_t)(m0 + m4)) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
            if (B_KCONTIG) {
                int n = (t >> 2) + ps * 64, k4 = (t & 3) * 4;
                rb[ps] = (k0 + k4 < kend) ? srcB.load4(n0 + n, (int32_t)(k0 + k4)) : make_float4(0.f, 0.f, 0.f, 0.f);
            } else {
                int k = (t >> 5) + ps * 8, n4 = (t & 31) * 4;
                rb[ps] = (k0 + k < kend) ? srcB.load4(k0 + k, n0 + n4) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    };
    if (kbeg < kend) fetch(kbeg);
    for (int64_t k0 = kbeg; k0 < kend; k0 += BK) {
        __syncthreads();      // previous tile fully consumed
#pragma unroll
        for (int ps = 0; ps < 2; ++ps) {
            if (A_KCONTIG) {
                int m = (t >> 2) + ps * 64, k4 = (t & 3) * 4;
                As[k4 + 0][m] = ra[ps].x; As[k4 + 1][m] = ra[ps].y;
                As[k4 + 2][m] = ra[ps].z; As[k4 + 3][m] = ra[ps].w;
            } else {
                int k = (t >> 5) + ps * 8, m4 = (t & 31) * 4;
                *reinterpret_cast<float4 *>(&As[k][m4]) = ra[ps];
            }
            if (B_KCONTIG) {
                int n = (t >> 2) + ps * 64, k4 = (t & 3) * 4;
                Bs[k4 + 0][n] = rb[ps].x; Bs[k4 + 1][n] = rb[ps].y;
                Bs[k4 + 2][n] = rb[ps].z; Bs[k4 + 3][n] = rb[ps].w;
            } else {
                int k = (t >> 5) + ps * 8, n4 = (t & 31) * 4;
                *reinterpret_cast<float4 *>(&Bs[k][n4]) = rb[ps];
            }
        }
        __syncthreads();
        if (k0 + BK < kend) fetch(k0 + BK);
        // ---- LDS -> matrix cores.  32x32x2: lane l supplies A[m = l%32][k = l/32], B[k = l/32][n = l%32]
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            int ka = kk + (lane >> 5);
            float a0 = As[ka][wm * 64 + (lane & 31)];
            float a1 = As[ka][wm * 64 + 32 + (lane & 31)];
            float b0 = Bs[ka][wn * 64 + (lane & 31)];
            float b1 = Bs[ka][wn * 64 + 32 + (lane & 31)];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
    }
    // ---- epilogue.  D register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32.
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int row = wm * 64 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                int col = wn * 64 + j * 32 + (lane & 31);
                epi.store(m0 + row, n0 + col, acc[i][j][v]);
            }
}

__global__ void k_zero16(float4 *p, int64_t n4)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n4; i += stride) p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

__global__ void k_zero4(uint32_t *p, int64_t n)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0u;
}

}  // namespace

// Zero `bytes` bytes (a multiple of 4, 4-byte aligned) with a fill kernel; no memset nodes,
// so callers may capture the step in a HIP graph.
int launch_fill_zero(void *ptr, size_t bytes, hipStream_t st)
{
    if (bytes == 0) return KGE_OK;
    KGE_REQUIRE(((uintptr_t)ptr % 4) == 0 && bytes % 4 == 0, KGE_EINVAL,
                "zero fill needs a 4-byte aligned buffer and size");
    KGE_PROF("zero", st);
    if (((uintptr_t)ptr % 16) == 0 && bytes % 16 == 0) {
        int64_t n4 = (int64_t)(bytes / 16);
        int64_t blocks = cdiv(n4, 256);
        if (blocks > 65536) blocks = 65536;
        k_zero16<<<(unsigned)blocks, 256, 0, st>>>(reinterpret_cast<float4 *>(ptr), n4);
    } else {
        int64_t n = (int64_t)(bytes / 4);
        int64_t blocks = cdiv(n, 256);
        if (blocks > 65536) blocks = 65536;
        k_zero4<<<(unsigned)blocks, 256, 0, st>>>(reinterpret_cast<uint32_t *>(ptr), n);
    }
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

int launch_project(const float *H, int64_t N, int32_t d_in, int32_t d_out, int32_t B, const float *V,
                   const float *W0, float *P, float *Self, hipStream_t st)
{
    if (N == 0) return KGE_OK;
    int32_t nc = (B + 1) * d_out;
    dim3 grid((unsigned)cdiv(N, BM), (unsigned)cdiv(nc, BN), 1);
    SrcRowMajorF32 sa{H, N, d_in};
    SrcWcat sb{V, W0, d_in, d_out, B};
    KGE_PROF("project", st);
    EpiProject ep{P, Self, N, d_out, B};
    k_gemm<SrcRowMajorF32, true, SrcWcat, false, EpiProject><<<grid, GT, 0, st>>>(sa, sb, ep, d_in, d_in);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

int launch_weight_grad(const float *H, int64_t N, int32_t d_in, int32_t d_out, int32_t B,
                       const float *dP, const float *G, float *dV, float *dW0, hipStream_t st)
{
    int rc = launch_fill_zero(dV, sizeof(float) * (size_t)B * d_in * d_out, st);
    if (rc != KGE_OK) return rc;
    rc = launch_fill_zero(dW0, sizeof(float) * (size_t)d_in * d_out, st);
    if (rc != KGE_OK) return rc;
    if (N == 0) return KGE_OK;
    int32_t nc = (B + 1) * d_out;
    int64_t tiles = cdiv(d_in, BM) * cdiv(nc, BN);
    // split the N-long contraction so that roughly 2048 blocks are in flight
    int64_t splits = cdiv(2048, tiles);
    int64_t kchunk = cdiv(cdiv(N, splits), BK) * BK;
    if (kchunk < 4 * BK) kchunk = 4 * BK;
    splits = cdiv(N, kchunk);
    dim3 grid((unsigned)cdiv(d_in, BM), (unsigned)cdiv(nc, BN), (unsigned)splits);
    SrcRowMajorF32 sa{H, N, d_in};
    EpiWeightGrad ep{dV, dW0, d_in, d_out, B};
    KGE_PROF("weight_grad", st);
    SrcXcat sb{dP, G, N, d_out, B};
    k_gemm<SrcRowMajorF32, false, SrcXcat, false, EpiWeightGrad><<<grid, GT, 0, st>>>(sa, sb, ep, N, kchunk);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

int launch_input_grad(const float *dP, const float *G, int64_t N, int32_t d_in,
                      int32_t d_out, int32_t B, const float *V, const float *W0, float *dH,
                      hipStream_t st)
{
    if (N == 0) return KGE_OK;
    int32_t nc = (B + 1) * d_out;
    dim3 grid((unsigned)cdiv(N, BM), (unsigned)cdiv(d_in, BN), 1);
    SrcWcat sb{V, W0, d_in, d_out, B};
    EpiRowMajor ep{dH, N, d_in};
    KGE_PROF("input_grad", st);
    SrcXcat sa{dP, G, N, d_out, B};
    k_gemm<SrcXcat, true, SrcWcat, true, EpiRowMajor><<<grid, GT, 0, st>>>(sa, sb, ep, nc, nc);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

int launch_rel_outer(const kge_partition *p, const float *Z, const float *G, int32_t d_in, int32_t d_out,
                     float *C, hipStream_t st)
{
    const int64_t R2 = 2 * (int64_t)p->n_relations;
    const int64_t dd = (int64_t)d_in * d_out;
    int rc = launch_fill_zero(C, sizeof(float) * (size_t)R2 * dd, st);
    if (rc != KGE_OK) return rc;
    if (p->n_seg == 0 || p->n_relc == 0) return KGE_OK;
    KGE_REQUIRE(p->n_relc <= 65535, KGE_ERANGE, "too many relation chunks (%d) for one launch", p->n_relc);
    {
        dim3 grid((unsigned)cdiv(d_in, BM), (unsigned)cdiv(d_out, BN), (unsigned)p->n_relc);
        SrcRowMajorF32 sa{Z, p->n_seg, d_in};
        SrcGatherRows sb{G, p->seg_dst, p->n_seg, d_out};
        EpiRelOuter ep{C, d_in, d_out, 0};
        KGE_PROF("rel_outer", st);
        k_gemm<SrcRowMajorF32, false, SrcGatherRows, false, EpiRelOuter><<<grid, GT, 0, st>>>(
            sa, sb, ep, p->n_seg, 0, p->relc_rel, p->relc_beg, p->relc_end);
        KGE_LAUNCH_CHECK();
    }
    return KGE_OK;
}

int launch_coeff_contract(const kge_partition *p, const float *C, const float *V, int32_t d_in, int32_t d_out,
                          int32_t B, float *da, hipStream_t st)
{
    const int64_t R2 = 2 * (int64_t)p->n_relations;
    const int64_t dd = (int64_t)d_in * d_out;
    int rc = launch_fill_zero(da, sizeof(float) * (size_t)R2 * B, st);
    if (rc != KGE_OK) return rc;
    if (p->n_seg == 0) return KGE_OK;
    {
        const int64_t tiles = cdiv(R2, BM) * cdiv(B, BN);
        int64_t splits = cdiv(512, tiles);
        int64_t kchunk = cdiv(cdiv(dd, splits), BK) * BK;
        if (kchunk < 4 * BK) kchunk = 4 * BK;
        splits = cdiv(dd, kchunk);
        dim3 grid((unsigned)cdiv(R2, BM), (unsigned)cdiv(B, BN), (unsigned)splits);
        SrcRowMajorF32 sa{C, R2, (int32_t)dd};
        SrcRowMajorF32 sb{V, B, (int32_t)dd};
        EpiRowMajorAtomic ep{da, R2, B};
        KGE_PROF("coeff_contract", st);
        k_gemm<SrcRowMajorF32, true, SrcRowMajorF32, true, EpiRowMajorAtomic><<<grid, GT, 0, st>>>(sa, sb, ep, dd, kchunk);
        KGE_LAUNCH_CHECK();
    }
    return KGE_OK;
}

// ---- relation-weight order ------------------------------------------------------------------
namespace {

// out[i][x] = sum_k c[i][k] M[k][x]   (c is [ni][nk])
// One block: 16 rows i, 1024 columns x (4 per thread); M is read once per 16 rows.
__global__ __launch_bounds__(256) void k_lincomb(const float *__restrict__ c, int32_t ni, int32_t nk,
                                                 const float *__restrict__ M, int64_t nx, float *__restrict__ out)
{
    __shared__ float sc[16][64];
    const int i0 = blockIdx.y * 16;
    const int64_t x = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    float4 acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int k0 = 0; k0 < nk; k0 += 64) {
        __syncthreads();
        for (int q = threadIdx.x; q < 16 * 64; q += 256) {
            const int j = q >> 6, kk = q & 63;
            const int i = i0 + j, k = k0 + kk;
            sc[j][kk] = (i < ni && k < nk) ? c[(int64_t)i * nk + k] : 0.f;
        }
        __syncthreads();
        const int kn = min(64, nk - k0);
        if (x < nx)
            for (int kk = 0; kk < kn; ++kk) {
                const float4 m = *reinterpret_cast<const float4 *>(M + (int64_t)(k0 + kk) * nx + x);
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const float w = sc[j][kk];
                    acc[j].x = fmaf(w, m.x, acc[j].x); acc[j].y = fmaf(w, m.y, acc[j].y);
                    acc[j].z = fmaf(w, m.z, acc[j].z); acc[j].w = fmaf(w, m.w, acc[j].w);
                }
            }
    }
    if (x < nx)
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (i0 + j < ni) *reinterpret_cast<float4 *>(out + (int64_t)(i0 + j) * nx + x) = acc[j];
}

}  // namespace

// Wrel[r] = sum_b a[r][b] V_b   ([2R][d_in*d_out] floats): Eq. 2 written out for every relation
int launch_relation_weights(const float *a, int32_t R2, int32_t B, const float *V, int64_t dd, float *Wrel,
                            hipStream_t st)
{
    if (R2 == 0) return KGE_OK;
    dim3 grid((unsigned)cdiv(dd, 1024), (unsigned)cdiv(R2, 16), 1);
    KGE_PROF("rel_weights", st);
    k_lincomb<<<grid, 256, 0, st>>>(a, R2, B, V, dd, Wrel);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

namespace {

// dV[b][x] += sum_{r in this block's chunk} a[r][b] C[r][x] for BB bases b at once: the block's 256 columns of C
// are read once for all of them (C, one matrix per relation, is the big operand).  A row's BB coefficients are
// uniform over the block and contiguous: they arrive through scalar loads and enter the multiply-adds as scalar
// operands.
template <int BB>
__global__ __launch_bounds__(256) void k_basis_grad_cols(const float *__restrict__ a, int32_t R2, int32_t B,
                                                         int32_t b_base, const float *__restrict__ C, int64_t nx,
                                                         int32_t rchunk, float *__restrict__ dV)
{
    const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int b0 = b_base + blockIdx.z * BB;
    const int rb = blockIdx.y * rchunk, re = min(rb + rchunk, R2);
    const bool in = x < nx;
    const float *cp = C + (in ? x : 0);
    float acc[BB];
#pragma unroll
    for (int j = 0; j < BB; ++j) acc[j] = 0.f;
    int r = rb;
    for (; r + 4 <= re; r += 4) {
        float c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) c[u] = cp[(int64_t)(r + u) * nx];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float *ar = a + (int64_t)(r + u) * B + b0;
#pragma unroll
            for (int j = 0; j < BB; ++j) acc[j] = fmaf(ar[j], c[u], acc[j]);
        }
    }
    for (; r < re; ++r) {
        const float c = cp[(int64_t)r * nx];
        const float *ar = a + (int64_t)r * B + b0;
#pragma unroll
        for (int j = 0; j < BB; ++j) acc[j] = fmaf(ar[j], c, acc[j]);
    }
    if (in)
#pragma unroll
        for (int j = 0; j < BB; ++j) atomicAdd(dV + (int64_t)(b0 + j) * nx + x, acc[j]);
}

template <int BB>
int basis_grad_groups(const float *a, int32_t R2, int32_t B, int32_t &b_done, const float *C, int64_t dd, float *dV,
                      hipStream_t st)
{
    const int64_t zb = (B - b_done) / BB;
    if (zb == 0) return KGE_OK;
    // the sum over relations is cut into chunks so that about 1536 blocks run (six per compute unit are resident
    // at once: one round of blocks, no tail); their partial sums meet in dV
    const int64_t xb = cdiv(dd, 256);
    int64_t chunks = cdiv(1536, xb * zb);
    if (chunks > cdiv(R2, 16)) chunks = cdiv(R2, 16);
    const int32_t rchunk = (int32_t)cdiv(R2, chunks);
    KGE_REQUIRE(xb <= 0x7fffffffLL && zb <= 65535, KGE_ERANGE, "basis gradient: too many columns or bases");
    dim3 grid((unsigned)xb, (unsigned)cdiv(R2, rchunk), (unsigned)zb);
    k_basis_grad_cols<BB><<<grid, 256, 0, st>>>(a, R2, B, b_done, C, dd, rchunk, dV);
    KGE_LAUNCH_CHECK();
    b_done += (int32_t)zb * BB;
    return KGE_OK;
}

}  // namespace

// dV_b = sum_r a[r][b] C[r]   (the chain rule on Wrel[r] = sum_b a[r][b] V_b with dWrel = C)
// Groups of 64 bases per block, then what is left in groups of 16, 4 and 1.
int launch_basis_grad_from_relations(const float *a, int32_t R2, int32_t B, const float *C, int64_t dd, float *dV,
                                     hipStream_t st)
{
    int rc = launch_fill_zero(dV, sizeof(float) * (size_t)B * dd, st);
    if (rc != KGE_OK || R2 == 0 || B == 0) return rc;
    KGE_PROF("basis_grad", st);
    int32_t b_done = 0;
    rc = basis_grad_groups<64>(a, R2, B, b_done, C, dd, dV, st);
    if (rc == KGE_OK) rc = basis_grad_groups<16>(a, R2, B, b_done, C, dd, dV, st);
    if (rc == KGE_OK) rc = basis_grad_groups<4>(a, R2, B, b_done, C, dd, dV, st);
    if (rc == KGE_OK) rc = basis_grad_groups<1>(a, R2, B, b_done, C, dd, dV, st);
    return rc;
}

// U[s] = Z[s] Wrel[rel(s)]   (S x d_in) -> (S x d_out), one row tile per (relation, <= 128 runs)
int launch_apply_relation_weights(const kge_partition *p, const float *Z, const float *Wrel, int32_t d_in,
                                  int32_t d_out, float *U, hipStream_t st)
{
    if (p->n_relt == 0) return KGE_OK;
    KGE_REQUIRE(cdiv(d_out, BN) <= 65535, KGE_ERANGE, "d_out too large");
    dim3 grid((unsigned)p->n_relt, (unsigned)cdiv(d_out, BN), 1);
    SrcRowMajorF32 sa{Z, p->n_seg, d_in};
    SrcGroupMat sb{Wrel, d_in, d_out};
    EpiRowMajor ep{U, p->n_seg, d_out};
    KGE_PROF("apply_rel", st);
    k_gemm<SrcRowMajorF32, true, SrcGroupMat, false, EpiRowMajor><<<grid, GT, 0, st>>>(
        sa, sb, ep, d_in, d_in, nullptr, nullptr, nullptr, p->relt_rel, p->relt_beg, p->relt_end);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

// dZ[s] = G[dst(s)] Wrel[rel(s)]^T   (S x d_out) -> (S x d_in)
int launch_apply_relation_weights_t(const kge_partition *p, const float *G, const float *Wrel, int32_t d_in,
                                    int32_t d_out, float *dZ, hipStream_t st)
{
    if (p->n_relt == 0) return KGE_OK;
    dim3 grid((unsigned)p->n_relt, (unsigned)cdiv(d_in, BN), 1);
    SrcGatherRows sa{G, p->seg_dst, p->n_seg, d_out};
    SrcGroupMat sb{Wrel, d_in, d_out};
    EpiRowMajor ep{dZ, p->n_seg, d_in};
    KGE_PROF("apply_rel_t", st);
    k_gemm<SrcGatherRows, true, SrcGroupMat, true, EpiRowMajor><<<grid, GT, 0, st>>>(
        sa, sb, ep, d_out, d_out, nullptr, nullptr, nullptr, p->relt_rel, p->relt_beg, p->relt_end);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}
