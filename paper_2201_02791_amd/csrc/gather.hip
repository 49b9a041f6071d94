// Neighbour aggregation of the RGCN layer (Eq. 1 with W_r = sum_b a_rb V_b, Eq. 2) and
// its backward counterparts.  All kernels here are bandwidth bound: they stream rows of
// the projected messages P[j][b][:] (or of the upstream gradient G) with 128-bit loads and do
// a handful of fp32 FMAs per loaded element.
//
// Work decomposition.  One wavefront per row (destination, source, or (relation, destination)
// run).  Rows with >= KGE_HEAVY edges are cut into units of KGE_HEAVY edges, one wavefront
// each, placed first in the grid; a unit writes a partial sum and a small finishing kernel adds
// the partials of a row in unit order.  No atomics: results are bit-reproducible.
//
// Lane layout.  A row of `d` elements is covered by LPR lanes, each holding VEC consecutive
// elements (VEC = 4 for fp32, 8 for bf16: one 16-byte load).  The 64 / LPR lane groups of a
// wavefront work on different (edge, basis) pairs in parallel: GB of them across bases,
// GE = groups / GB across edges.
#include "common.h"

namespace {

constexpr int WPB = 4;                 // wavefronts per block

template <bool BF16> struct MsgRow;
template <> struct MsgRow<false> {
    static constexpr int VEC = 4;
    static __device__ __forceinline__ uint4 load_raw(const void *base, int64_t off)
    {
        return *reinterpret_cast<const uint4 *>(reinterpret_cast<const float *>(base) + off);
    }
    static __device__ __forceinline__ void unpack(const uint4 &x, float (&v)[4])
    {
        v[0] = __uint_as_float(x.x); v[1] = __uint_as_float(x.y);
        v[2] = __uint_as_float(x.z); v[3] = __uint_as_float(x.w);
    }
};
template <> struct MsgRow<true> {
    static constexpr int VEC = 8;
    static __device__ __forceinline__ uint4 load_raw(const void *base, int64_t off)
    {
        return *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(base) + off);
    }
    static __device__ __forceinline__ void unpack(const uint4 &x, float (&v)[8])
    {
        v[0] = __uint_as_float(x.x << 16); v[1] = __uint_as_float(x.x & 0xffff0000u);
        v[2] = __uint_as_float(x.y << 16); v[3] = __uint_as_float(x.y & 0xffff0000u);
        v[4] = __uint_as_float(x.z << 16); v[5] = __uint_as_float(x.z & 0xffff0000u);
        v[6] = __uint_as_float(x.w << 16); v[7] = __uint_as_float(x.w & 0xffff0000u);
    }
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)   // two fp32 -> packed bf16x2, nearest even
{
    // one v_cvt_pk_bf16_f32 on gfx950
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float floatx2_t __attribute__((ext_vector_type(2)));
    const floatx2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ float act_apply(int act, float x) { return act == KGE_ACT_RELU ? fmaxf(x, 0.f) : x; }

// Which row and edge range a wavefront works on.  Wavefronts [0, n_units) take the units of heavy
// rows; wavefront n_units + r takes light row r (and leaves at once if r is heavy).
struct RowWork {
    int64_t row;       // row id, or -1: nothing to do
    int32_t beg, end;  // edge range
    int32_t unit;      // >= 0: partial result goes to slot `unit`; -1: the row is finished here
};
__device__ __forceinline__ RowWork row_work(int64_t wid, const int32_t *__restrict__ ptr, int64_t n_rows,
                                            int32_t n_units, const int32_t *__restrict__ hv_row,
                                            const int32_t *__restrict__ hv_unit_ptr,
                                            const int32_t *__restrict__ unit_hv)
{
    RowWork w;
    if (wid < n_units) {
        const int32_t h = unit_hv[wid];
        w.row = hv_row[h];
        w.unit = (int32_t)wid;
        w.beg = ptr[w.row] + (int32_t)(wid - hv_unit_ptr[h]) * KGE_HEAVY;
        w.end = min(w.beg + KGE_HEAVY, ptr[w.row + 1]);
        return w;
    }
    w.row = wid - n_units;
    w.unit = -1;
    if (w.row >= n_rows) { w.row = -1; w.beg = w.end = 0; return w; }
    w.beg = ptr[w.row];
    w.end = ptr[w.row + 1];
    if (w.end - w.beg >= KGE_HEAVY) w.row = -1;
    return w;
}

// ------------------------------------------------------------------ forward
//   out[i][:] = act( sum_e invc_e sum_b a[rel_e][b] P[src_e][b][:] + Self[i][:] )
// PLAIN (B = 1, no coefficient table, dm_rel unused): out[i] = act( sum_e w_e P[idx_e] + Self[i] ),
// w = 1 if dm_invc is null.
template <bool BF16, int LPR, bool PLAIN>
__global__ __launch_bounds__(64 * WPB) void k_gather_fwd(
    const int32_t *__restrict__ dm_ptr, const int32_t *__restrict__ dm_src,
    const int32_t *__restrict__ dm_rel, const float *__restrict__ dm_invc, int64_t N,
    int32_t n_units, const int32_t *__restrict__ hv_row, const int32_t *__restrict__ hv_unit_ptr,
    const int32_t *__restrict__ unit_hv,
    const void *__restrict__ P, const float *__restrict__ a, int32_t B, int32_t d, int32_t gb_count,
    const float *__restrict__ Self, int act, float *__restrict__ out, float *__restrict__ out2,
    uint16_t *__restrict__ outbf, float *__restrict__ partial, const uint8_t *__restrict__ active)
{
    // outbf (optional): a bf16 copy of the output rows (the next layer's bf16 input, written here instead of by a
    // conversion pass over `out`)
    constexpr int VEC = MsgRow<BF16>::VEC;
    constexpr int G = 64 / LPR;
    constexpr int U = 8;
    const int lane = threadIdx.x & 63;
    const int64_t wid = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
    const int kl = lane % LPR, g = lane / LPR;
    if (active && wid >= n_units && wid - n_units < N && !active[wid - n_units]) {
        // a row outside the batch's sub-graph, seen before its edge range is even fetched: a zero row
        // (a heavy row's zeros are written once more by the finishing kernel)
        if (g == 0 && kl * VEC < d) {
            const int64_t o = (wid - n_units) * d + kl * VEC;
#pragma unroll
            for (int v4 = 0; v4 < VEC; v4 += 4) {
                *reinterpret_cast<float4 *>(out + o + v4) = make_float4(0.f, 0.f, 0.f, 0.f);
                if (out2) *reinterpret_cast<float4 *>(out2 + o + v4) = make_float4(0.f, 0.f, 0.f, 0.f);
                if (outbf) *reinterpret_cast<uint2 *>(outbf + o + v4) = make_uint2(0u, 0u);
            }
        }
        return;
    }
    const RowWork rw = row_work(wid, dm_ptr, N, n_units, hv_row, hv_unit_ptr, unit_hv);
    if (rw.row < 0) return;                             // whole wavefront leaves together
    if (active && !active[rw.row]) {                    // a unit of a heavy row outside the sub-graph
        if (rw.unit < 0 && g == 0 && kl * VEC < d) {
            const int64_t o = rw.row * d + kl * VEC;
#pragma unroll
            for (int v4 = 0; v4 < VEC; v4 += 4) {
                *reinterpret_cast<float4 *>(out + o + v4) = make_float4(0.f, 0.f, 0.f, 0.f);
                if (out2) *reinterpret_cast<float4 *>(out2 + o + v4) = make_float4(0.f, 0.f, 0.f, 0.f);
                if (outbf) *reinterpret_cast<uint2 *>(outbf + o + v4) = make_uint2(0u, 0u);
            }
        }
        return;
    }
    const int GB = gb_count, GE = G / GB;
    const int gb = g % GB, ge = g / GB;
    const bool kact = kl * VEC < d;
    const int nb = (B + GB - 1) / GB;                   // basis slots per edge for this group

    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
    // the row's self-loop part is fetched ahead of the edges (it is only needed at the end; loaded there it would
    // add one more memory round trip to every wavefront)
    float4 selfv[VEC / 4];
#pragma unroll
    for (int v4 = 0; v4 < VEC / 4; ++v4) selfv[v4] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (g == 0 && kact && rw.unit < 0) {
#pragma unroll
        for (int v4 = 0; v4 < VEC / 4; ++v4)
            selfv[v4] = *reinterpret_cast<const float4 *>(Self + rw.row * d + kl * VEC + 4 * v4);
    }

    for (int32_t e0 = rw.beg; e0 < rw.end; e0 += 64) {
        const int cnt = min(64, rw.end - e0);
        int32_t my_src = 0, my_rel = 0;
        float my_w = 0.f;
        if (lane < cnt) {
            my_src = dm_src[e0 + lane];
            if (PLAIN) {
                my_w = dm_invc ? dm_invc[e0 + lane] : 1.f;
            } else {
                my_rel = dm_rel[e0 + lane];
                my_w = dm_invc[e0 + lane];
            }
        }
        const int erounds = (cnt + GE - 1) / GE;        // uniform trip counts for all lanes
        const int items = erounds * nb;
        int er = 0, bi = 0;                             // current (edge round, basis slot)
        for (int q0 = 0; q0 < items; q0 += U) {
            float coef[U];
            uint4 raw[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int el = er * GE + ge;
                const int b = bi * GB + gb;
                // a slot past the end repeats the chunk's first edge with coefficient 0, and a lane past the
                // row's width reads its start: every load is unconditional (no divergent branch around it)
                const bool ok = (q0 + u < items) && el < cnt && b < B;
                const int els = ok ? el : 0, bs = ok ? b : 0;
                const int32_t src = __shfl(my_src, els, 64);
                const int32_t rel = __shfl(my_rel, els, 64);
                const float w = __shfl(my_w, els, 64);
                const float cf = PLAIN ? w : a[(int64_t)rel * B + bs] * w;
                coef[u] = ok ? cf : 0.f;
                raw[u] = MsgRow<BF16>::load_raw(P, ((int64_t)src * B + bs) * d + (kact ? kl * VEC : 0));
                if (++bi == nb) { bi = 0; ++er; }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float val[VEC];
                MsgRow<BF16>::unpack(raw[u], val);
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[v] = fmaf(coef[u], val[v], acc[v]);
            }
        }
    }
    // fold the lane groups together (fixed order: deterministic)
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] += __shfl_xor(acc[v], off, 64);

    if (g == 0 && kact) {
        if (rw.unit >= 0) {
            float *q = partial + (int64_t)rw.unit * d + kl * VEC;
#pragma unroll
            for (int v4 = 0; v4 < VEC; v4 += 4)
                *reinterpret_cast<float4 *>(q + v4) = make_float4(acc[v4], acc[v4 + 1], acc[v4 + 2], acc[v4 + 3]);
            return;
        }
        const int64_t o = rw.row * d + kl * VEC;
#pragma unroll
        for (int v4 = 0; v4 < VEC; v4 += 4) {
            const float4 s = selfv[v4 / 4];
            float4 r = make_float4(act_apply(act, acc[v4] + s.x), act_apply(act, acc[v4 + 1] + s.y),
                                   act_apply(act, acc[v4 + 2] + s.z), act_apply(act, acc[v4 + 3] + s.w));
            *reinterpret_cast<float4 *>(out + o + v4) = r;
            if (out2) *reinterpret_cast<float4 *>(out2 + o + v4) = r;
            if (outbf) *reinterpret_cast<uint2 *>(outbf + o + v4) = make_uint2(pack_bf16x2(r.x, r.y), pack_bf16x2(r.z, r.w));
        }
    }
}

// Heavy destinations: out[i] = act(sum of the row's unit partials + Self[i]).  One thread per float4.
__global__ void k_gather_fwd_finish(int32_t n_hv, const int32_t *__restrict__ hv_row,
                                    const int32_t *__restrict__ hv_unit_ptr, const float *__restrict__ partial,
                                    int32_t d, const float *__restrict__ Self, int act,
                                    float *__restrict__ out, float *__restrict__ out2,
                                    uint16_t *__restrict__ outbf, const uint8_t *__restrict__ active)
{
    const int d4 = d >> 2;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)n_hv * d4) return;
    const int32_t h = (int32_t)(idx / d4);
    const int k4 = (int)(idx - (int64_t)h * d4) * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (active && !active[hv_row[h]]) {
        const int64_t oz = (int64_t)hv_row[h] * d + k4;
        *reinterpret_cast<float4 *>(out + oz) = s;
        if (out2) *reinterpret_cast<float4 *>(out2 + oz) = s;
        if (outbf) *reinterpret_cast<uint2 *>(outbf + oz) = make_uint2(0u, 0u);
        return;
    }
    for (int32_t u = hv_unit_ptr[h]; u < hv_unit_ptr[h + 1]; ++u) {
        const float4 x = *reinterpret_cast<const float4 *>(partial + (int64_t)u * d + k4);
        s.x += x.x; s.y += x.y; s.z += x.z; s.w += x.w;
    }
    const int64_t o = (int64_t)hv_row[h] * d + k4;
    const float4 sf = *reinterpret_cast<const float4 *>(Self + o);
    const float4 r = make_float4(act_apply(act, s.x + sf.x), act_apply(act, s.y + sf.y),
                                 act_apply(act, s.z + sf.z), act_apply(act, s.w + sf.w));
    *reinterpret_cast<float4 *>(out + o) = r;
    if (out2) *reinterpret_cast<float4 *>(out2 + o) = r;
    if (outbf) *reinterpret_cast<uint2 *>(outbf + o) = make_uint2(pack_bf16x2(r.x, r.y), pack_bf16x2(r.z, r.w));
}

// ------------------------------------------------------------------ activation backward
__global__ void k_act_backward(const float4 *__restrict__ dH, const float4 *__restrict__ Hout, int act,
                               int64_t n4, float4 *__restrict__ G)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n4; i += stride) {
        float4 g = dH[i];
        if (act == KGE_ACT_RELU) {
            float4 h = Hout[i];
            g.x = h.x > 0.f ? g.x : 0.f; g.y = h.y > 0.f ? g.y : 0.f;
            g.z = h.z > 0.f ? g.z : 0.f; g.w = h.w > 0.f ? g.w : 0.f;
        }
        G[i] = g;
    }
}

// ------------------------------------------------------------------ transposed gather
// One wavefront per (source row work, chunk of bases) on the source-major view:
//   dP[j][b][:] = sum_{e out of j} a[rel_e][b] invc_e G[dst_e][:]
// A G row (fp32) is covered by LPR lanes x 4 floats.  Of the 64/LPR lane groups, GBT take
// different bases (NB bases each, so a chunk is GBT*NB bases) and the other 64/(LPR*GBT) take
// different edges; UE rounds of edges are in flight at a time.
// GIN: the gathered rows are bf16 instead of fp32.
template <bool BF16, bool GIN, int LPR, int NB, int UE>
__global__ __launch_bounds__(64 * WPB) void k_gather_t(
    const int32_t *__restrict__ sm_ptr, const int32_t *__restrict__ sm_dst,
    const int32_t *__restrict__ sm_rel, const float *__restrict__ sm_invc, int64_t N,
    int32_t n_units, const int32_t *__restrict__ hv_row, const int32_t *__restrict__ hv_unit_ptr,
    const int32_t *__restrict__ unit_hv,
    const void *__restrict__ Gv, const float *__restrict__ a, int32_t B, int32_t d, int32_t n_chunks,
    int32_t gbt_count, void *__restrict__ dP, int64_t ld, float *__restrict__ partial,
    const uint8_t *__restrict__ active, const uint8_t *__restrict__ row_active)
{
    constexpr int NG = 64 / LPR;
    const int lane = threadIdx.x & 63;
    const int64_t wid_all = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
    const int64_t wid = wid_all / n_chunks;
    const int bc = (int)(wid_all - wid * n_chunks);
    const RowWork rw = row_work(wid, sm_ptr, N, n_units, hv_row, hv_unit_ptr, unit_hv);
    if (rw.row < 0) return;
    if (row_active && !row_active[rw.row]) return;       // the row is not needed: left unwritten
    const int kl = lane % LPR, g = lane / LPR;
    const int GBT = gbt_count, GET = NG / GBT;
    const int gbt = g % GBT, get = g / GBT;
    const bool kact = kl * 4 < d;
    const int b0 = (bc * GBT + gbt) * NB;

    float acc[NB][4];
#pragma unroll
    for (int n = 0; n < NB; ++n)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[n][v] = 0.f;

    for (int32_t e0 = rw.beg; e0 < rw.end; e0 += 64) {
        const int cnt = min(64, rw.end - e0);
        int32_t my_dst = 0, my_rel = 0;
        float my_w = 0.f;
        if (lane < cnt) {
            my_dst = sm_dst[e0 + lane]; my_rel = sm_rel[e0 + lane]; my_w = sm_invc ? sm_invc[e0 + lane] : 1.f;
            if (active && !active[my_dst]) my_dst = -1;   // destination outside the sub-graph: G row is zero
        }
        const int rounds = (cnt + GET - 1) / GET;       // uniform trip count
        for (int r0 = 0; r0 < rounds; r0 += UE) {
            float4 gv[UE];
            float w[UE];
            const float *arow[UE];
#pragma unroll
            for (int u = 0; u < UE; ++u) {
                const int el = (r0 + u) * GET + get;
                const bool ok = (r0 + u < rounds) && el < cnt;
                const int els = ok ? el : 0;
                int32_t dst, rel;
                float ww;
                if (NG == 1) {            // one lane group: the edge is wavefront-uniform (scalar path)
                    dst = __builtin_amdgcn_readlane(my_dst, els);
                    rel = __builtin_amdgcn_readlane(my_rel, els);
                    ww = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_w), els));
                } else {
                    dst = __shfl(my_dst, els, 64);
                    rel = __shfl(my_rel, els, 64);
                    ww = __shfl(my_w, els, 64);
                }
                // a slot without an edge (or an edge into a row outside the sub-graph) reads row 0 with weight 0,
                // a lane past the row's width its start: the load itself is unconditional
                const bool live = ok && dst >= 0;
                w[u] = live ? ww : 0.f;
                arow[u] = a + (int64_t)rel * B;
                const int64_t goff = (int64_t)(live ? dst : 0) * d + (kact ? kl * 4 : 0);
                if (GIN) {
                    const uint2 x = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(Gv) + goff);
                    gv[u] = make_float4(__uint_as_float(x.x << 16), __uint_as_float(x.x & 0xffff0000u),
                                        __uint_as_float(x.y << 16), __uint_as_float(x.y & 0xffff0000u));
                } else {
                    gv[u] = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(Gv) + goff);
                }
            }
#pragma unroll
            for (int u = 0; u < UE; ++u)
#pragma unroll
                for (int n = 0; n < NB; ++n) {
                    const float cv = arow[u][b0 + n < B ? b0 + n : B - 1];
                    const float c = (b0 + n < B) ? cv * w[u] : 0.f;
                    acc[n][0] = fmaf(c, gv[u].x, acc[n][0]); acc[n][1] = fmaf(c, gv[u].y, acc[n][1]);
                    acc[n][2] = fmaf(c, gv[u].z, acc[n][2]); acc[n][3] = fmaf(c, gv[u].w, acc[n][3]);
                }
        }
    }
    // fold the edge groups together (fixed order)
    for (int off = LPR * GBT; off < 64; off <<= 1)
#pragma unroll
        for (int n = 0; n < NB; ++n)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[n][v] += __shfl_xor(acc[n][v], off, 64);
    if (!kact || get != 0) return;
#pragma unroll
    for (int n = 0; n < NB; ++n) {
        if (b0 + n >= B) continue;
        if (rw.unit >= 0) {
            *reinterpret_cast<float4 *>(partial + ((int64_t)rw.unit * B + b0 + n) * d + kl * 4) =
                make_float4(acc[n][0], acc[n][1], acc[n][2], acc[n][3]);
        } else {
            const int64_t o = (int64_t)rw.row * ld + (int64_t)(b0 + n) * d + kl * 4;
            if (BF16) {
                uint2 x;
                x.x = pack_bf16x2(acc[n][0], acc[n][1]); x.y = pack_bf16x2(acc[n][2], acc[n][3]);
                *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(dP) + o) = x;
            } else {
                *reinterpret_cast<float4 *>(reinterpret_cast<float *>(dP) + o) =
                    make_float4(acc[n][0], acc[n][1], acc[n][2], acc[n][3]);
            }
        }
    }
}

// The same transposed gather for many bases (B >= 32) on the matrix cores: for one source,
//   dP[j] (B x d) = W^T (B x deg) * Gg (deg x d),  W[e][b] = a[rel_e][b] invc_e,  Gg[e] = G[dst_e],
// a small dense product whose inner dimension is the source's out-degree.  v_mfma_f32_32x32x2_f32
// keeps fp32 inputs; one wavefront owns a (32 bases x 128 columns) block = 1 x 4 tiles and walks
// the edges two at a time (lane half h supplies edge k+h: 32 coefficients and 32 columns of G).
typedef float gt_floatx16 __attribute__((ext_vector_type(16)));

template <bool BF16, bool GIN, int NBT>
__global__ __launch_bounds__(64 * WPB) void k_gather_t_mfma(
    const int32_t *__restrict__ sm_ptr, const int32_t *__restrict__ sm_dst,
    const int32_t *__restrict__ sm_rel, const float *__restrict__ sm_invc, int64_t N,
    int32_t n_units, const int32_t *__restrict__ hv_row, const int32_t *__restrict__ hv_unit_ptr,
    const int32_t *__restrict__ unit_hv,
    const void *__restrict__ Gv, const float *__restrict__ a, int32_t B, int32_t d, int32_t n_bchunks,
    int32_t n_cchunks, void *__restrict__ dP, int64_t ld, float *__restrict__ partial,
    const uint8_t *__restrict__ active, const uint8_t *__restrict__ row_active)
{
    constexpr int UK = 4;                                  // edge pairs in flight
    __shared__ float stage[WPB][32][36];                   // one 32x32 tile per wavefront (bf16 epilogue)
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int64_t wid_all = (int64_t)blockIdx.x * WPB + wv;
    const int n_chunks = n_bchunks * n_cchunks;
    const int64_t wid = wid_all / n_chunks;
    const int chunk = (int)(wid_all - wid * n_chunks);
    const int bchunk = chunk / n_cchunks, cchunk = chunk - bchunk * n_cchunks;
    const RowWork rw = row_work(wid, sm_ptr, N, n_units, hv_row, hv_unit_ptr, unit_hv);
    if (rw.row < 0) return;
    if (row_active && !row_active[rw.row]) return;
    const int h = lane >> 5, l32 = lane & 31;
    const int bbase = bchunk * 32 * NBT, cbase = cchunk * 128;

    gt_floatx16 acc[NBT][4];
#pragma unroll
    for (int t = 0; t < NBT; ++t)
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][c][v] = 0.f;

    for (int32_t e0 = rw.beg; e0 < rw.end; e0 += 64) {
        const int cnt = min(64, rw.end - e0);
        int32_t my_dst = 0, my_rel = 0;
        float my_w = 0.f;
        if (lane < cnt) {
            my_dst = sm_dst[e0 + lane]; my_rel = sm_rel[e0 + lane]; my_w = sm_invc ? sm_invc[e0 + lane] : 1.f;
            if (active && !active[my_dst]) my_dst = -1;   // destination outside the sub-graph: G row is zero
        }
        for (int k0 = 0; k0 < cnt; k0 += 2 * UK) {
            float wa[UK][NBT], gb[UK][4];
#pragma unroll
            for (int u = 0; u < UK; ++u) {
                const int el = k0 + 2 * u + h;
                const bool ok = el < cnt;
                const int els = ok ? el : 0;
                const int32_t dst = __shfl(my_dst, els, 64);
                const int32_t rel = __shfl(my_rel, els, 64);
                const float wsh = __shfl(my_w, els, 64);       // every lane takes part: a shuffle under a
                const bool live = ok && dst >= 0;              // condition would read zeros from idle lanes
                const float ww = live ? wsh : 0.f;
#pragma unroll
                for (int t = 0; t < NBT; ++t) {
                    const int b = bbase + t * 32 + l32;
                    wa[u][t] = (live && b < B) ? a[(int64_t)rel * B + b] * ww : 0.f;
                }
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int col = cbase + c * 32 + l32;
                    gb[u][c] = 0.f;
                    if (live && col < d)
                        gb[u][c] = GIN ? __uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(Gv)[(int64_t)dst * d + col] << 16)
                                       : reinterpret_cast<const float *>(Gv)[(int64_t)dst * d + col];
                }
            }
#pragma unroll
            for (int u = 0; u < UK; ++u)
#pragma unroll
                for (int t = 0; t < NBT; ++t)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        acc[t][c] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[u][t], gb[u][c], acc[t][c], 0, 0, 0);
        }
    }
    // D register v of lane l: base 8*(v/4) + 4*(l/32) + v%4, column l%32 of its tile
#pragma unroll
    for (int t = 0; t < NBT; ++t)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int tb = bbase + t * 32, tc = cbase + c * 32;
            if (tb >= B || tc >= d) continue;              // uniform
            if (rw.unit >= 0 || !BF16) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int b = tb + 8 * (v >> 2) + 4 * h + (v & 3), col = tc + l32;
                    if (b < B && col < d) {
                        if (rw.unit >= 0) partial[((int64_t)rw.unit * B + b) * d + col] = acc[t][c][v];
                        else reinterpret_cast<float *>(dP)[(int64_t)rw.row * ld + (int64_t)b * d + col] = acc[t][c][v];
                    }
                }
            } else {
                // through LDS so that each lane writes 16 consecutive bf16 of one base row
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int v = 0; v < 16; ++v) stage[wv][8 * (v >> 2) + 4 * h + (v & 3)][l32] = acc[t][c][v];
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
                const int br = lane >> 1, c16 = (lane & 1) * 16;
                const float4 x0 = *reinterpret_cast<const float4 *>(&stage[wv][br][c16]);
                const float4 x1 = *reinterpret_cast<const float4 *>(&stage[wv][br][c16 + 4]);
                const float4 x2 = *reinterpret_cast<const float4 *>(&stage[wv][br][c16 + 8]);
                const float4 x3 = *reinterpret_cast<const float4 *>(&stage[wv][br][c16 + 12]);
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                if (tb + br < B) {
                    uint16_t *q = reinterpret_cast<uint16_t *>(dP) + (int64_t)rw.row * ld + (int64_t)(tb + br) * d + tc + c16;
                    *reinterpret_cast<uint4 *>(q) = make_uint4(pack_bf16x2(x0.x, x0.y), pack_bf16x2(x0.z, x0.w),
                                                               pack_bf16x2(x1.x, x1.y), pack_bf16x2(x1.z, x1.w));
                    *reinterpret_cast<uint4 *>(q + 8) = make_uint4(pack_bf16x2(x2.x, x2.y), pack_bf16x2(x2.z, x2.w),
                                                                   pack_bf16x2(x3.x, x3.y), pack_bf16x2(x3.z, x3.w));
                }
            }
        }
}

// The same per-source product for workloads that keep messages in bf16, on v_mfma_f32_32x32x16_bf16:
//   dP[j] (B x d, bf16) = W^T (B x deg) * Gg (deg x d),  W[e][b] = a[rel_e][b] invc_e (rounded to bf16),  Gg[e] = Gbf[dst_e].
// One block of four wavefronts per (source or heavy unit, chunk of 64 bases, chunk of 256 columns).  The block
// stages up to 32 edges at a time in LDS, as they lie in memory and with 16-byte loads: the gathered rows of G
// ([edge][column]) and the coefficient rows ([edge][base], multiplied by 1/c and rounded on the way).  The edge is
// the contraction index of both, so the matrix-core operands are fetched with the transposing LDS read, two per
// operand; wavefront w owns bases 32 (w / 2) .. and columns 128 (w % 2) ..: one coefficient operand feeds four
// products.  Sixteen edges per matrix-core instruction instead of two, and the gathered rows are read once per
// block instead of once per wavefront.
constexpr int GTB_EP = 32;                 // edges per pass
constexpr int GTB_PG = 256 + 32;           // LDS pitches, elements: 64 bytes modulo 256 (the four rows that 16
constexpr int GTB_PC = 64 + 96;            // lanes read at once fall in different quarters of the banks)

__global__ __launch_bounds__(256) void k_gather_t_bf16(
    const int32_t *__restrict__ sm_ptr, const int32_t *__restrict__ sm_dst,
    const int32_t *__restrict__ sm_rel, const float *__restrict__ sm_invc, int64_t N,
    int32_t n_units, const int32_t *__restrict__ hv_row, const int32_t *__restrict__ hv_unit_ptr,
    const int32_t *__restrict__ unit_hv,
    const uint16_t *__restrict__ Gbf, int64_t ldg, const float *__restrict__ a, int32_t B, int32_t d,
    int32_t n_bchunks, int32_t n_cchunks, uint16_t *__restrict__ dP, int64_t ld, float *__restrict__ partial,
    const uint8_t *__restrict__ active)
{
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __bf16 gtb_bf16x8 __attribute__((ext_vector_type(8)));
    __shared__ __attribute__((aligned(16))) uint16_t Gs[GTB_EP * GTB_PG];     // 18,432 B; the epilogue's staging too
    __shared__ __attribute__((aligned(16))) uint16_t Cs[GTB_EP * GTB_PC];     // 10,240 B
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int n_chunks = n_bchunks * n_cchunks;
    const int64_t wid = (int64_t)blockIdx.x / n_chunks;
    const int chunk = (int)((int64_t)blockIdx.x - wid * n_chunks);
    const int bbase = (chunk / n_cchunks) * 64, cbase = (chunk % n_cchunks) * 256;
    const RowWork rw = row_work(wid, sm_ptr, N, n_units, hv_row, hv_unit_ptr, unit_hv);
    if (rw.row < 0) return;                               // uniform over the block
    const int wm = w >> 1, wn = w & 1;

    gt_floatx16 acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;

    // this thread's part of a pass: edge t / 8; of its G row the 16-byte chunks (t % 8) + 8 p, of its coefficient
    // row the 8 bases from 8 (t % 8)
    const int el = t >> 3, sub = t & 7;
    const int l16 = lane & 15, kr0 = 8 * (lane >> 5) + (l16 >> 2), mc = 16 * ((lane >> 4) & 1) + 4 * (l16 & 3);
    auto frag = [&](const uint16_t *tile, int pitch, int kr, int col) __attribute__((always_inline)) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4 __attribute__((address_space(3))) *)(tile + kr * pitch + col));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4 __attribute__((address_space(3))) *)(tile + (kr + 4) * pitch + col));
        return __builtin_bit_cast(gtb_bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    for (int32_t e0 = rw.beg; e0 < rw.end; e0 += GTB_EP) {
        const int cnt = min(GTB_EP, rw.end - e0);
        int32_t dst = -1, rel = 0;
        float wgt = 0.f;
        if (el < cnt) {
            dst = sm_dst[e0 + el]; rel = sm_rel[e0 + el]; wgt = sm_invc ? sm_invc[e0 + el] : 1.f;
            if (active && !active[dst]) dst = -1;         // destination outside the sub-graph: its G row is zero
        }
        uint4 gq[4];
        float cf[8];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int col = cbase + 8 * (sub + 8 * p);
            gq[p] = make_uint4(0u, 0u, 0u, 0u);
            if (dst >= 0 && col < d) gq[p] = *reinterpret_cast<const uint4 *>(Gbf + (int64_t)dst * ldg + col);
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int b = bbase + 8 * sub + q;
            cf[q] = (dst >= 0 && b < B) ? a[(int64_t)rel * B + b] * wgt : 0.f;
        }
        __syncthreads();                                  // the previous pass's operands are consumed
#pragma unroll
        for (int p = 0; p < 4; ++p)
            *reinterpret_cast<uint4 *>(&Gs[el * GTB_PG + 8 * (sub + 8 * p)]) = gq[p];
        *reinterpret_cast<uint4 *>(&Cs[el * GTB_PC + 8 * sub]) =
            make_uint4(pack_bf16x2(cf[0], cf[1]), pack_bf16x2(cf[2], cf[3]), pack_bf16x2(cf[4], cf[5]), pack_bf16x2(cf[6], cf[7]));
        __syncthreads();
        if (bbase + 32 * wm < B) {                        // uniform per wavefront
#pragma unroll
            for (int ks = 0; ks < GTB_EP; ks += 16) {
                if (ks >= cnt) break;                     // uniform
                const gtb_bf16x8 af = frag(Cs, GTB_PC, ks + kr0, 32 * wm + mc);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (cbase + 128 * wn + 32 * c >= d) continue;     // uniform
                    const gtb_bf16x8 bfr = frag(Gs, GTB_PG, ks + kr0, 128 * wn + 32 * c + mc);
                    acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr, acc[c], 0, 0, 0);
                }
            }
        }
    }
    __syncthreads();                                      // Gs is free: each wavefront stages its tiles in its quarter
    // D register v of lane l: base 8*(v/4) + 4*(l/32) + v%4, column l%32 of its tile
    const int h = lane >> 5, l32 = lane & 31;
    float (*stage)[36] = reinterpret_cast<float (*)[36]>(reinterpret_cast<float *>(Gs) + w * 32 * 36);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int tb = bbase + 32 * wm, tc = cbase + 128 * wn + 32 * c;
        if (tb >= B || tc >= d) continue;                 // uniform
        if (rw.unit >= 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int b = tb + 8 * (v >> 2) + 4 * h + (v & 3);
                if (b < B) partial[((int64_t)rw.unit * B + b) * d + tc + l32] = acc[c][v];
            }
        } else {
            // through LDS so that each lane writes 16 consecutive bf16 of one base row
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int v = 0; v < 16; ++v) stage[8 * (v >> 2) + 4 * h + (v & 3)][l32] = acc[c][v];
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const int br = lane >> 1, c16 = (lane & 1) * 16;
            const float4 x0 = *reinterpret_cast<const float4 *>(&stage[br][c16]);
            const float4 x1 = *reinterpret_cast<const float4 *>(&stage[br][c16 + 4]);
            const float4 x2 = *reinterpret_cast<const float4 *>(&stage[br][c16 + 8]);
            const float4 x3 = *reinterpret_cast<const float4 *>(&stage[br][c16 + 12]);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            if (tb + br < B) {
                uint16_t *q = dP + (int64_t)rw.row * ld + (int64_t)(tb + br) * d + tc + c16;
                *reinterpret_cast<uint4 *>(q) = make_uint4(pack_bf16x2(x0.x, x0.y), pack_bf16x2(x0.z, x0.w),
                                                           pack_bf16x2(x1.x, x1.y), pack_bf16x2(x1.z, x1.w));
                *reinterpret_cast<uint4 *>(q + 8) = make_uint4(pack_bf16x2(x2.x, x2.y), pack_bf16x2(x2.z, x2.w),
                                                               pack_bf16x2(x3.x, x3.y), pack_bf16x2(x3.z, x3.w));
            }
        }
    }
}

// Heavy sources: dP[j] = sum of the row's unit partials.  One thread per float4 of a [B*d] row.
template <bool BF16>
__global__ void k_gather_t_finish(int32_t n_hv, const int32_t *__restrict__ hv_row,
                                  const int32_t *__restrict__ hv_unit_ptr, const float *__restrict__ partial,
                                  int32_t bd, void *__restrict__ dP, int64_t ld,
                                  const uint8_t *__restrict__ row_active)
{
    const int bd4 = bd >> 2;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)n_hv * bd4) return;
    const int32_t h = (int32_t)(idx / bd4);
    if (row_active && !row_active[hv_row[h]]) return;
    const int k4 = (int)(idx - (int64_t)h * bd4) * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int32_t u = hv_unit_ptr[h]; u < hv_unit_ptr[h + 1]; ++u) {
        const float4 x = *reinterpret_cast<const float4 *>(partial + (int64_t)u * bd + k4);
        s.x += x.x; s.y += x.y; s.z += x.z; s.w += x.w;
    }
    const int64_t o = (int64_t)hv_row[h] * ld + k4;
    if (BF16) {
        uint2 x;
        x.x = pack_bf16x2(s.x, s.y); x.y = pack_bf16x2(s.z, s.w);
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(dP) + o) = x;
    } else {
        *reinterpret_cast<float4 *>(reinterpret_cast<float *>(dP) + o) = s;
    }
}

// ------------------------------------------------------------------ run means
// One wavefront per (relation, destination) run s (or per unit of a long run):
//   Z[s][:] = invc_s * sum_{j in run s} H[j][:]
// the normalised neighbour sum of Eq. 1 for one relation, before any weight is applied.
// BF16: the input rows and Z are bf16 (sums stay fp32).
template <bool BF16, int LPR>
__global__ __launch_bounds__(64 * WPB) void k_run_mean(
    const int32_t *__restrict__ seg_ptr, const int32_t *__restrict__ seg_dst,
    const float *__restrict__ inv_c, const int32_t *__restrict__ col_src, int64_t S,
    int32_t n_units, const int32_t *__restrict__ hv_row, const int32_t *__restrict__ hv_unit_ptr,
    const int32_t *__restrict__ unit_hv, const void *__restrict__ H, int32_t d,
    void *__restrict__ Z, float *__restrict__ partial, const uint8_t *__restrict__ active, int skip_single)
{
    constexpr int VEC = MsgRow<BF16>::VEC;
    constexpr int NG = 64 / LPR;
    constexpr int U = (NG >= 8) ? 2 : (NG >= 2 ? 4 : 8);     // row loads in flight per lane
    const int lane = threadIdx.x & 63;
    const int64_t wid = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
    const RowWork rw = row_work(wid, seg_ptr, S, n_units, hv_row, hv_unit_ptr, unit_hv);
    if (rw.row < 0) return;
    if (skip_single && rw.unit < 0 && rw.end - rw.beg == 1) return;    // read in place by the consumer
    const int kl = lane % LPR, g = lane / LPR;
    const bool kact = kl * VEC < d;
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
    const bool skip = active && !active[seg_dst[rw.row]];     // destination outside the sub-graph: zeros
    if (skip && rw.unit >= 0) return;
    const int len = skip ? 0 : rw.end - rw.beg;
    for (int e0 = 0; e0 < len; e0 += NG * U) {
        uint4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int el = e0 + u * NG + g;
            x[u] = make_uint4(0u, 0u, 0u, 0u);
            if (el < len && kact) {
                const int32_t src = col_src[rw.beg + el];
                x[u] = MsgRow<BF16>::load_raw(H, (int64_t)src * d + kl * VEC);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float val[VEC];
            MsgRow<BF16>::unpack(x[u], val);
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] += val[v];
        }
    }
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] += __shfl_xor(acc[v], off, 64);
    if (g != 0 || !kact) return;
    if (rw.unit >= 0) {
#pragma unroll
        for (int v4 = 0; v4 < VEC; v4 += 4)
            *reinterpret_cast<float4 *>(partial + (int64_t)rw.unit * d + kl * VEC + v4) =
                make_float4(acc[v4], acc[v4 + 1], acc[v4 + 2], acc[v4 + 3]);
        return;
    }
    const float w = skip ? 0.f : inv_c[rw.row];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] *= w;
    if (BF16) {
        *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(Z) + rw.row * d + kl * VEC) =
            make_uint4(pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]),
                       pack_bf16x2(acc[4 % VEC], acc[5 % VEC]), pack_bf16x2(acc[6 % VEC], acc[7 % VEC]));
    } else {
        typedef float rm_f32x4 __attribute__((ext_vector_type(4)));
        __builtin_nontemporal_store(rm_f32x4{acc[0], acc[1], acc[2], acc[3]},
                                    reinterpret_cast<rm_f32x4 *>(reinterpret_cast<float *>(Z) + rw.row * d + kl * VEC));
    }
}

// The same run means when most runs are very short (many relations: a run is often a single edge).
// One wavefront takes RPW consecutive runs; each lane group owns every NG-th of them and has the
// first source row of all its runs in flight at once, which is the whole sum for most.  Runs of
// KGE_HEAVY edges or more are left to the unit wavefronts of k_run_mean and k_run_mean_finish.
template <bool BF16, int LPR, int RPW>
__global__ __launch_bounds__(64 * WPB) void k_run_mean_multi(
    const int32_t *__restrict__ seg_ptr, const int32_t *__restrict__ seg_dst,
    const float *__restrict__ inv_c, const int32_t *__restrict__ col_src, int64_t S,
    const void *__restrict__ H, int32_t d, void *__restrict__ Z, const uint8_t *__restrict__ active, int skip_single,
    const int32_t *__restrict__ run_list)
{
    // run_list (optional): the wavefronts walk runs run_list[0 .. S) instead of runs 0 .. S
    constexpr int VEC = MsgRow<BF16>::VEC;
    constexpr int NG = 64 / LPR;
    constexpr int PER = RPW / NG;                          // runs per lane group
    static_assert(RPW % NG == 0 && RPW < 64, "runs per wavefront must be a multiple of the lane groups");
    const int lane = threadIdx.x & 63;
    const int64_t s0 = ((int64_t)blockIdx.x * WPB + (threadIdx.x >> 6)) * RPW;
    if (s0 >= S) return;
    const int kl = lane % LPR, g = lane / LPR;
    const bool kact = kl * VEC < d;
    // bounds of the RPW runs: lanes 0 .. RPW hold seg_ptr[s0 + lane]; with a list, lane r holds its run's
    // id and both of its bounds
    int32_t pv = 0, pe = 0, pid = 0;
    if (run_list) {
        if (lane < RPW && s0 + lane < S) { pid = run_list[s0 + lane]; pv = seg_ptr[pid]; pe = seg_ptr[pid + 1]; }
    } else if (lane <= RPW) {
        pv = seg_ptr[min(s0 + lane, S)];
    }
    int32_t beg[PER], len[PER], src0[PER], rid[PER];
    float w[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int r = i * NG + g;
        const int32_t b = __shfl(pv, r, 64), e1 = __shfl(pv, r + 1, 64), e2 = __shfl(pe, r, 64), id = __shfl(pid, r, 64);
        const int32_t e = run_list ? e2 : e1;
        const bool exists = s0 + r < S;
        const int64_t sr = run_list ? (int64_t)id : s0 + r;
        rid[i] = (int32_t)sr;
        beg[i] = b;
        len[i] = exists ? e - b : -1;                      // -1: no such run
        w[i] = 0.f;
        src0[i] = 0;
        if (len[i] >= KGE_HEAVY) len[i] = -1;              // written by the finishing kernel
        if (skip_single && len[i] == 1) len[i] = -1;       // read in place by the consumer
        if (len[i] > 0) {
            if (active && !active[seg_dst[sr]]) len[i] = 0;            // outside the sub-graph: a zero row
            else { w[i] = inv_c[sr]; src0[i] = col_src[b]; }
        }
    }
    uint4 x0[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        x0[i] = make_uint4(0u, 0u, 0u, 0u);
        if (len[i] > 0 && kact) x0[i] = MsgRow<BF16>::load_raw(H, (int64_t)src0[i] * d + kl * VEC);
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        if (len[i] < 0) continue;
        float acc[VEC];
        MsgRow<BF16>::unpack(x0[i], acc);
        for (int el = 1; el < len[i]; el += 2) {           // the rest of a longer run, two rows at a time
            const bool two = el + 1 < len[i];
            uint4 xa = make_uint4(0u, 0u, 0u, 0u), xb = make_uint4(0u, 0u, 0u, 0u);
            const int32_t sa = col_src[beg[i] + el], sb = two ? col_src[beg[i] + el + 1] : 0;
            if (kact) {
                xa = MsgRow<BF16>::load_raw(H, (int64_t)sa * d + kl * VEC);
                if (two) xb = MsgRow<BF16>::load_raw(H, (int64_t)sb * d + kl * VEC);
            }
            float va[VEC], vb[VEC];
            MsgRow<BF16>::unpack(xa, va);
            MsgRow<BF16>::unpack(xb, vb);
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] += va[v] + vb[v];
        }
        if (!kact) continue;
        const int64_t o = (int64_t)rid[i] * d + kl * VEC;
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] *= w[i];
        if (BF16) {
            typedef uint32_t rm_u32x4 __attribute__((ext_vector_type(4)));
            __builtin_nontemporal_store(rm_u32x4{pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]),
                                                 pack_bf16x2(acc[4 % VEC], acc[5 % VEC]), pack_bf16x2(acc[6 % VEC], acc[7 % VEC])},
                                        reinterpret_cast<rm_u32x4 *>(reinterpret_cast<uint16_t *>(Z) + o));
        } else {
            *reinterpret_cast<float4 *>(reinterpret_cast<float *>(Z) + o) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        }
    }
}

// Long runs: Z[s] = invc_s * sum of the run's unit partials.  One thread per float4.
template <bool BF16>
__global__ void k_run_mean_finish(int32_t n_hv, const int32_t *__restrict__ hv_row,
                                  const int32_t *__restrict__ hv_unit_ptr, const float *__restrict__ partial,
                                  const float *__restrict__ inv_c, int32_t d, void *__restrict__ Z,
                                  const int32_t *__restrict__ seg_dst, const uint8_t *__restrict__ active)
{
    const int d4 = d >> 2;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)n_hv * d4) return;
    const int32_t h = (int32_t)(idx / d4);
    const int k4 = (int)(idx - (int64_t)h * d4) * 4;
    const int64_t row = hv_row[h];
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (!(active && !active[seg_dst[row]])) {
        for (int32_t u = hv_unit_ptr[h]; u < hv_unit_ptr[h + 1]; ++u) {
            const float4 x = *reinterpret_cast<const float4 *>(partial + (int64_t)u * d + k4);
            s.x += x.x; s.y += x.y; s.z += x.z; s.w += x.w;
        }
        const float w = inv_c[row];
        s.x *= w; s.y *= w; s.z *= w; s.w *= w;
    }
    if (BF16)
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(Z) + row * d + k4) =
            make_uint2(pack_bf16x2(s.x, s.y), pack_bf16x2(s.z, s.w));
    else
        *reinterpret_cast<float4 *>(reinterpret_cast<float *>(Z) + row * d + k4) = s;
}

// ------------------------------------------------------------------ coefficient gradient
// One wavefront per (relation, destination) run s = (r, i) (or per unit of a long run):
//   seg_out[s][b] = invc_s * sum_{j in run} < P[j][b][:], G[i][:] >
// and da[r][b] is the sum of seg_out over the runs of relation r (k_coeff_reduce).
// UB basis slots x UE edge rounds are in flight at a time.
template <bool BF16, int LPR, int UB, int UE>
__global__ __launch_bounds__(64 * WPB) void k_coeff_seg(
    const int32_t *__restrict__ seg_ptr, const int32_t *__restrict__ seg_dst,
    const float *__restrict__ inv_c, const int32_t *__restrict__ col_src, int64_t S,
    int32_t n_units, const int32_t *__restrict__ hv_row, const int32_t *__restrict__ hv_unit_ptr,
    const int32_t *__restrict__ unit_hv,
    const void *__restrict__ P, const float *__restrict__ G, int32_t B, int32_t d, int32_t gb_count,
    float *__restrict__ seg_out, float *__restrict__ partial, const uint8_t *__restrict__ active)
{
    constexpr int VEC = MsgRow<BF16>::VEC;
    constexpr int NG = 64 / LPR;
    const int lane = threadIdx.x & 63;
    const int64_t wid = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
    const RowWork rw = row_work(wid, seg_ptr, S, n_units, hv_row, hv_unit_ptr, unit_hv);
    if (rw.row < 0) return;
    if (active && !active[seg_dst[rw.row]]) {           // destination outside the sub-graph: G row is zero
        if (rw.unit < 0)
            for (int b = lane; b < B; b += 64) seg_out[rw.row * B + b] = 0.f;
        return;
    }
    const int kl = lane % LPR, g = lane / LPR;
    const int GB = gb_count, GE = NG / GB;
    const int gb = g % GB, ge = g / GB;
    const bool kact = kl * VEC < d;
    const int nb = (B + GB - 1) / GB;

    const int32_t i = seg_dst[rw.row];
    const float scale = rw.unit >= 0 ? 1.f : inv_c[rw.row];
    float gv[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) gv[v] = 0.f;
    if (kact) {
#pragma unroll
        for (int v4 = 0; v4 < VEC; v4 += 4) {
            float4 x = *reinterpret_cast<const float4 *>(G + (int64_t)i * d + kl * VEC + v4);
            gv[v4] = x.x; gv[v4 + 1] = x.y; gv[v4 + 2] = x.z; gv[v4 + 3] = x.w;
        }
    }
    const int len = rw.end - rw.beg;
    const int erounds = (len + GE - 1) / GE;
    float *dst_out = rw.unit >= 0 ? partial + (int64_t)rw.unit * B : seg_out + rw.row * B;
    for (int bi0 = 0; bi0 < nb; bi0 += UB) {
        float part[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) part[u] = 0.f;
        for (int er0 = 0; er0 < erounds; er0 += UE) {
            uint4 raw[UE][UB];
#pragma unroll
            for (int x = 0; x < UE; ++x) {
                const int el = (er0 + x) * GE + ge;
                const bool eok = el < len;
                const int32_t src = eok ? col_src[rw.beg + el] : 0;
#pragma unroll
                for (int u = 0; u < UB; ++u) {
                    const int b = (bi0 + u) * GB + gb;
                    raw[x][u] = make_uint4(0u, 0u, 0u, 0u);
                    if (eok && kact && (bi0 + u) < nb && b < B)
                        raw[x][u] = MsgRow<BF16>::load_raw(P, ((int64_t)src * B + b) * d + kl * VEC);
                }
            }
#pragma unroll
            for (int x = 0; x < UE; ++x)
#pragma unroll
                for (int u = 0; u < UB; ++u) {
                    float val[VEC];
                    MsgRow<BF16>::unpack(raw[x][u], val);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) part[u] = fmaf(val[v], gv[v], part[u]);
                }
        }
        // sum over the LPR lanes of a row and over the GE edge groups; skip the offsets that
        // would mix different bases (LPR .. LPR*GB/2)
#pragma unroll
        for (int u = 0; u < UB; ++u) {
#pragma unroll
            for (int off = 1; off < LPR; off <<= 1) part[u] += __shfl_xor(part[u], off, 64);
            for (int off = LPR * GB; off < 64; off <<= 1) part[u] += __shfl_xor(part[u], off, 64);
        }
        if (kl == 0 && ge == 0) {
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int b = (bi0 + u) * GB + gb;
                if ((bi0 + u) < nb && b < B) dst_out[b] = scale * part[u];
            }
        }
    }
}

// Long runs: seg_out[s][b] = invc_s * sum of the run's unit partials.
__global__ void k_coeff_finish(int32_t n_hv, const int32_t *__restrict__ hv_row,
                               const int32_t *__restrict__ hv_unit_ptr, const float *__restrict__ partial,
                               const float *__restrict__ inv_c, int32_t B, float *__restrict__ seg_out,
                               const int32_t *__restrict__ seg_dst, const uint8_t *__restrict__ active)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)n_hv * B) return;
    const int32_t h = (int32_t)(idx / B);
    const int b = (int)(idx - (int64_t)h * B);
    const int64_t row = hv_row[h];
    if (active && !active[seg_dst[row]]) { seg_out[row * B + b] = 0.f; return; }
    float s = 0.f;
    for (int32_t u = hv_unit_ptr[h]; u < hv_unit_ptr[h + 1]; ++u) s += partial[(int64_t)u * B + b];
    seg_out[row * B + b] = inv_c[row] * s;
}

// da[r][b] += sum of seg_out[s][b] over one chunk of relation r's runs (the partition's chunk list: every chunk lies
// in one relation).  A run's B values are covered by TPR threads of V floats each (V = 4 when B is a multiple
// of 4); the block's 256 / TPR run slots walk the chunk with four rows in flight per thread.
template <int V>
__global__ __launch_bounds__(256) void k_coeff_reduce(const int32_t *__restrict__ c_rel, const int32_t *__restrict__ c_beg,
                                                      const int32_t *__restrict__ c_end,
                                                      const float *__restrict__ seg_out, int32_t B, int32_t TPR,
                                                      float *__restrict__ da)
{
    __shared__ float red[256 * V];
    const int r = c_rel[blockIdx.x];
    const int64_t beg = c_beg[blockIdx.x], end = c_end[blockIdx.x];
    const int slots = 256 / TPR;
    const int b = (threadIdx.x % TPR) * V, slot = threadIdx.x / TPR;
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.f;
    if (b < B) {
        int64_t s = beg + slot;
        for (; s + 3 * slots < end; s += 4 * slots) {
            float x[4][V];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float *q = seg_out + (s + (int64_t)u * slots) * B + b;
                if (V == 4) { const float4 t4 = *reinterpret_cast<const float4 *>(q); x[u][0] = t4.x; x[u][1 % V] = t4.y; x[u][2 % V] = t4.z; x[u][3 % V] = t4.w; }
                else x[u][0] = q[0];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < V; ++v) acc[v] += x[u][v];
        }
        for (; s < end; s += slots)
#pragma unroll
            for (int v = 0; v < V; ++v) acc[v] += seg_out[s * B + b + v];
    }
#pragma unroll
    for (int v = 0; v < V; ++v) red[threadIdx.x * V + v] = acc[v];
    __syncthreads();
    if (slot == 0 && b < B) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
            float t = 0.f;
            for (int k = 0; k < slots; ++k) t += red[(k * TPR + threadIdx.x) * V + v];
            if (t != 0.f) unsafeAtomicAdd(&da[(int64_t)r * B + b + v], t);
        }
    }
}

int pow2_at_least(int x) { int p = 1; while (p < x) p <<= 1; return p; }
int largest_pow2_dividing(int x, int cap) { int p = 1; while (p * 2 <= cap && x % (p * 2) == 0) p <<= 1; return p; }

}  // namespace

// ------------------------------------------------------------------ launchers
#define DISPATCH_LPR(LPRV, CALL)                                                        \
    switch (LPRV) {                                                                     \
    case 1: { constexpr int L = 1; CALL; } break;                                       \
    case 2: { constexpr int L = 2; CALL; } break;                                       \
    case 4: { constexpr int L = 4; CALL; } break;                                       \
    case 8: { constexpr int L = 8; CALL; } break;                                       \
    case 16: { constexpr int L = 16; CALL; } break;                                     \
    case 32: { constexpr int L = 32; CALL; } break;                                     \
    default: { constexpr int L = 64; CALL; } break;                                     \
    }

int launch_gather_forward(const kge_partition *p, const void *P, int msg_bf16, const float *a,
                          int32_t B, int32_t d, const float *Self, int act, float *out, float *out2,
                          float *partial, const uint8_t *active, hipStream_t st)
{
    const int64_t N = p->n_vert;
    if (N == 0) return KGE_OK;
    const int vec = msg_bf16 ? 8 : 4;
    const int lpr = pow2_at_least((d + vec - 1) / vec);
    KGE_REQUIRE(lpr <= 64, KGE_EINVAL, "feature width %d too large for the aggregation kernel", d);
    const int gbc = largest_pow2_dividing(B, 64 / lpr);
    const kge_heavy_index &hx = p->hv_dm;
    const unsigned grid = (unsigned)cdiv(N + hx.n_units, WPB);
    {
        KGE_PROF("gather_fwd", st);
#define GF_ARGS p->dm_ptr, p->dm_src, p->dm_rel, p->dm_invc, N, hx.n_units, hx.hv_row, hx.hv_unit_ptr, hx.unit_hv, \
                P, a, B, d, gbc, Self, act, out, out2, nullptr, partial, active
        if (msg_bf16) { DISPATCH_LPR(lpr, (k_gather_fwd<true, L, false><<<grid, 64 * WPB, 0, st>>>(GF_ARGS))); }
        else { DISPATCH_LPR(lpr, (k_gather_fwd<false, L, false><<<grid, 64 * WPB, 0, st>>>(GF_ARGS))); }
#undef GF_ARGS
    }
    KGE_LAUNCH_CHECK();
    if (hx.n_hv > 0) {
        KGE_PROF("gather_fwd_fin", st);
        const int64_t n = (int64_t)hx.n_hv * (d / 4);
        k_gather_fwd_finish<<<(unsigned)cdiv(n, 256), 256, 0, st>>>(hx.n_hv, hx.hv_row, hx.hv_unit_ptr, partial, d,
                                                                   Self, act, out, out2, nullptr, active);
        KGE_LAUNCH_CHECK();
    }
    return KGE_OK;
}

// out[i] = act( sum_{q in row i of the view} w_q X[idx_q][:] + Self[i] ),  X rows of d elements (fp32 or bf16)
static int launch_row_sum(const int32_t *ptr, const int32_t *idx, const float *w, int64_t n_rows,
                          const kge_heavy_index &hx, const char *name, const void *X, int x_bf16, int32_t d,
                          const float *Self, int act, float *out, float *out2, uint16_t *outbf, float *partial,
                          const uint8_t *active, hipStream_t st)
{
    if (n_rows == 0) return KGE_OK;
    const int vec = x_bf16 ? 8 : 4;
    const int lpr = pow2_at_least((d + vec - 1) / vec);
    KGE_REQUIRE(lpr <= 64, KGE_EINVAL, "feature width %d too large for the aggregation kernel", d);
    const unsigned grid = (unsigned)cdiv(n_rows + hx.n_units, WPB);
    {
        KGE_PROF(name, st);
#define RS_ARGS ptr, idx, nullptr, w, n_rows, hx.n_units, hx.hv_row, hx.hv_unit_ptr, hx.unit_hv, X, nullptr, 1, d, 1, \
                Self, act, out, out2, outbf, partial, active
        if (x_bf16) { DISPATCH_LPR(lpr, (k_gather_fwd<true, L, true><<<grid, 64 * WPB, 0, st>>>(RS_ARGS))); }
        else { DISPATCH_LPR(lpr, (k_gather_fwd<false, L, true><<<grid, 64 * WPB, 0, st>>>(RS_ARGS))); }
#undef RS_ARGS
    }
    KGE_LAUNCH_CHECK();
    if (hx.n_hv > 0) {
        KGE_PROF("gather_fwd_fin", st);
        const int64_t n = (int64_t)hx.n_hv * (d / 4);
        k_gather_fwd_finish<<<(unsigned)cdiv(n, 256), 256, 0, st>>>(hx.n_hv, hx.hv_row, hx.hv_unit_ptr, partial, d,
                                                                   Self, act, out, out2, outbf, active);
        KGE_LAUNCH_CHECK();
    }
    return KGE_OK;
}

// out[i] = act( sum over the runs (r, i) of destination i of U[run][:] + Self[i] )
int launch_sum_runs(const kge_partition *p, const void *U, int u_bf16, int32_t d, const float *Self, int act,
                    float *out, float *out2, void *out_bf16, float *partial, const uint8_t *active, hipStream_t st)
{
    return launch_row_sum(p->dr_ptr, p->dr_seg, nullptr, p->n_vert, p->hv_dr, "sum_runs", U, u_bf16, d, Self, act,
                          out, out2, reinterpret_cast<uint16_t *>(out_bf16), partial, active, st);
}

// dH[j] = sum over the edges e out of j of invc_e dZ[run(e)][:] + Self[j]
int launch_sum_edges_out(const kge_partition *p, const void *dZ, int z_bf16, int32_t d, const float *Self,
                         float *out, float *partial, const uint8_t *active, hipStream_t st)
{
    return launch_row_sum(p->sm_ptr, p->sm_seg, p->sm_invc, p->n_vert, p->hv_sm, "sum_edges_out", dZ, z_bf16, d, Self,
                          KGE_ACT_IDENTITY, out, nullptr, nullptr, partial, active, st);
}

int launch_act_backward(const float *dHout, const float *Hout, int act, int64_t n, float *G, hipStream_t st)
{
    if (n == 0) return KGE_OK;
    int64_t n4 = n / 4;
    int64_t blocks = cdiv(n4, 256);
    if (blocks > 65536) blocks = 65536;
    KGE_PROF("act_bwd", st);
    k_act_backward<<<(unsigned)blocks, 256, 0, st>>>(reinterpret_cast<const float4 *>(dHout),
                                                    reinterpret_cast<const float4 *>(Hout), act, n4,
                                                    reinterpret_cast<float4 *>(G));
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

// A CSR view whose rows each sum coefficient-weighted rows of another matrix:
//   out[row][b][:] = sum_{q in row} a[rel[q]][b] * w[q] * X[idx[q]][:]       (w = 1 if null)
struct TView {
    const int32_t *ptr, *idx, *rel;
    const float *w;
    int64_t n_rows;
    const kge_heavy_index *hx;
    const char *name;
};

template <bool BF16, bool GIN, int LPR>
static int launch_gather_t_nb(const TView &vw, const void *G, const float *a, int32_t B, int32_t d,
                              void *dP, int64_t ld, float *partial, const uint8_t *active,
                              const uint8_t *row_active, hipStream_t st)
{
    constexpr int NG = 64 / LPR;
    const int64_t N = vw.n_rows;
    const kge_heavy_index &hx = *vw.hx;
    KGE_PROF(vw.name, st);
    // NB bases per lane (a power of two, at most 16); lane groups first cover the bases of a row,
    // the remaining groups split the edges
#define GT_CALL(NBV, UEV)                                                                             \
    {                                                                                                 \
        int gbt = 1;                                                                                  \
        while (gbt * 2 <= NG && gbt * NBV < B) gbt *= 2;                                              \
        const int n_chunks = (B + gbt * NBV - 1) / (gbt * NBV);                                       \
        const int64_t waves = (N + hx.n_units) * n_chunks;                                            \
        KGE_REQUIRE(cdiv(waves, WPB) < 0x7fffffffLL, KGE_ERANGE, "grid too large");                   \
        k_gather_t<BF16, GIN, LPR, NBV, UEV><<<(unsigned)cdiv(waves, WPB), 64 * WPB, 0, st>>>(              \
            vw.ptr, vw.idx, vw.rel, vw.w, N, hx.n_units, hx.hv_row, hx.hv_unit_ptr,                   \
            hx.unit_hv, G, a, B, d, n_chunks, gbt, dP, ld, partial, active, row_active);              \
    }
    if (B >= 16) GT_CALL(16, 2)
    else if (B >= 8) GT_CALL(8, 4)
    else if (B >= 4) GT_CALL(4, 4)
    else if (B >= 2) GT_CALL(2, 8)
    else GT_CALL(1, 8)
#undef GT_CALL
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

static int launch_tview(const TView &vw, const void *G, int g_bf16, const float *a, int32_t B, int32_t d,
                        void *dP, int64_t ld, int msg_bf16, float *partial, const uint8_t *active,
                        const uint8_t *row_active, hipStream_t st)
{
    KGE_REQUIRE(!g_bf16 || msg_bf16, KGE_EINVAL, "bf16 input rows are only used with bf16 output");
    if (vw.n_rows == 0) return KGE_OK;
    const int lpr = pow2_at_least((d + 3) / 4);
    KGE_REQUIRE(lpr <= 64, KGE_EINVAL, "feature width %d too large for the transposed aggregation kernel", d);
    int rc = KGE_OK;
    if (B >= 32 && d % 32 == 0) {
        // many bases: the per-source product runs on the matrix cores
        const kge_heavy_index &hxm = *vw.hx;
        const int n_bchunks = (B + 31) / 32, n_cchunks = (d + 127) / 128;
        const int64_t waves = (vw.n_rows + hxm.n_units) * n_bchunks * n_cchunks;
        KGE_REQUIRE(cdiv(waves, WPB) < 0x7fffffffLL, KGE_ERANGE, "grid too large");
        KGE_PROF(vw.name, st);
#define GTM_ARGS vw.ptr, vw.idx, vw.rel, vw.w, vw.n_rows, hxm.n_units, hxm.hv_row, hxm.hv_unit_ptr, \
                 hxm.unit_hv, G, a, B, d, n_bchunks, n_cchunks, dP, ld, partial, active, row_active
        if (g_bf16) k_gather_t_mfma<true, true, 1><<<(unsigned)cdiv(waves, WPB), 64 * WPB, 0, st>>>(GTM_ARGS);
        else if (msg_bf16) k_gather_t_mfma<true, false, 1><<<(unsigned)cdiv(waves, WPB), 64 * WPB, 0, st>>>(GTM_ARGS);
        else k_gather_t_mfma<false, false, 1><<<(unsigned)cdiv(waves, WPB), 64 * WPB, 0, st>>>(GTM_ARGS);
#undef GTM_ARGS
        KGE_LAUNCH_CHECK();
    } else if (g_bf16) { DISPATCH_LPR(lpr, (rc = launch_gather_t_nb<true, true, L>(vw, G, a, B, d, dP, ld, partial, active, row_active, st))); }
    else if (msg_bf16) { DISPATCH_LPR(lpr, (rc = launch_gather_t_nb<true, false, L>(vw, G, a, B, d, dP, ld, partial, active, row_active, st))); }
    else { DISPATCH_LPR(lpr, (rc = launch_gather_t_nb<false, false, L>(vw, G, a, B, d, dP, ld, partial, active, row_active, st))); }
    if (rc != KGE_OK) return rc;
    const kge_heavy_index &hx = *vw.hx;
    if (hx.n_hv > 0) {
        KGE_PROF("gather_t_fin", st);
        const int bd = B * d;
        const int64_t n = (int64_t)hx.n_hv * (bd / 4);
        if (msg_bf16) k_gather_t_finish<true><<<(unsigned)cdiv(n, 256), 256, 0, st>>>(hx.n_hv, hx.hv_row, hx.hv_unit_ptr, partial, bd, dP, ld, row_active);
        else k_gather_t_finish<false><<<(unsigned)cdiv(n, 256), 256, 0, st>>>(hx.n_hv, hx.hv_row, hx.hv_unit_ptr, partial, bd, dP, ld, row_active);
        KGE_LAUNCH_CHECK();
    }
    return KGE_OK;
}

int launch_gather_transpose(const kge_partition *p, const float *G, const float *a, int32_t B, int32_t d,
                            void *dP, int64_t ld, int msg_bf16, float *partial, const uint8_t *active,
                            hipStream_t st)
{
    const TView vw{p->sm_ptr, p->sm_dst, p->sm_rel, p->sm_invc, p->n_vert, &p->hv_sm, "gather_t"};
    return launch_tview(vw, G, 0, a, B, d, dP, ld, msg_bf16, partial, active, nullptr, st);
}

// The bf16 form: Gbf = the bf16 copy of G, rows `ldg` elements apart.  Takes the matrix-core kernel above when the
// layer has at least 32 bases and a width that is a multiple of 32; other shapes convert nothing and go the
// general way from the fp32 G.
bool gather_transpose_bf16_supported(int32_t B, int32_t d) { return B >= 32 && d % 32 == 0 && d >= 32; }

int launch_gather_transpose_bf16(const kge_partition *p, const void *Gbf, int64_t ldg, const float *a, int32_t B,
                                 int32_t d, void *dP, int64_t ld, float *partial, const uint8_t *active, hipStream_t st)
{
    KGE_REQUIRE(gather_transpose_bf16_supported(B, d), KGE_EINVAL, "transposed aggregation: shape not supported by the bf16 kernel");
    KGE_REQUIRE(ldg % 8 == 0 && ((uintptr_t)Gbf % 16) == 0 && ld % 8 == 0 && ((uintptr_t)dP % 16) == 0, KGE_EINVAL,
                "transposed aggregation: rows must be 16-byte aligned");
    const kge_heavy_index &hx = p->hv_sm;
    if (p->n_vert == 0) return KGE_OK;
    const int n_bchunks = (B + 63) / 64, n_cchunks = (d + 255) / 256;
    const int64_t blocks = ((int64_t)p->n_vert + hx.n_units) * n_bchunks * n_cchunks;
    KGE_REQUIRE(blocks < 0x7fffffffLL, KGE_ERANGE, "grid too large");
    {
        KGE_PROF("gather_t", st);
        k_gather_t_bf16<<<(unsigned)blocks, 256, 0, st>>>(p->sm_ptr, p->sm_dst, p->sm_rel, p->sm_invc, p->n_vert, hx.n_units,
                                                         hx.hv_row, hx.hv_unit_ptr, hx.unit_hv,
                                                         reinterpret_cast<const uint16_t *>(Gbf), ldg, a, B, d, n_bchunks,
                                                         n_cchunks, reinterpret_cast<uint16_t *>(dP), ld, partial, active);
        KGE_LAUNCH_CHECK();
    }
    if (hx.n_hv > 0) {
        KGE_PROF("gather_t_fin", st);
        const int bd = B * d;
        const int64_t n = (int64_t)hx.n_hv * (bd / 4);
        k_gather_t_finish<true><<<(unsigned)cdiv(n, 256), 256, 0, st>>>(hx.n_hv, hx.hv_row, hx.hv_unit_ptr, partial, bd, dP, ld, nullptr);
        KGE_LAUNCH_CHECK();
    }
    return KGE_OK;
}

template <bool BF16, int LPR>
static int launch_coeff_seg(const kge_partition *p, const void *P, const float *G, int32_t B, int32_t d,
                            int gbc, float *seg_scratch, float *partial, const uint8_t *active, hipStream_t st)
{
    const int64_t S = p->n_seg;
    const kge_heavy_index &hx = p->hv_seg;
    const unsigned grid = (unsigned)cdiv(S + hx.n_units, WPB);
    const int nb = (B + gbc - 1) / gbc;
#define CS_ARGS p->seg_ptr, p->seg_dst, p->inv_c, p->col_src, S, hx.n_units, hx.hv_row, hx.hv_unit_ptr, hx.unit_hv, \
                P, G, B, d, gbc, seg_scratch, partial, active
    // base slots x edges in flight per wavefront: with many bases, eight slots of one edge at a time (most runs
    // have one edge; 212 against 225 ms per launch at 25 M runs, 64 bases, d = 256; 4 x 1: 221, 8 x 2: 220, 16 x 1: 215)
    if (nb >= 8) k_coeff_seg<BF16, LPR, 8, 1><<<grid, 64 * WPB, 0, st>>>(CS_ARGS);
    else if (nb >= 4) k_coeff_seg<BF16, LPR, 4, 2><<<grid, 64 * WPB, 0, st>>>(CS_ARGS);
    else if (nb >= 2) k_coeff_seg<BF16, LPR, 2, 4><<<grid, 64 * WPB, 0, st>>>(CS_ARGS);
    else k_coeff_seg<BF16, LPR, 1, 8><<<grid, 64 * WPB, 0, st>>>(CS_ARGS);
#undef CS_ARGS
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

int launch_coeff_grad(const kge_partition *p, const void *P, int msg_bf16, const float *G, int32_t B,
                      int32_t d, float *seg_scratch, float *partial, float *da, const uint8_t *active,
                      hipStream_t st)
{
    const int64_t S = p->n_seg;
    const int32_t R2 = 2 * p->n_relations;
    int rc = launch_fill_zero(da, sizeof(float) * (size_t)R2 * B, st);
    if (rc != KGE_OK) return rc;
    if (S == 0) return KGE_OK;
    KGE_REQUIRE(B <= 256, KGE_EINVAL, "more than 256 bases are not supported");
    const int vec = msg_bf16 ? 8 : 4;
    const int lpr = pow2_at_least((d + vec - 1) / vec);
    KGE_REQUIRE(lpr <= 64, KGE_EINVAL, "feature width %d too large for the coefficient-gradient kernel", d);
    const int gbc = largest_pow2_dividing(B, 64 / lpr);
    {
        KGE_PROF("coeff_seg", st);
        if (msg_bf16) { DISPATCH_LPR(lpr, (rc = launch_coeff_seg<true, L>(p, P, G, B, d, gbc, seg_scratch, partial, active, st))); }
        else { DISPATCH_LPR(lpr, (rc = launch_coeff_seg<false, L>(p, P, G, B, d, gbc, seg_scratch, partial, active, st))); }
    }
    if (rc != KGE_OK) return rc;
    const kge_heavy_index &hx = p->hv_seg;
    if (hx.n_hv > 0) {
        KGE_PROF("coeff_fin", st);
        const int64_t n = (int64_t)hx.n_hv * B;
        k_coeff_finish<<<(unsigned)cdiv(n, 256), 256, 0, st>>>(hx.n_hv, hx.hv_row, hx.hv_unit_ptr, partial, p->inv_c, B, seg_scratch, p->seg_dst, active);
        KGE_LAUNCH_CHECK();
    }
    if (p->n_relc == 0) return KGE_OK;
    KGE_PROF("coeff_reduce", st);
    if (B % 4 == 0) k_coeff_reduce<4><<<(unsigned)p->n_relc, 256, 0, st>>>(p->relc_rel, p->relc_beg, p->relc_end, seg_scratch, B,
                                                                    pow2_at_least(B / 4), da);
    else k_coeff_reduce<1><<<(unsigned)p->n_relc, 256, 0, st>>>(p->relc_rel, p->relc_beg, p->relc_end, seg_scratch, B,
                                                                pow2_at_least(B), da);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

// Z[s][:] = invc_s * sum_{j in run s} H[j][:]; H and Z fp32, or both bf16; `partial`: [hv_seg.n_units][d] floats
int launch_run_mean(const kge_partition *p, const void *H, int32_t d, void *Z, int bf16, float *partial,
                    const uint8_t *active, int skip_single, hipStream_t st)
{
    const int64_t S = p->n_seg;
    if (S == 0) return KGE_OK;
    // single-edge runs skipped: only the listed runs of two or more edges are visited
    const int32_t *run_list = skip_single && p->mrun ? p->mrun : nullptr;
    const int64_t n_visit = run_list ? p->n_mrun : S;
    const int vec = bf16 ? 8 : 4;
    const int lpr = pow2_at_least((d + vec - 1) / vec);
    KGE_REQUIRE(lpr <= 64, KGE_EINVAL, "feature width %d too large for the run-mean kernel", d);
    const kge_heavy_index &hx = p->hv_seg;
    if (p->n_edge < 3 * S && lpr >= 8) {
        // mostly very short runs: several runs per wavefront; the unit wavefronts of the general kernel
        // still take the heavy runs (it is launched with no light rows)
        constexpr int RPW = 8;
        KGE_PROF("run_mean", st);
        const unsigned gridm = (unsigned)cdiv(cdiv(n_visit, RPW), WPB);
#define RMM_ARGS p->seg_ptr, p->seg_dst, p->inv_c, p->col_src, n_visit, H, d, Z, active, skip_single, run_list
        if (bf16) { DISPATCH_LPR(lpr, (k_run_mean_multi<true, (L < 8 ? 8 : L), RPW><<<gridm, 64 * WPB, 0, st>>>(RMM_ARGS))); }
        else { DISPATCH_LPR(lpr, (k_run_mean_multi<false, (L < 8 ? 8 : L), RPW><<<gridm, 64 * WPB, 0, st>>>(RMM_ARGS))); }
#undef RMM_ARGS
        KGE_LAUNCH_CHECK();
        if (hx.n_units > 0) {
            const unsigned gridu = (unsigned)cdiv(hx.n_units, WPB);
#define RMU_ARGS p->seg_ptr, p->seg_dst, p->inv_c, p->col_src, (int64_t)0, hx.n_units, hx.hv_row, hx.hv_unit_ptr, hx.unit_hv, \
                 H, d, Z, partial, active, 0
            if (bf16) { DISPATCH_LPR(lpr, (k_run_mean<true, L><<<gridu, 64 * WPB, 0, st>>>(RMU_ARGS))); }
            else { DISPATCH_LPR(lpr, (k_run_mean<false, L><<<gridu, 64 * WPB, 0, st>>>(RMU_ARGS))); }
#undef RMU_ARGS
            KGE_LAUNCH_CHECK();
        }
    } else {
    const unsigned grid = (unsigned)cdiv(S + hx.n_units, WPB);
    {
        KGE_PROF("run_mean", st);
#define RM_ARGS p->seg_ptr, p->seg_dst, p->inv_c, p->col_src, S, hx.n_units, hx.hv_row, hx.hv_unit_ptr, hx.unit_hv, \
                H, d, Z, partial, active, skip_single
        if (bf16) { DISPATCH_LPR(lpr, (k_run_mean<true, L><<<grid, 64 * WPB, 0, st>>>(RM_ARGS))); }
        else { DISPATCH_LPR(lpr, (k_run_mean<false, L><<<grid, 64 * WPB, 0, st>>>(RM_ARGS))); }
#undef RM_ARGS
    }
    KGE_LAUNCH_CHECK();
    }
    if (hx.n_hv > 0) {
        KGE_PROF("run_mean_fin", st);
        const int64_t n = (int64_t)hx.n_hv * (d / 4);
        if (bf16) k_run_mean_finish<true><<<(unsigned)cdiv(n, 256), 256, 0, st>>>(hx.n_hv, hx.hv_row, hx.hv_unit_ptr, partial,
                                                                                p->inv_c, d, Z, p->seg_dst, active);
        else k_run_mean_finish<false><<<(unsigned)cdiv(n, 256), 256, 0, st>>>(hx.n_hv, hx.hv_row, hx.hv_unit_ptr, partial,
                                                                             p->inv_c, d, Z, p->seg_dst, active);
        KGE_LAUNCH_CHECK();
    }
    return KGE_OK;
}
