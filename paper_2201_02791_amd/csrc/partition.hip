// build_partition on the GPU: core-edge selection by head hash (Sec. 3.2.1), n-hop
// Neighborhood Expansion by frontier marking (Sec. 3.2.2), local relabelling, and the
// (relation, destination, source, id)-sorted edge list with its runs, by a hand-written
// stable LSD radix sort.  Two more stable sorts give the destination-major and source-major
// views the aggregation kernels walk.  Runs once per partition; nothing here is in the
// timed training step.
#include <stdarg.h>
#include <string.h>

#include <vector>

#include "common.h"
#include <algorithm>
#include "sort_scan.h"

// slab of the destination range by which the transposed products' ranges are ordered (a test hook can shrink it)
static int64_t g_rel_slab = KGE_REL_SLAB, g_rel_min_runs = 0;

namespace {

__device__ __forceinline__ uint32_t part_of_head(int32_t head, uint32_t n_parts)
{
    return (((uint32_t)head * 0x9E3779B1u) >> 8) % n_parts;
}

// ---------------------------------------------------------------- marking
__global__ void k_check_ids(const int32_t *head, const int32_t *rel, const int32_t *tail, int64_t M,
                            int32_t n_ent, int32_t n_rel, uint32_t *bad)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    uint32_t h = (uint32_t)head[i], r = (uint32_t)rel[i], t = (uint32_t)tail[i];
    if (h >= (uint32_t)n_ent || t >= (uint32_t)n_ent || r >= (uint32_t)n_rel) *bad = 1u;
}

__global__ void k_mark_core(const int32_t *head, const int32_t *tail, int64_t M, uint32_t n_parts,
                            uint32_t part_id, uint32_t *core_flag, uint32_t *s0)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    uint32_t c = part_of_head(head[i], n_parts) == part_id ? 1u : 0u;
    core_flag[i] = c;
    if (c) { s0[head[i]] = 1u; s0[tail[i]] = 1u; }
}

// One expansion hop: a triple (s,r,t) carries s->t and t->s, so each endpoint in the
// previous set pulls in the other.  prev is read-only during the pass.
__global__ void k_expand(const int32_t *head, const int32_t *tail, int64_t M, const uint32_t *prev,
                         uint32_t *cur)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    int32_t s = head[i], t = tail[i];
    if (prev[t]) cur[s] = 1u;
    if (prev[s]) cur[t] = 1u;
}

// Build-time wrappers: the scratch of the scan and of the sort is allocated here (nothing in this file is
// in the timed training step).
int exclusive_scan(const uint32_t *in, uint32_t *out, int64_t n, hipStream_t st)
{
    uint32_t *scratch = nullptr;
    const size_t words = scan_scratch_words(n);
    if (words) KGE_HIP(hipMalloc(&scratch, sizeof(uint32_t) * words));
    int rc = exclusive_scan_ws(in, out, n, scratch, st);
    if (rc == KGE_OK && hipStreamSynchronize(st) != hipSuccess) { kge_set_error("scan failed"); rc = KGE_EHIP; }
    if (scratch) (void)hipFree(scratch);
    return rc;
}

template <typename K>
int radix_sort(K **keys, uint32_t **vals, K **keys_alt, uint32_t **vals_alt, int64_t n, int bits,
               hipStream_t st)
{
    if (n == 0) return KGE_OK;
    uint32_t *scratch = nullptr;
    KGE_HIP(hipMalloc(&scratch, sizeof(uint32_t) * radix_scratch_words(n)));
    int rc = radix_sort_ws<K>(keys, vals, keys_alt, vals_alt, n, bits, scratch, st);
    (void)hipStreamSynchronize(st);
    (void)hipFree(scratch);
    return rc;
}

// ---------------------------------------------------------------- compaction kernels
__global__ void k_vert_compact(const uint32_t *flag, const uint32_t *pos, int32_t n_ent,
                               int32_t *vert_gid, int32_t *lid)
{
    int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= n_ent) return;
    if (flag[g]) { vert_gid[pos[g]] = (int32_t)g; lid[g] = (int32_t)pos[g]; }
    else lid[g] = -1;
}

__global__ void k_cand_compact(const uint32_t *flag, const uint32_t *pos, int32_t n_ent,
                               const int32_t *lid, int32_t *cand)
{
    int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= n_ent) return;
    if (flag[g]) cand[pos[g]] = lid[g];
}

__global__ void k_core_compact(const uint32_t *flag, const uint32_t *pos, int64_t M,
                               const int32_t *head, const int32_t *rel, const int32_t *tail,
                               const int32_t *lid, int32_t *core_eid, int32_t *core_h,
                               int32_t *core_r, int32_t *core_t)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M || !flag[i]) return;
    uint32_t q = pos[i];
    core_eid[q] = (int32_t)i;
    core_h[q] = lid[head[i]];
    core_r[q] = rel[i];
    core_t[q] = lid[tail[i]];
}

// Message edge e in [0, 2M): e < M is triple e in the given direction (dst = tail),
// e >= M is the inverse of triple e-M (dst = head).  Kept iff dst is in S_{L-1}.
__global__ void k_edge_flag(const int32_t *head, const int32_t *tail, int64_t M,
                            const uint32_t *dstset, uint32_t *eflag)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= 2 * M) return;
    int32_t dst = e < M ? tail[e] : head[e - M];
    eflag[e] = dstset[dst] ? 1u : 0u;
}

__global__ void k_edge_emit(const int32_t *head, const int32_t *rel, const int32_t *tail, int64_t M,
                            int32_t n_rel, const uint32_t *eflag, const uint32_t *epos,
                            const int32_t *lid, int vbits, uint64_t *keys, uint32_t *vals)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= 2 * M || !eflag[e]) return;
    int64_t i = e < M ? e : e - M;
    uint64_t r = e < M ? (uint64_t)rel[i] : (uint64_t)(rel[i] + n_rel);
    uint64_t dst = (uint64_t)(e < M ? lid[tail[i]] : lid[head[i]]);
    uint64_t src = (uint64_t)(e < M ? lid[head[i]] : lid[tail[i]]);
    uint32_t q = epos[e];
    keys[q] = (r << (2 * vbits)) | (dst << vbits) | src;
    vals[q] = (uint32_t)e;
}

// ---------------------------------------------------------------- runs and views
__global__ void k_seg_flag(const uint64_t *keys, int64_t E, int vbits, uint32_t *flag)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    flag[e] = (e == 0 || (keys[e] >> vbits) != (keys[e - 1] >> vbits)) ? 1u : 0u;
}

__global__ void k_seg_emit(const uint64_t *keys, const uint32_t *vals, int64_t E, int vbits,
                           const uint32_t *flag, const uint32_t *fpos, int32_t *seg_ptr,
                           int32_t *seg_rel, int32_t *seg_dst, int32_t *col_src, int32_t *edge_id,
                           uint32_t *edge_seg)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    uint64_t k = keys[e], vmask = (1ull << vbits) - 1ull;
    col_src[e] = (int32_t)(k & vmask);
    edge_id[e] = (int32_t)vals[e];
    uint32_t s = fpos[e] + flag[e] - 1u;    // index of the run this edge belongs to
    edge_seg[e] = s;
    if (flag[e]) {
        seg_ptr[s] = (int32_t)e;
        seg_rel[s] = (int32_t)(k >> (2 * vbits));
        seg_dst[s] = (int32_t)((k >> vbits) & vmask);
    }
}

__global__ void k_seg_zrow(const int32_t *seg_ptr, const int32_t *col_src, int64_t S, int32_t N, int32_t *zrow)
{
    int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= S) return;
    const int32_t b = seg_ptr[s];
    zrow[s] = seg_ptr[s + 1] - b == 1 ? col_src[b] : N + (int32_t)s;
}

__global__ void k_multi_flag(const int32_t *seg_ptr, int64_t S, uint32_t *flag)
{
    int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s < S) flag[s] = seg_ptr[s + 1] - seg_ptr[s] >= 2 ? 1u : 0u;
}

__global__ void k_multi_emit(const uint32_t *flag, const uint32_t *pos, int64_t S, int32_t *mrun)
{
    int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s < S && flag[s]) mrun[pos[s]] = (int32_t)s;
}

__global__ void k_inv_c(const int32_t *seg_ptr, int64_t S, float *inv_c)
{
    int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= S) return;
    inv_c[s] = 1.0f / (float)(seg_ptr[s + 1] - seg_ptr[s]);
}

// keys2[e] = field of the sorted key selected by (shift, mask); vals2[e] = e
__global__ void k_view_keys(const uint64_t *keys, int64_t E, int shift, uint64_t mask, uint32_t *k2,
                            uint32_t *v2)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    k2[e] = (uint32_t)((keys[e] >> shift) & mask);
    v2[e] = (uint32_t)e;
}

// After sorting positions by one endpoint: other endpoint, relation and 1/c of every edge.
__global__ void k_view_emit(const uint32_t *pos_sorted, int64_t E, const uint64_t *keys, int vbits,
                            int other_shift, const uint32_t *edge_seg, const float *inv_c,
                            int32_t *o_vert, int32_t *o_rel, float *o_invc, int32_t *o_seg)
{
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= E) return;
    uint32_t e = pos_sorted[q];
    uint64_t k = keys[e], vmask = (1ull << vbits) - 1ull;
    o_vert[q] = (int32_t)((k >> other_shift) & vmask);
    o_rel[q] = (int32_t)(k >> (2 * vbits));
    o_invc[q] = inv_c[edge_seg[e]];
    if (o_seg) o_seg[q] = (int32_t)edge_seg[e];
}

// keys[s] = destination of run s, vals[s] = s
__global__ void k_run_keys(const int32_t *seg_dst, int64_t S, uint32_t *k, uint32_t *v)
{
    int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= S) return;
    k[s] = (uint32_t)seg_dst[s];
    v[s] = (uint32_t)s;
}

__global__ void k_run_emit(const uint32_t *sorted_run, int64_t S, const int32_t *seg_rel, int32_t *dr_seg,
                           int32_t *dr_rel)
{
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= S) return;
    const uint32_t s = sorted_run[q];
    dr_seg[q] = (int32_t)s;
    dr_rel[q] = seg_rel[s];
}

__global__ void k_max_degree(const int32_t *ptr, int64_t nv, int32_t *out)
{
    int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= nv) return;
    atomicMax(out, ptr[v + 1] - ptr[v]);
}

// Heavy-row index: rows with at least KGE_HEAVY edges, cut into units of KGE_HEAVY edges.
__global__ void k_heavy_flag(const int32_t *ptr, int64_t n_rows, uint32_t *flag, uint32_t *units)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows) return;
    int32_t deg = ptr[i + 1] - ptr[i];
    uint32_t f = deg >= KGE_HEAVY ? 1u : 0u;
    flag[i] = f;
    units[i] = f ? (uint32_t)((deg + KGE_HEAVY - 1) / KGE_HEAVY) : 0u;
}

__global__ void k_heavy_emit(int64_t n_rows, const uint32_t *flag, const uint32_t *hpos,
                             const uint32_t *units, const uint32_t *upos, int32_t *hv_row,
                             int32_t *hv_unit_ptr, int32_t *unit_hv)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows || !flag[i]) return;
    uint32_t h = hpos[i], u0 = upos[i], n = units[i];
    hv_row[h] = (int32_t)i;
    hv_unit_ptr[h] = (int32_t)u0;
    for (uint32_t k = 0; k < n; ++k) unit_hv[u0 + k] = (int32_t)h;
}

__global__ void k_iota(int32_t *a, int64_t n)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) a[i] = (int32_t)i;
}

int bits_for(uint64_t n_values)   // bits to hold ids 0..n_values-1 (at least 1)
{
    int b = 1;
    while ((1ull << b) < n_values) ++b;
    return b;
}

struct TempBufs {
    std::vector<void *> ptrs;
    ~TempBufs() { for (void *q : ptrs) (void)hipFree(q); }
    template <typename T> int alloc(T **out, size_t count)
    {
        void *q = nullptr;
        hipError_t e = hipMalloc(&q, sizeof(T) * (count ? count : 1));
        if (e != hipSuccess) { kge_set_error("hipMalloc of %zu bytes failed: %s", sizeof(T) * count, hipGetErrorString(e)); return KGE_ENOMEM; }
        ptrs.push_back(q);
        *out = (T *)q;
        return KGE_OK;
    }
};

template <typename T> int palloc(T **out, size_t count)
{
    void *q = nullptr;
    hipError_t e = hipMalloc(&q, sizeof(T) * (count ? count : 1));
    if (e != hipSuccess) { kge_set_error("hipMalloc of %zu bytes failed: %s", sizeof(T) * count, hipGetErrorString(e)); return KGE_ENOMEM; }
    *out = (T *)q;
    return KGE_OK;
}

#define TRY(x) do { int rc__ = (x); if (rc__ != KGE_OK) return rc__; } while (0)
inline unsigned grid_for(int64_t n) { return (unsigned)(n > 0 ? cdiv(n, TB) : 1); }

int build_heavy_index(const int32_t *ptr, int64_t n_rows, kge_heavy_index *hx, hipStream_t st)
{
    TempBufs tmp;
    uint32_t *flag, *units, *hpos, *upos;
    TRY(tmp.alloc(&flag, n_rows)); TRY(tmp.alloc(&units, n_rows));
    TRY(tmp.alloc(&hpos, (size_t)n_rows + 1)); TRY(tmp.alloc(&upos, (size_t)n_rows + 1));
    if (n_rows > 0) { k_heavy_flag<<<grid_for(n_rows), TB, 0, st>>>(ptr, n_rows, flag, units); KGE_LAUNCH_CHECK(); }
    TRY(exclusive_scan(flag, hpos, n_rows, st));
    TRY(exclusive_scan(units, upos, n_rows, st));
    uint32_t nh = 0, nu = 0;
    KGE_HIP(hipMemcpy(&nh, hpos + n_rows, sizeof(uint32_t), hipMemcpyDeviceToHost));
    KGE_HIP(hipMemcpy(&nu, upos + n_rows, sizeof(uint32_t), hipMemcpyDeviceToHost));
    hx->n_hv = (int32_t)nh; hx->n_units = (int32_t)nu;
    TRY(palloc(&hx->hv_row, nh)); TRY(palloc(&hx->hv_unit_ptr, (size_t)nh + 1)); TRY(palloc(&hx->unit_hv, nu));
    if (n_rows > 0) {
        k_heavy_emit<<<grid_for(n_rows), TB, 0, st>>>(n_rows, flag, hpos, units, upos, hx->hv_row,
                                                     hx->hv_unit_ptr, hx->unit_hv);
        KGE_LAUNCH_CHECK();
    }
    int32_t nu_i = (int32_t)nu;
    KGE_HIP(hipMemcpyAsync(hx->hv_unit_ptr + nh, &nu_i, sizeof(int32_t), hipMemcpyHostToDevice, st));
    KGE_HIP(hipStreamSynchronize(st));
    return KGE_OK;
}

int build_impl(const int32_t *h_head, const int32_t *h_rel, const int32_t *h_tail, int64_t M,
               int32_t n_ent, int32_t n_rel, int32_t n_parts, int32_t part_id, int32_t n_hops,
               int32_t neg_domain, kge_partition *p)
{
    hipStream_t st = nullptr;
    TempBufs tmp;
    int32_t *head, *rel, *tail;
    TRY(tmp.alloc(&head, M)); TRY(tmp.alloc(&rel, M)); TRY(tmp.alloc(&tail, M));
    KGE_HIP(hipMemcpy(head, h_head, sizeof(int32_t) * M, hipMemcpyHostToDevice));
    KGE_HIP(hipMemcpy(rel, h_rel, sizeof(int32_t) * M, hipMemcpyHostToDevice));
    KGE_HIP(hipMemcpy(tail, h_tail, sizeof(int32_t) * M, hipMemcpyHostToDevice));

    uint32_t *bad;
    TRY(tmp.alloc(&bad, 1));
    KGE_HIP(hipMemsetAsync(bad, 0, sizeof(uint32_t), st));
    if (M > 0) { k_check_ids<<<grid_for(M), TB, 0, st>>>(head, rel, tail, M, n_ent, n_rel, bad); KGE_LAUNCH_CHECK(); }
    uint32_t h_bad = 0;
    KGE_HIP(hipMemcpy(&h_bad, bad, sizeof(uint32_t), hipMemcpyDeviceToHost));
    KGE_REQUIRE(!h_bad, KGE_ERANGE, "a triple has an entity or relation id out of range");

    // --- core edges and S_0
    uint32_t *core_flag, *s0, *prev, *cur, *dstset;
    TRY(tmp.alloc(&core_flag, M)); TRY(tmp.alloc(&s0, n_ent)); TRY(tmp.alloc(&prev, n_ent));
    TRY(tmp.alloc(&cur, n_ent)); TRY(tmp.alloc(&dstset, n_ent));
    KGE_HIP(hipMemsetAsync(s0, 0, sizeof(uint32_t) * n_ent, st));
    KGE_HIP(hipMemsetAsync(dstset, 0, sizeof(uint32_t) * n_ent, st));
    if (M > 0) { k_mark_core<<<grid_for(M), TB, 0, st>>>(head, tail, M, (uint32_t)n_parts, (uint32_t)part_id, core_flag, s0); KGE_LAUNCH_CHECK(); }
    KGE_HIP(hipMemcpyAsync(cur, s0, sizeof(uint32_t) * n_ent, hipMemcpyDeviceToDevice, st));
    // --- expansion
    for (int k = 1; k <= n_hops; ++k) {
        KGE_HIP(hipMemcpyAsync(prev, cur, sizeof(uint32_t) * n_ent, hipMemcpyDeviceToDevice, st));
        if (M > 0) { k_expand<<<grid_for(M), TB, 0, st>>>(head, tail, M, prev, cur); KGE_LAUNCH_CHECK(); }
    }
    if (n_hops >= 1) KGE_HIP(hipMemcpyAsync(dstset, prev, sizeof(uint32_t) * n_ent, hipMemcpyDeviceToDevice, st));

    // --- local ids
    uint32_t *vpos;
    int32_t *lid;
    TRY(tmp.alloc(&vpos, (size_t)n_ent + 1)); TRY(tmp.alloc(&lid, n_ent));
    TRY(exclusive_scan(cur, vpos, n_ent, st));
    uint32_t N32 = 0;
    KGE_HIP(hipMemcpy(&N32, vpos + n_ent, sizeof(uint32_t), hipMemcpyDeviceToHost));
    const int64_t N = N32;
    p->n_vert = N;
    TRY(palloc(&p->vert_gid, N));
    k_vert_compact<<<grid_for(n_ent), TB, 0, st>>>(cur, vpos, n_ent, p->vert_gid, lid);
    KGE_LAUNCH_CHECK();

    // --- negative candidates
    if (neg_domain == KGE_DOMAIN_CORE) {
        uint32_t *cpos;
        TRY(tmp.alloc(&cpos, (size_t)n_ent + 1));
        TRY(exclusive_scan(s0, cpos, n_ent, st));
        uint32_t nc = 0;
        KGE_HIP(hipMemcpy(&nc, cpos + n_ent, sizeof(uint32_t), hipMemcpyDeviceToHost));
        p->n_cand = nc;
        TRY(palloc(&p->cand, nc));
        k_cand_compact<<<grid_for(n_ent), TB, 0, st>>>(s0, cpos, n_ent, lid, p->cand);
        KGE_LAUNCH_CHECK();
    } else {
        p->n_cand = N;
        TRY(palloc(&p->cand, N));
        if (N > 0) { k_iota<<<grid_for(N), TB, 0, st>>>(p->cand, N); KGE_LAUNCH_CHECK(); }
    }

    // --- core triples
    {
        uint32_t *kpos;
        TRY(tmp.alloc(&kpos, (size_t)M + 1));
        TRY(exclusive_scan(core_flag, kpos, M, st));
        uint32_t nk = 0;
        KGE_HIP(hipMemcpy(&nk, kpos + M, sizeof(uint32_t), hipMemcpyDeviceToHost));
        p->n_core = nk;
        TRY(palloc(&p->core_eid, nk)); TRY(palloc(&p->core_h, nk));
        TRY(palloc(&p->core_r, nk)); TRY(palloc(&p->core_t, nk));
        if (M > 0) {
            k_core_compact<<<grid_for(M), TB, 0, st>>>(core_flag, kpos, M, head, rel, tail, lid,
                                                      p->core_eid, p->core_h, p->core_r, p->core_t);
            KGE_LAUNCH_CHECK();
        }
    }

    // --- message edges into S_{L-1}
    const int vbits = bits_for((uint64_t)(N > 0 ? N : 1));
    const int rbits = bits_for((uint64_t)2 * n_rel);
    KGE_REQUIRE(rbits + 2 * vbits <= 64, KGE_ERANGE,
                "sort key needs %d bits (> 64): too many vertices or relations", rbits + 2 * vbits);
    uint32_t *eflag, *epos;
    TRY(tmp.alloc(&eflag, (size_t)2 * M)); TRY(tmp.alloc(&epos, (size_t)2 * M + 1));
    if (M > 0) { k_edge_flag<<<grid_for(2 * M), TB, 0, st>>>(head, tail, M, dstset, eflag); KGE_LAUNCH_CHECK(); }
    TRY(exclusive_scan(eflag, epos, 2 * M, st));
    uint32_t E32 = 0;
    KGE_HIP(hipMemcpy(&E32, epos + 2 * M, sizeof(uint32_t), hipMemcpyDeviceToHost));
    const int64_t E = E32;
    KGE_REQUIRE(E < 0x7fffffffLL, KGE_ERANGE, "too many message edges");
    p->n_edge = E;

    uint64_t *keys, *keys_alt;
    uint32_t *vals, *vals_alt;
    TRY(tmp.alloc(&keys, E)); TRY(tmp.alloc(&keys_alt, E));
    TRY(tmp.alloc(&vals, E)); TRY(tmp.alloc(&vals_alt, E));
    if (M > 0) {
        k_edge_emit<<<grid_for(2 * M), TB, 0, st>>>(head, rel, tail, M, n_rel, eflag, epos, lid, vbits, keys, vals);
        KGE_LAUNCH_CHECK();
    }
    TRY(radix_sort<uint64_t>(&keys, &vals, &keys_alt, &vals_alt, E, rbits + 2 * vbits, st));

    // --- runs
    uint32_t *sflag, *spos, *edge_seg;
    TRY(tmp.alloc(&sflag, E)); TRY(tmp.alloc(&spos, (size_t)E + 1)); TRY(tmp.alloc(&edge_seg, E));
    if (E > 0) { k_seg_flag<<<grid_for(E), TB, 0, st>>>(keys, E, vbits, sflag); KGE_LAUNCH_CHECK(); }
    TRY(exclusive_scan(sflag, spos, E, st));
    uint32_t S32 = 0;
    KGE_HIP(hipMemcpy(&S32, spos + E, sizeof(uint32_t), hipMemcpyDeviceToHost));
    const int64_t S = S32;
    p->n_seg = S;
    TRY(palloc(&p->seg_ptr, S + 1)); TRY(palloc(&p->seg_rel, S)); TRY(palloc(&p->seg_dst, S));
    TRY(palloc(&p->inv_c, S)); TRY(palloc(&p->col_src, E)); TRY(palloc(&p->edge_id, E));
    if (E > 0) {
        k_seg_emit<<<grid_for(E), TB, 0, st>>>(keys, vals, E, vbits, sflag, spos, p->seg_ptr, p->seg_rel,
                                              p->seg_dst, p->col_src, p->edge_id, edge_seg);
        KGE_LAUNCH_CHECK();
    }
    int32_t E_i32 = (int32_t)E;
    KGE_HIP(hipMemcpyAsync(p->seg_ptr + S, &E_i32, sizeof(int32_t), hipMemcpyHostToDevice, st));
    KGE_HIP(hipStreamSynchronize(st));
    if (S > 0) { k_inv_c<<<grid_for(S), TB, 0, st>>>(p->seg_ptr, S, p->inv_c); KGE_LAUNCH_CHECK(); }
    if (S > 0 && N + S < 0x7FFFFFFFll) {
        TRY(palloc(&p->seg_zrow, S));
        k_seg_zrow<<<grid_for(S), TB, 0, st>>>(p->seg_ptr, p->col_src, S, (int32_t)N, p->seg_zrow);
        KGE_LAUNCH_CHECK();
        uint32_t *mflag, *mpos;
        TRY(tmp.alloc(&mflag, S)); TRY(tmp.alloc(&mpos, (size_t)S + 1));
        k_multi_flag<<<grid_for(S), TB, 0, st>>>(p->seg_ptr, S, mflag);
        KGE_LAUNCH_CHECK();
        TRY(exclusive_scan(mflag, mpos, S, st));
        uint32_t n_multi = 0;
        KGE_HIP(hipMemcpy(&n_multi, mpos + S, sizeof(uint32_t), hipMemcpyDeviceToHost));
        p->n_mrun = n_multi;
        TRY(palloc(&p->mrun, n_multi));
        if (n_multi > 0) { k_multi_emit<<<grid_for(S), TB, 0, st>>>(mflag, mpos, S, p->mrun); KGE_LAUNCH_CHECK(); }
    }
    TRY(palloc(&p->rel_ptr, (size_t)2 * n_rel + 1));
    k_ptr_from_sorted<int32_t><<<grid_for(S + 1), TB, 0, st>>>(p->seg_rel, S, 2 * (int64_t)n_rel, p->rel_ptr);
    KGE_LAUNCH_CHECK();

    // --- destination-major and source-major views: stable sorts of edge positions
    TRY(palloc(&p->dm_ptr, N + 1)); TRY(palloc(&p->dm_src, E)); TRY(palloc(&p->dm_rel, E)); TRY(palloc(&p->dm_invc, E));
    TRY(palloc(&p->sm_ptr, N + 1)); TRY(palloc(&p->sm_dst, E)); TRY(palloc(&p->sm_rel, E)); TRY(palloc(&p->sm_invc, E));
    TRY(palloc(&p->sm_seg, E));
    uint32_t *k2, *k2_alt, *v2, *v2_alt;
    TRY(tmp.alloc(&k2, E)); TRY(tmp.alloc(&k2_alt, E)); TRY(tmp.alloc(&v2, E)); TRY(tmp.alloc(&v2_alt, E));
    int32_t *maxdeg;
    TRY(tmp.alloc(&maxdeg, 2));
    KGE_HIP(hipMemsetAsync(maxdeg, 0, 2 * sizeof(int32_t), st));
    const uint64_t vmask = (1ull << vbits) - 1ull;
    for (int view = 0; view < 2; ++view) {
        const int key_shift = view == 0 ? vbits : 0;       // sort by dst (view 0) or src (view 1)
        const int other_shift = view == 0 ? 0 : vbits;
        int32_t *ptr = view == 0 ? p->dm_ptr : p->sm_ptr;
        if (E > 0) { k_view_keys<<<grid_for(E), TB, 0, st>>>(keys, E, key_shift, vmask, k2, v2); KGE_LAUNCH_CHECK(); }
        TRY(radix_sort<uint32_t>(&k2, &v2, &k2_alt, &v2_alt, E, vbits, st));
        if (E > 0) {
            k_view_emit<<<grid_for(E), TB, 0, st>>>(v2, E, keys, vbits, other_shift, edge_seg, p->inv_c,
                                                   view == 0 ? p->dm_src : p->sm_dst,
                                                   view == 0 ? p->dm_rel : p->sm_rel,
                                                   view == 0 ? p->dm_invc : p->sm_invc,
                                                   view == 0 ? nullptr : p->sm_seg);
            KGE_LAUNCH_CHECK();
        }
        k_ptr_from_sorted<uint32_t><<<grid_for(E + 1), TB, 0, st>>>(k2, E, N, ptr);
        KGE_LAUNCH_CHECK();
        if (N > 0) { k_max_degree<<<grid_for(N), TB, 0, st>>>(ptr, N, maxdeg + view); KGE_LAUNCH_CHECK(); }
    }
    TRY(build_heavy_index(p->dm_ptr, N, &p->hv_dm, st));
    TRY(build_heavy_index(p->sm_ptr, N, &p->hv_sm, st));
    TRY(build_heavy_index(p->seg_ptr, S, &p->hv_seg, st));

    // --- the runs grouped by destination: a stable sort of run ids by destination keeps the
    // relation order inside a destination
    TRY(palloc(&p->dr_ptr, N + 1)); TRY(palloc(&p->dr_seg, S)); TRY(palloc(&p->dr_rel, S));
    {
        uint32_t *rk, *rk_alt, *rv, *rv_alt;
        TRY(tmp.alloc(&rk, S)); TRY(tmp.alloc(&rk_alt, S)); TRY(tmp.alloc(&rv, S)); TRY(tmp.alloc(&rv_alt, S));
        if (S > 0) { k_run_keys<<<grid_for(S), TB, 0, st>>>(p->seg_dst, S, rk, rv); KGE_LAUNCH_CHECK(); }
        TRY(radix_sort<uint32_t>(&rk, &rv, &rk_alt, &rv_alt, S, vbits, st));
        if (S > 0) { k_run_emit<<<grid_for(S), TB, 0, st>>>(rv, S, p->seg_rel, p->dr_seg, p->dr_rel); KGE_LAUNCH_CHECK(); }
        k_ptr_from_sorted<uint32_t><<<grid_for(S + 1), TB, 0, st>>>(rk, S, N, p->dr_ptr);
        KGE_LAUNCH_CHECK();
    }
    TRY(build_heavy_index(p->dr_ptr, N, &p->hv_dr, st));

    // --- chunks of each relation's run range (host side: 2R+1 offsets)
    {
        const int64_t R2 = 2 * (int64_t)n_rel;
        std::vector<int32_t> h_rel_ptr((size_t)R2 + 1), c_rel, c_beg, c_end, t_rel, t_beg, t_end;
        KGE_HIP(hipMemcpy(h_rel_ptr.data(), p->rel_ptr, sizeof(int32_t) * (size_t)(R2 + 1), hipMemcpyDeviceToHost));
        // chunk length: about 2048 chunks over all runs (every chunk ends in one atomic accumulation of a
        // whole d_in x d_out tile, so fewer, longer chunks are cheaper as long as the chip stays full)
        int32_t chunk = (int32_t)((S / 2048 + 31) / 32 * 32);
        if (chunk < KGE_REL_CHUNK) chunk = KGE_REL_CHUNK;
        if (chunk > 8 * KGE_REL_CHUNK) chunk = 8 * KGE_REL_CHUNK;
        // and into row tiles of at most KGE_REL_TILE runs (one output tile of the per-relation products)
        for (int64_t r = 0; r < R2; ++r)
            for (int32_t b = h_rel_ptr[r]; b < h_rel_ptr[r + 1]; b += KGE_REL_TILE) {
                t_rel.push_back((int32_t)r); t_beg.push_back(b);
                t_end.push_back(b + KGE_REL_TILE < h_rel_ptr[r + 1] ? b + KGE_REL_TILE : h_rel_ptr[r + 1]);
            }
        // Ranges of at most KGE_REL_RANGE runs of one relation (what a block of the bf16 per-run products takes),
        // ordered by slab of the destination range first and relation second.  A relation's runs are sorted by
        // destination, so a slab is a sub-range of them, and the blocks that run at the same time then gather the
        // output-gradient rows of one slab, which the last-level cache holds (KGE_REL_SLAB vertices: 128 MB of
        // bf16 rows at d = 256): the transposed products 4.95 -> 4.68 ms per launch at 25 M runs with four slabs.  A relation with fewer than two ranges' worth of runs stays whole, in the
        // first slab's group: cutting it would only make blocks with little to do (with those cut as well the
        // forward products lost what the transposed ones gained).
        const int64_t n_slabs = N > g_rel_slab ? cdiv(N, g_rel_slab) : 1;
        const int64_t slab = cdiv(N, n_slabs);
        std::vector<int32_t> h_dst;
        if (n_slabs > 1) {
            h_dst.resize((size_t)S);
            KGE_HIP(hipMemcpy(h_dst.data(), p->seg_dst, sizeof(int32_t) * (size_t)S, hipMemcpyDeviceToHost));
        }
        auto slab_ordered = [&](int32_t piece, std::vector<int32_t> &o_rel, std::vector<int32_t> &o_beg,
                                std::vector<int32_t> &o_end) {
            std::vector<int32_t> cut((size_t)R2 * (n_slabs + 1));     // cut[r][k]: first run of relation r in slab k
            for (int64_t r = 0; r < R2; ++r) {
                int32_t *c = cut.data() + r * (n_slabs + 1);
                c[0] = h_rel_ptr[r];
                c[n_slabs] = h_rel_ptr[r + 1];
                const bool whole = (int64_t)h_rel_ptr[r + 1] - h_rel_ptr[r] < (g_rel_min_runs > 0 ? g_rel_min_runs : 2 * (int64_t)piece);
                for (int64_t k = 1; k < n_slabs; ++k) {
                    if (whole) { c[k] = h_rel_ptr[r + 1]; continue; }
                    const int32_t *b0 = h_dst.data() + h_rel_ptr[r], *b1 = h_dst.data() + h_rel_ptr[r + 1];
                    c[k] = h_rel_ptr[r] + (int32_t)(std::lower_bound(b0, b1, (int32_t)(k * slab)) - b0);
                }
            }
            for (int64_t k = 0; k < n_slabs; ++k)
                for (int64_t r = 0; r < R2; ++r) {
                    const int32_t lo = cut[r * (n_slabs + 1) + k], hi = cut[r * (n_slabs + 1) + k + 1];
                    for (int32_t b = lo; b < hi; b += piece) {
                        o_rel.push_back((int32_t)r); o_beg.push_back(b);
                        o_end.push_back(b + piece < hi ? b + piece : hi);
                    }
                }
        };
        // the chunks keep the plain order, relation by relation: cut by slab they made the relation matrices'
        // gradient slower (4.23 against 3.9 ms per launch at 25 M runs)
        for (int64_t r = 0; r < R2; ++r)
            for (int32_t b = h_rel_ptr[r]; b < h_rel_ptr[r + 1]; b += chunk) {
                c_rel.push_back((int32_t)r); c_beg.push_back(b);
                c_end.push_back(b + chunk < h_rel_ptr[r + 1] ? b + chunk : h_rel_ptr[r + 1]);
            }
        {
            std::vector<int32_t> g_rel, g_beg, g_end;
            slab_ordered(KGE_REL_RANGE, g_rel, g_beg, g_end);
            p->n_rels = (int32_t)g_rel.size();
            TRY(palloc(&p->rels_rel, g_rel.size())); TRY(palloc(&p->rels_beg, g_rel.size())); TRY(palloc(&p->rels_end, g_rel.size()));
            if (!g_rel.empty()) {
                KGE_HIP(hipMemcpy(p->rels_rel, g_rel.data(), sizeof(int32_t) * g_rel.size(), hipMemcpyHostToDevice));
                KGE_HIP(hipMemcpy(p->rels_beg, g_beg.data(), sizeof(int32_t) * g_beg.size(), hipMemcpyHostToDevice));
                KGE_HIP(hipMemcpy(p->rels_end, g_end.data(), sizeof(int32_t) * g_end.size(), hipMemcpyHostToDevice));
            }
        }
        {
            // and in the plain order, relation by relation, for the forward products (their rows are gathered by
            // source: the slab order gains them nothing and its extra ranges cost 0.1 ms per launch)
            std::vector<int32_t> g_rel, g_beg, g_end;
            for (int64_t r = 0; r < R2; ++r)
                for (int32_t b = h_rel_ptr[r]; b < h_rel_ptr[r + 1]; b += KGE_REL_RANGE) {
                    g_rel.push_back((int32_t)r); g_beg.push_back(b);
                    g_end.push_back(b + KGE_REL_RANGE < h_rel_ptr[r + 1] ? b + KGE_REL_RANGE : h_rel_ptr[r + 1]);
                }
            p->n_relr = (int32_t)g_rel.size();
            TRY(palloc(&p->relr_rel, g_rel.size())); TRY(palloc(&p->relr_beg, g_rel.size())); TRY(palloc(&p->relr_end, g_rel.size()));
            if (!g_rel.empty()) {
                KGE_HIP(hipMemcpy(p->relr_rel, g_rel.data(), sizeof(int32_t) * g_rel.size(), hipMemcpyHostToDevice));
                KGE_HIP(hipMemcpy(p->relr_beg, g_beg.data(), sizeof(int32_t) * g_beg.size(), hipMemcpyHostToDevice));
                KGE_HIP(hipMemcpy(p->relr_end, g_end.data(), sizeof(int32_t) * g_end.size(), hipMemcpyHostToDevice));
            }
        }
        p->n_relt = (int32_t)t_rel.size();
        TRY(palloc(&p->relt_rel, t_rel.size())); TRY(palloc(&p->relt_beg, t_rel.size())); TRY(palloc(&p->relt_end, t_rel.size()));
        if (!t_rel.empty()) {
            KGE_HIP(hipMemcpy(p->relt_rel, t_rel.data(), sizeof(int32_t) * t_rel.size(), hipMemcpyHostToDevice));
            KGE_HIP(hipMemcpy(p->relt_beg, t_beg.data(), sizeof(int32_t) * t_beg.size(), hipMemcpyHostToDevice));
            KGE_HIP(hipMemcpy(p->relt_end, t_end.data(), sizeof(int32_t) * t_end.size(), hipMemcpyHostToDevice));
        }
        p->n_relc = (int32_t)c_rel.size();
        TRY(palloc(&p->relc_rel, c_rel.size())); TRY(palloc(&p->relc_beg, c_rel.size())); TRY(palloc(&p->relc_end, c_rel.size()));
        if (!c_rel.empty()) {
            KGE_HIP(hipMemcpy(p->relc_rel, c_rel.data(), sizeof(int32_t) * c_rel.size(), hipMemcpyHostToDevice));
            KGE_HIP(hipMemcpy(p->relc_beg, c_beg.data(), sizeof(int32_t) * c_beg.size(), hipMemcpyHostToDevice));
            KGE_HIP(hipMemcpy(p->relc_end, c_end.data(), sizeof(int32_t) * c_end.size(), hipMemcpyHostToDevice));
        }
    }
    int32_t h_maxdeg[2] = {0, 0};
    KGE_HIP(hipMemcpy(h_maxdeg, maxdeg, sizeof(h_maxdeg), hipMemcpyDeviceToHost));
    p->max_in_degree = h_maxdeg[0];
    p->max_out_degree = h_maxdeg[1];
    KGE_HIP(hipStreamSynchronize(st));
    return KGE_OK;
}

}  // namespace

// ------------------------------------------------------------------ ABI
extern "C" void kge_test_set_rel_slab(int32_t vertices, int32_t min_runs)
{
    g_rel_slab = vertices > 0 ? vertices : KGE_REL_SLAB;
    g_rel_min_runs = min_runs > 0 ? min_runs : 0;
}

static thread_local char g_err[512] = "";

void kge_set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

extern "C" const char *kge_last_error(void) { return g_err; }

extern "C" void kge_partition_destroy(kge_partition *p)
{
    if (!p) return;
    void *arrs[] = {p->vert_gid, p->core_eid, p->core_h, p->core_r, p->core_t, p->seg_ptr, p->seg_rel,
                    p->seg_dst, p->inv_c, p->col_src, p->edge_id, p->cand, p->dm_ptr, p->dm_src,
                    p->dm_rel, p->dm_invc, p->sm_ptr, p->sm_dst, p->sm_rel, p->sm_invc, p->rel_ptr,
                    p->hv_dm.hv_row, p->hv_dm.hv_unit_ptr, p->hv_dm.unit_hv,
                    p->hv_sm.hv_row, p->hv_sm.hv_unit_ptr, p->hv_sm.unit_hv,
                    p->hv_seg.hv_row, p->hv_seg.hv_unit_ptr, p->hv_seg.unit_hv,
                    p->dr_ptr, p->dr_seg, p->dr_rel, p->hv_dr.hv_row, p->hv_dr.hv_unit_ptr, p->hv_dr.unit_hv,
                    p->relc_rel, p->relc_beg, p->relc_end, p->sm_seg, p->relt_rel, p->relt_beg, p->relt_end,
                    p->relr_rel, p->relr_beg, p->relr_end, p->rels_rel, p->rels_beg, p->rels_end, p->seg_zrow, p->mrun,
                    p->bad_ids};
    for (void *q : arrs) if (q) (void)hipFree(q);
    delete p;
}

extern "C" int kge_build_partition(const int32_t *head, const int32_t *rel, const int32_t *tail,
                                   int64_t n_triples, int32_t n_entities, int32_t n_relations,
                                   int32_t n_parts, int32_t part_id, int32_t n_hops,
                                   int32_t neg_domain, kge_partition **out)
{
    KGE_REQUIRE(out, KGE_EINVAL, "out is NULL");
    *out = nullptr;
    KGE_REQUIRE(n_triples >= 0 && (n_triples == 0 || (head && rel && tail)), KGE_EINVAL,
                "triple arrays are NULL or n_triples < 0");
    KGE_REQUIRE(n_entities > 0 && n_relations > 0, KGE_EINVAL, "n_entities and n_relations must be positive");
    KGE_REQUIRE(n_parts > 0 && part_id >= 0 && part_id < n_parts, KGE_EINVAL, "bad n_parts / part_id");
    KGE_REQUIRE(n_hops >= 0 && n_hops <= 16, KGE_EINVAL, "n_hops must be in [0, 16]");
    KGE_REQUIRE(neg_domain == KGE_DOMAIN_CORE || neg_domain == KGE_DOMAIN_ALL, KGE_EINVAL, "bad neg_domain");
    KGE_REQUIRE(n_triples < 0x3fffffffLL, KGE_ERANGE, "n_triples must be below 2^30");
    KGE_REQUIRE(n_relations < 0x3fffffff, KGE_ERANGE, "n_relations too large");
    kge_partition *p = new kge_partition();
    memset(p, 0, sizeof *p);
    KGE_HIP(hipGetDevice(&p->device));
    p->n_triples = n_triples; p->n_entities = n_entities; p->n_relations = n_relations;
    p->n_parts = n_parts; p->part_id = part_id; p->n_hops = n_hops; p->neg_domain = neg_domain;
    int rc = build_impl(head, rel, tail, n_triples, n_entities, n_relations, n_parts, part_id,
                        n_hops, neg_domain, p);
    if (rc != KGE_OK) { kge_partition_destroy(p); return rc; }
    hipError_t e = hipMalloc((void **)&p->bad_ids, sizeof(uint32_t));
    if (e == hipSuccess) e = hipMemset(p->bad_ids, 0, sizeof(uint32_t));
    if (e != hipSuccess) {
        kge_set_error("allocating the partition's id counter failed: %s", hipGetErrorString(e));
        kge_partition_destroy(p);
        return KGE_ENOMEM;
    }
    *out = p;
    return KGE_OK;
}

extern "C" int kge_partition_bad_ids(const kge_partition *p, int64_t *host_count)
{
    KGE_REQUIRE(p && host_count, KGE_EINVAL, "NULL argument");
    uint32_t n = 0;
    KGE_HIP(hipDeviceSynchronize());
    KGE_HIP(hipMemcpy(&n, p->bad_ids, sizeof n, hipMemcpyDeviceToHost));
    *host_count = (int64_t)n;
    return KGE_OK;
}

extern "C" int kge_partition_info(const kge_partition *p, kge_part_info *o)
{
    KGE_REQUIRE(p && o, KGE_EINVAL, "NULL argument");
    o->n_vert = p->n_vert; o->n_edge = p->n_edge; o->n_seg = p->n_seg; o->n_core = p->n_core;
    o->n_cand = p->n_cand; o->n_triples = p->n_triples; o->n_entities = p->n_entities;
    o->n_relations = p->n_relations; o->n_parts = p->n_parts; o->part_id = p->part_id;
    o->n_hops = p->n_hops; o->neg_domain = p->neg_domain; o->max_in_degree = p->max_in_degree;
    o->max_out_degree = p->max_out_degree;
    return KGE_OK;
}

extern "C" int kge_partition_export(const kge_partition *p, int32_t which, void *host_dst, int64_t bytes)
{
    KGE_REQUIRE(p && (host_dst || bytes == 0), KGE_EINVAL, "NULL argument");
    const void *src = nullptr;
    int64_t n = 0;
    switch (which) {
    case KGE_ARR_VERT_GID: src = p->vert_gid; n = p->n_vert; break;
    case KGE_ARR_CORE_EID: src = p->core_eid; n = p->n_core; break;
    case KGE_ARR_CORE_H: src = p->core_h; n = p->n_core; break;
    case KGE_ARR_CORE_R: src = p->core_r; n = p->n_core; break;
    case KGE_ARR_CORE_T: src = p->core_t; n = p->n_core; break;
    case KGE_ARR_SEG_PTR: src = p->seg_ptr; n = p->n_seg + 1; break;
    case KGE_ARR_SEG_REL: src = p->seg_rel; n = p->n_seg; break;
    case KGE_ARR_SEG_DST: src = p->seg_dst; n = p->n_seg; break;
    case KGE_ARR_INV_C: src = p->inv_c; n = p->n_seg; break;
    case KGE_ARR_COL_SRC: src = p->col_src; n = p->n_edge; break;
    case KGE_ARR_EDGE_ID: src = p->edge_id; n = p->n_edge; break;
    case KGE_ARR_CAND: src = p->cand; n = p->n_cand; break;
    case KGE_ARR_DM_PTR: src = p->dm_ptr; n = p->n_vert + 1; break;
    case KGE_ARR_DM_SRC: src = p->dm_src; n = p->n_edge; break;
    case KGE_ARR_DM_REL: src = p->dm_rel; n = p->n_edge; break;
    case KGE_ARR_DM_INVC: src = p->dm_invc; n = p->n_edge; break;
    case KGE_ARR_SM_PTR: src = p->sm_ptr; n = p->n_vert + 1; break;
    case KGE_ARR_SM_DST: src = p->sm_dst; n = p->n_edge; break;
    case KGE_ARR_SM_REL: src = p->sm_rel; n = p->n_edge; break;
    case KGE_ARR_SM_INVC: src = p->sm_invc; n = p->n_edge; break;
    case KGE_ARR_REL_PTR: src = p->rel_ptr; n = 2 * (int64_t)p->n_relations + 1; break;
    case KGE_ARR_DR_PTR: src = p->dr_ptr; n = p->n_vert + 1; break;
    case KGE_ARR_DR_SEG: src = p->dr_seg; n = p->n_seg; break;
    case KGE_ARR_DR_REL: src = p->dr_rel; n = p->n_seg; break;
    case KGE_ARR_SM_SEG: src = p->sm_seg; n = p->n_edge; break;
    default: KGE_REQUIRE(false, KGE_EINVAL, "unknown array id %d", which);
    }
    KGE_REQUIRE(bytes == 4 * n, KGE_EINVAL, "array %d has %lld bytes, caller gave %lld", which,
                (long long)(4 * n), (long long)bytes);
    if (n > 0) KGE_HIP(hipMemcpy(host_dst, src, (size_t)bytes, hipMemcpyDeviceToHost));
    return KGE_OK;
}
