// Computational sub-graph of one edge batch (Sec. 3.3, Algorithm 1 "getComputeGraph"), on the GPU.
//
// The batch's embeddings after the last layer depend only on vertices within L hops along incoming
// message edges.  active[l][i] (one byte per vertex) says whether layer l+1 must produce a row for
// vertex i:  active[L-1] = the batch's vertices;  active[l-1] = active[l] united with the sources
// of all edges into active[l].  The aggregation kernels skip every other destination, which is
// exact: those rows never reach the batch, and their upstream gradients are zero.
//
// Marking is idempotent (every writer stores the byte 1), so no atomics are needed; the counts
// are integer sums and therefore exact whatever the order.
#include "common.h"

struct kge_cgraph {
    int device;
    int64_t N, stride;      // vertices; bytes between the layers' flag rows
    int32_t n_layers;
    uint8_t *active;        // [n_layers + 1][stride]; row n_layers: the rows of the first layer's INPUT the step reads
    unsigned long long *stats;   // [n_layers + 1][4]: active vertices, edges into them, runs into them, edges out of them
};

namespace {

__global__ void k_cg_mark_batch(const int32_t *__restrict__ core_h, const int32_t *__restrict__ core_t,
                                const int32_t *__restrict__ pos, int64_t n_pos,
                                const int32_t *__restrict__ neg_ent, int64_t n_neg_entries,
                                uint32_t n_vert, uint32_t n_core, uint32_t *__restrict__ bad,
                                uint8_t *__restrict__ top)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_pos) {
        const uint32_t c = (uint32_t)pos[i];
        if (c >= n_core) { atomicAdd(bad, 1u); return; }      // outside the partition: counted, never an address
        top[core_h[c]] = 1;
        top[core_t[c]] = 1;
    } else if (i - n_pos < n_neg_entries) {
        const uint32_t e = (uint32_t)neg_ent[i - n_pos];
        if (e >= n_vert) { atomicAdd(bad, 1u); return; }
        top[e] = 1;
    }
}

// One wavefront per destination of the destination-major view.
__global__ __launch_bounds__(256) void k_cg_expand(const int32_t *__restrict__ dm_ptr,
                                                   const int32_t *__restrict__ dm_src, int64_t N,
                                                   const uint8_t *__restrict__ cur, uint8_t *__restrict__ below)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= N || !cur[i]) return;
    if (lane == 0) below[i] = 1;
    const int32_t end = dm_ptr[i + 1];
    for (int32_t e = dm_ptr[i] + lane; e < end; e += 64) below[dm_src[e]] = 1;
}

__device__ __forceinline__ void block_add4(unsigned long long a, unsigned long long b, unsigned long long c,
                                           unsigned long long e, unsigned long long *out)
{
    __shared__ unsigned long long red[4][4];
    for (int off = 32; off > 0; off >>= 1) {
        a += __shfl_xor(a, off, 64); b += __shfl_xor(b, off, 64); c += __shfl_xor(c, off, 64);
        e += __shfl_xor(e, off, 64);
    }
    const int wv = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { red[0][wv] = a; red[1][wv] = b; red[2][wv] = c; red[3][wv] = e; }
    __syncthreads();
    if (threadIdx.x < 4) {
        unsigned long long sum = 0;
        for (int k = 0; k < 4; ++k) sum += red[threadIdx.x][k];
        if (sum) atomicAdd(out + threadIdx.x, sum);
    }
}

// counts of one layer: active vertices and edges (over vertices), active runs (over runs)
__global__ __launch_bounds__(256) void k_cg_stats(const int32_t *__restrict__ dm_ptr,
                                                  const int32_t *__restrict__ sm_ptr, int64_t N,
                                                  const int32_t *__restrict__ seg_dst, int64_t S,
                                                  const uint8_t *__restrict__ act, unsigned long long *out)
{
    unsigned long long nv = 0, ne = 0, ns = 0, no = 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += stride)
        if (act[i]) {
            nv += 1;
            ne += (unsigned long long)(dm_ptr[i + 1] - dm_ptr[i]);
            no += (unsigned long long)(sm_ptr[i + 1] - sm_ptr[i]);
        }
    for (int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; s < S; s += stride)
        if (act[seg_dst[s]]) ns += 1;
    block_add4(nv, ne, ns, no, out);
}

}  // namespace

extern "C" int kge_cgraph_create(const kge_partition *p, int32_t n_layers, kge_cgraph **out)
{
    KGE_REQUIRE(p && out, KGE_EINVAL, "NULL argument");
    KGE_REQUIRE(n_layers >= 1 && n_layers <= 16, KGE_EINVAL, "n_layers must be in [1, 16]");
    *out = nullptr;
    kge_cgraph *cg = new kge_cgraph();
    cg->device = p->device;
    cg->N = p->n_vert;
    cg->stride = (int64_t)align_up((size_t)(p->n_vert > 0 ? p->n_vert : 1), 256);
    cg->n_layers = n_layers;
    cg->active = nullptr;
    cg->stats = nullptr;
    hipError_t e = hipMalloc((void **)&cg->active, (size_t)cg->stride * (n_layers + 1));
    if (e == hipSuccess) e = hipMalloc((void **)&cg->stats, sizeof(unsigned long long) * 4 * (n_layers + 1));
    if (e == hipSuccess) e = hipMemset(cg->active, 0, (size_t)cg->stride * (n_layers + 1));
    if (e == hipSuccess) e = hipMemset(cg->stats, 0, sizeof(unsigned long long) * 4 * (n_layers + 1));
    if (e != hipSuccess) {
        kge_set_error("allocating the sub-graph flags failed: %s", hipGetErrorString(e));
        if (cg->active) (void)hipFree(cg->active);
        if (cg->stats) (void)hipFree(cg->stats);
        delete cg;
        return KGE_EHIP;
    }
    *out = cg;
    return KGE_OK;
}

extern "C" void kge_cgraph_destroy(kge_cgraph *cg)
{
    if (!cg) return;
    (void)hipFree(cg->active);
    (void)hipFree(cg->stats);
    delete cg;
}

extern "C" int kge_compute_graph(const kge_partition *p, kge_cgraph *cg, const int32_t *pos_core_idx,
                                 int64_t n_pos, const int32_t *neg_ent, int64_t n_neg_entries, void *stream)
{
    KGE_REQUIRE(p && cg, KGE_EINVAL, "NULL partition or sub-graph object");
    KGE_REQUIRE(cg->N == p->n_vert && cg->device == p->device, KGE_EINVAL,
                "the sub-graph object was created for another partition");
    KGE_REQUIRE(n_pos >= 0 && n_neg_entries >= 0, KGE_EINVAL, "negative count");
    KGE_REQUIRE(n_pos == 0 || pos_core_idx, KGE_EINVAL, "pos_core_idx is NULL");
    KGE_REQUIRE(n_neg_entries == 0 || neg_ent, KGE_EINVAL, "neg_ent is NULL");
    KGE_REQUIRE(n_pos == 0 || p->n_core > 0, KGE_EINVAL, "the partition has no core edge");
    hipStream_t st = (hipStream_t)stream;
    const int L = cg->n_layers;
    KGE_PROF("compute_graph", st);
    int rc = launch_fill_zero(cg->active, (size_t)cg->stride * (L + 1), st);
    if (rc != KGE_OK) return rc;
    rc = launch_fill_zero(cg->stats, sizeof(unsigned long long) * 4 * (L + 1), st);
    if (rc != KGE_OK) return rc;
    if (p->n_vert == 0) return KGE_OK;
    const int64_t n_mark = n_pos + n_neg_entries;
    if (n_mark > 0) {
        k_cg_mark_batch<<<(unsigned)cdiv(n_mark, 256), 256, 0, st>>>(p->core_h, p->core_t, pos_core_idx, n_pos,
                                                                    neg_ent, n_neg_entries, (uint32_t)p->n_vert,
                                                                    (uint32_t)p->n_core, p->bad_ids,
                                                                    cg->active + (size_t)(L - 1) * cg->stride);
        KGE_LAUNCH_CHECK();
    }
    for (int l = L - 1; l >= 1; --l) {
        k_cg_expand<<<(unsigned)cdiv(p->n_vert, 4), 256, 0, st>>>(p->dm_ptr, p->dm_src, p->n_vert,
                                                                 cg->active + (size_t)l * cg->stride,
                                                                 cg->active + (size_t)(l - 1) * cg->stride);
        KGE_LAUNCH_CHECK();
    }
    // one hop further: the rows of the first layer's input that layer reads (its active destinations and the
    // sources of every edge into them) - the embedding rows this step has a gradient for
    k_cg_expand<<<(unsigned)cdiv(p->n_vert, 4), 256, 0, st>>>(p->dm_ptr, p->dm_src, p->n_vert, cg->active,
                                                             cg->active + (size_t)L * cg->stride);
    KGE_LAUNCH_CHECK();
    for (int l = 0; l <= L; ++l) {
        k_cg_stats<<<1024, 256, 0, st>>>(p->dm_ptr, p->sm_ptr, p->n_vert, p->seg_dst, p->n_seg,
                                         cg->active + (size_t)l * cg->stride, cg->stats + 4 * l);
        KGE_LAUNCH_CHECK();
    }
    return KGE_OK;
}

extern "C" int kge_cgraph_input_rows(const kge_cgraph *cg, const uint8_t **device_flags, uint8_t *host_flags,
                                     int64_t *host_count)
{
    KGE_REQUIRE(cg, KGE_EINVAL, "NULL sub-graph object");
    const uint8_t *row = cg->active + (size_t)cg->n_layers * cg->stride;
    if (device_flags) *device_flags = row;
    if (host_flags || host_count) {
        KGE_HIP(hipDeviceSynchronize());
        if (host_flags) KGE_HIP(hipMemcpy(host_flags, row, (size_t)cg->N, hipMemcpyDeviceToHost));
        if (host_count) {
            unsigned long long n = 0;
            KGE_HIP(hipMemcpy(&n, cg->stats + 4 * cg->n_layers, sizeof n, hipMemcpyDeviceToHost));
            *host_count = (int64_t)n;
        }
    }
    return KGE_OK;
}

extern "C" int kge_cgraph_export(const kge_cgraph *cg, uint8_t *host_active, int64_t *host_stats)
{
    KGE_REQUIRE(cg, KGE_EINVAL, "NULL sub-graph object");
    KGE_HIP(hipDeviceSynchronize());
    if (host_active)
        for (int l = 0; l < cg->n_layers; ++l)
            KGE_HIP(hipMemcpy(host_active + (size_t)l * cg->N, cg->active + (size_t)l * cg->stride, (size_t)cg->N,
                              hipMemcpyDeviceToHost));
    if (host_stats) {
        unsigned long long tmp[64];
        KGE_HIP(hipMemcpy(tmp, cg->stats, sizeof(unsigned long long) * 4 * cg->n_layers, hipMemcpyDeviceToHost));
        for (int k = 0; k < 4 * cg->n_layers; ++k) host_stats[k] = (int64_t)tmp[k];
    }
    return KGE_OK;
}

const uint8_t *kge_cgraph_layer(const kge_cgraph *cg, int32_t layer)
{
    if (!cg) return nullptr;
    // layer -1: the rows of the first layer's input the batch reads (kept behind the layers' rows)
    return cg->active + (size_t)(layer < 0 ? cg->n_layers : layer) * cg->stride;
}

int kge_cgraph_check(const kge_partition *p, const kge_cgraph *cg, int32_t n_layers)
{
    if (!cg) return KGE_OK;
    KGE_REQUIRE(cg->N == p->n_vert && cg->device == p->device, KGE_EINVAL,
                "the sub-graph object was created for another partition");
    KGE_REQUIRE(cg->n_layers == n_layers, KGE_EINVAL, "the sub-graph object has %d layers, the model %d",
                cg->n_layers, n_layers);
    return KGE_OK;
}
