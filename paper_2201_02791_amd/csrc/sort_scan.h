// Stable LSD radix sort and exclusive scan on the GPU, with caller-provided scratch: only kernel launches,
// so they can run inside the per-step calls (no allocation, no synchronisation).  Used by the partition
// build and by the per-batch index of the scoring call.  Everything lives in an anonymous namespace: each
// translation unit that includes this header gets its own copy of the kernels.
#pragma once
#include "common.h"

namespace {

constexpr int TB = 256;              // threads per block (4 wavefronts of 64)
constexpr int SCAN_ITEMS = 8;        // items per thread in the scan kernels
constexpr int SCAN_TILE = TB * SCAN_ITEMS;
constexpr int SORT_ROWS = 8;         // 64-element rows per wavefront in a sort tile
constexpr int SORT_TILE = TB * SORT_ROWS;

// ---------------------------------------------------------------- scan
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    int lane = threadIdx.x & 63;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint32_t o = __shfl_up(v, off, 64);
        if (lane >= off) v += o;
    }
    return v;
}

// Inclusive scan of one value per thread across the block; returns the exclusive prefix of
// this thread and the block total.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *total)
{
    __shared__ uint32_t wsum[TB / 64];
    int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t inc = wave_incl_scan(v);
    if (lane == 63) wsum[w] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int k = 0; k < TB / 64; ++k) {
        uint32_t s = wsum[k];
        if (k < w) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

__global__ void k_scan_reduce(const uint32_t *in, int64_t n, uint32_t *block_sums)
{
    int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    uint32_t s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k)
        if (base + k < n) s += in[base + k];
    uint32_t tot;
    block_excl_scan(s, &tot);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = tot;
}

__global__ void k_scan_apply(const uint32_t *in, int64_t n, const uint32_t *block_offs, uint32_t *out)
{
    int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    uint32_t v[SCAN_ITEMS], s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        v[k] = (base + k < n) ? in[base + k] : 0u;
        s += v[k];
    }
    uint32_t tot;
    uint32_t run = block_excl_scan(s, &tot) + block_offs[blockIdx.x];
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        if (base + k < n) out[base + k] = run;
        run += v[k];
    }
}

// Single block: exclusive scan of up to any n (loops), writes total to out[n].
__global__ void k_scan_small(const uint32_t *in, int64_t n, uint32_t *out)
{
    __shared__ uint32_t carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int64_t start = 0; start < n; start += SCAN_TILE) {
        int64_t base = start + (int64_t)threadIdx.x * SCAN_ITEMS;
        uint32_t v[SCAN_ITEMS], s = 0;
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) {
            v[k] = (base + k < n) ? in[base + k] : 0u;
            s += v[k];
        }
        uint32_t tot;
        uint32_t run = block_excl_scan(s, &tot) + carry;
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) {
            if (base + k < n) out[base + k] = run;
            run += v[k];
        }
        __syncthreads();
        if (threadIdx.x == 0) carry += tot;
        __syncthreads();
    }
    if (threadIdx.x == 0) out[n] = carry;
}

__global__ void k_copy_word(const uint32_t *src, uint32_t *dst) { *dst = *src; }

// Words of scratch exclusive_scan_ws needs for n inputs (block sums and their offsets, level by level).
inline size_t scan_scratch_words(int64_t n)
{
    size_t words = 0;
    while (n > 4 * SCAN_TILE) {
        const int64_t nb = (n + SCAN_TILE - 1) / SCAN_TILE;
        words += 2 * (size_t)(nb + 1);
        n = nb;
    }
    return words;
}

// out[0..n) = exclusive prefix sums of in[0..n), out[n] = total.  out has n+1 entries and may not alias in.
// scratch: scan_scratch_words(n) words of device memory.  Only kernel launches on `st`: no allocation, no
// synchronisation, no memset or memcpy nodes (safe under graph capture).
inline int exclusive_scan_ws(const uint32_t *in, uint32_t *out, int64_t n, uint32_t *scratch, hipStream_t st)
{
    if (n <= 4 * SCAN_TILE) {
        k_scan_small<<<1, TB, 0, st>>>(in, n, out);
        KGE_LAUNCH_CHECK();
        return KGE_OK;
    }
    const int64_t nb = cdiv(n, SCAN_TILE);
    uint32_t *sums = scratch, *offs = scratch + (nb + 1);
    k_scan_reduce<<<(unsigned)nb, TB, 0, st>>>(in, n, sums);
    KGE_LAUNCH_CHECK();
    int rc = exclusive_scan_ws(sums, offs, nb, scratch + 2 * (nb + 1), st);
    if (rc != KGE_OK) return rc;
    k_scan_apply<<<(unsigned)nb, TB, 0, st>>>(in, n, offs, out);
    KGE_LAUNCH_CHECK();
    k_copy_word<<<1, 1, 0, st>>>(offs + nb, out + n);      // total
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

// ---------------------------------------------------------------- radix sort
// Stable LSD radix sort, 8 bits per pass.  A tile of SORT_TILE elements is split so that
// wavefront w owns the contiguous chunk [w*512, (w+1)*512): ascending index order is then
// (wavefront, row, lane), which is the order ranks are handed out in.
template <typename K>
__global__ void k_radix_hist(const K *keys, int64_t n, int shift, uint32_t *hist, int64_t nblk)
{
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    int64_t base = (int64_t)blockIdx.x * SORT_TILE;
#pragma unroll
    for (int k = 0; k < SORT_ROWS; ++k) {
        int64_t idx = base + (int64_t)k * TB + threadIdx.x;
        if (idx < n) atomicAdd(&h[(uint32_t)(keys[idx] >> shift) & 255u], 1u);
    }
    __syncthreads();
    hist[(int64_t)threadIdx.x * nblk + blockIdx.x] = h[threadIdx.x];
}

template <typename K>
__global__ void k_radix_scatter(const K *keys_in, const uint32_t *vals_in, K *keys_out,
                                uint32_t *vals_out, int64_t n, int shift, const uint32_t *offs,
                                int64_t nblk)
{
    __shared__ uint32_t cnt[TB / 64][256];
    __shared__ uint32_t base[TB / 64][256];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
    for (int k = 0; k < TB / 64; ++k) cnt[k][threadIdx.x] = 0;
    __syncthreads();

    const int64_t start = (int64_t)blockIdx.x * SORT_TILE + (int64_t)w * (64 * SORT_ROWS);
    K key[SORT_ROWS];
    uint32_t val[SORT_ROWS], rank[SORT_ROWS];
#pragma unroll
    for (int it = 0; it < SORT_ROWS; ++it) {
        int64_t idx = start + it * 64 + lane;
        bool valid = idx < n;
        key[it] = valid ? keys_in[idx] : (K)0;
        val[it] = valid ? vals_in[idx] : 0u;
        uint32_t digit = (uint32_t)(key[it] >> shift) & 255u;
        unsigned long long mask = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            bool bit = (digit >> b) & 1u;
            unsigned long long bal = __ballot(valid && bit);
            mask &= bit ? bal : ~bal;
        }
        // mask: valid lanes of this row holding the same digit as this lane
        uint32_t below = (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
        uint32_t same = (uint32_t)__popcll(mask);
        uint32_t prev = 0;
        if (valid && below == 0) {          // lowest lane of its digit group updates the counter
            prev = cnt[w][digit];
            cnt[w][digit] = prev + same;
        }
        int leader = valid ? (__ffsll((long long)mask) - 1) : lane;
        prev = __shfl(prev, leader, 64);
        rank[it] = prev + below;
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    {
        uint32_t run = offs[(int64_t)threadIdx.x * nblk + blockIdx.x];
#pragma unroll
        for (int k = 0; k < TB / 64; ++k) {
            base[k][threadIdx.x] = run;
            run += cnt[k][threadIdx.x];
        }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < SORT_ROWS; ++it) {
        int64_t idx = start + it * 64 + lane;
        if (idx < n) {
            uint32_t digit = (uint32_t)(key[it] >> shift) & 255u;
            uint32_t pos = base[w][digit] + rank[it];
            keys_out[pos] = key[it];
            vals_out[pos] = val[it];
        }
    }
}

// Words of scratch radix_sort_ws needs for n elements: the per-block digit histogram, its offsets, and the
// scan's own scratch.
inline size_t radix_scratch_words(int64_t n)
{
    const int64_t nblk = (n + SORT_TILE - 1) / SORT_TILE;
    return 2 * (size_t)(256 * nblk + 1) + scan_scratch_words(256 * nblk);
}

// Sort (keys, vals) by the low `bits` bits of the key, stable.  Buffers ping-pong; on return
// *keys / *vals point at the sorted data (either the original or the alternate buffers).
// scratch: radix_scratch_words(n) words.  Kernel launches on `st` only.
template <typename K>
int radix_sort_ws(K **keys, uint32_t **vals, K **keys_alt, uint32_t **vals_alt, int64_t n, int bits,
                  uint32_t *scratch, hipStream_t st)
{
    if (n == 0) return KGE_OK;
    const int64_t nblk = cdiv(n, SORT_TILE);
    uint32_t *hist = scratch, *offs = scratch + (256 * nblk + 1), *scan_ws = scratch + 2 * (256 * nblk + 1);
    for (int shift = 0; shift < bits; shift += 8) {
        k_radix_hist<K><<<(unsigned)nblk, TB, 0, st>>>(*keys, n, shift, hist, nblk);
        KGE_LAUNCH_CHECK();
        int rc = exclusive_scan_ws(hist, offs, 256 * nblk, scan_ws, st);
        if (rc != KGE_OK) return rc;
        k_radix_scatter<K><<<(unsigned)nblk, TB, 0, st>>>(*keys, *vals, *keys_alt, *vals_alt, n,
                                                         shift, offs, nblk);
        KGE_LAUNCH_CHECK();
        K *tk = *keys; *keys = *keys_alt; *keys_alt = tk;
        uint32_t *tv = *vals; *vals = *vals_alt; *vals_alt = tv;
    }
    return KGE_OK;
}

// ptr[v] = first position q with sorted[q] >= v, for v in [0, nv]; ptr[nv] = n.
template <typename T>
__global__ void k_ptr_from_sorted(const T *sorted, int64_t n, int64_t nv, int32_t *ptr)
{
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q > n) return;
    int64_t lo = (q == 0) ? 0 : (int64_t)sorted[q - 1] + 1;
    int64_t hi = (q == n) ? nv : (int64_t)sorted[q];
    for (int64_t v = lo; v <= hi; ++v) ptr[v] = (int32_t)q;
}

}  // namespace
