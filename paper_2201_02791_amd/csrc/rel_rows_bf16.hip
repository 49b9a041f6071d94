// The per-run products of a layer that applies W_r per (relation, destination) run (Eq. 1-2 regrouped:
// u_s = z_s W_r forward, dz_s = G_dst(s) W_r^T backward), bf16 in, fp32 accumulate, bf16 out, for the common
// case of a contraction width K that is a multiple of 32 up to 256 and at most 256 output columns.
//
//   out[s][:] = A[row(s)][0..K) * Wk[rel]^T        Wk[rel]: [N][K] bf16, k contiguous;  s in a range of one relation
//
// The work is HBM traffic (one K-wide row in, one N-wide row out per run; intensity about 128 flop/B at
// K = N = 256, under the bf16 ridge), so the kernel is built around keeping a steady stream of row loads and
// stores in flight, not around the matrix cores:
//
//  * a block (8 wavefronts, one per compute unit) takes a range of up to KGE_REL_RANGE runs of ONE relation and
//    keeps that relation's matrix in REGISTERS for the whole range: wavefront w holds the 32 output columns
//    [32 w, 32 w + 32) as matrix-core operands (K / 16 operands of 8 bf16 per lane, 64 registers at K = 256).
//    The matrix is read once per range (3 % of a full range's traffic) instead of once per 128-row tile;
//    measured at 25 M runs, K = N = 256: ranges of 512 runs 6.1 ms, 1024 5.6, 2048 5.35, 4096 5.3, 8192 5.4;
//  * rows go through LDS in tiles of 128, two buffers: while tile i is multiplied out of one buffer, tile i + 1
//    sits in registers (its loads were issued a whole tile earlier) and is written to the other buffer, and the
//    loads of tile i + 2 are issued - so one full tile of row loads (64 KB per compute unit) is always in flight;
//  * every wavefront multiplies all 128 rows of the tile by its 32 columns (4 accumulator tiles of 32 x 32), with
//    the operands swapped (W as the row operand) so that a lane ends up with 4 consecutive output columns of one
//    row per register quad: results are rounded to bf16 in registers, staged by 8-byte LDS writes into the buffer
//    that was just consumed, and leave as 16-byte, row-contiguous stores;
//  * two barriers per tile.
#include "common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int RT = 128;          // rows per tile
constexpr int RNT = 512;         // threads per block

__device__ __forceinline__ uint32_t pack2(float lo, float hi)   // two fp32 -> packed bf16x2, nearest even
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float floatx2_t __attribute__((ext_vector_type(2)));
    const floatx2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// NP = K / 32: 16-byte chunks per thread and tile (a tile is 128 rows of K / 8 chunks, 512 threads)
template <int NP>
__global__ __launch_bounds__(RNT) void k_rel_rows_bf16(
    const uint16_t *__restrict__ A, int64_t lda, const int32_t *__restrict__ aidx,
    const uint16_t *__restrict__ Wk, int64_t w_stride, int32_t N, uint16_t *__restrict__ out, int64_t ldo,
    const int32_t *__restrict__ r_rel, const int32_t *__restrict__ r_beg, const int32_t *__restrict__ r_end,
    int32_t n_groups, int64_t rows_total,   // without a range list: block i takes range i / n_groups of group i % n_groups
    int32_t pitch)                          // LDS row pitch in elements: max(K, N) + 8
{
    constexpr int K = 32 * NP, KS = 2 * NP;      // contraction width, matrix-core steps of 16
    constexpr int CPR = K / 8;                   // 16-byte chunks per row
    constexpr int RPP = RNT / CPR;               // rows per pass of the block
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t *buf0 = reinterpret_cast<uint16_t *>(smem);
    uint16_t *buf1 = buf0 + (size_t)RT * pitch;

    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int lrow = lane & 31, half = lane >> 5;
    int64_t m_beg, m_end;
    int32_t group;
    if (r_beg) {
        m_beg = r_beg[blockIdx.x]; m_end = r_end[blockIdx.x]; group = r_rel[blockIdx.x];
    } else {
        // every matrix over every range of rows, the groups of one range next to each other: they are dispatched
        // together (round-robin over the eight L2s), so a range's rows come from HBM once and from cache after that
        group = (int32_t)(blockIdx.x % (uint32_t)n_groups);
        m_beg = (int64_t)(blockIdx.x / (uint32_t)n_groups) * KGE_REL_RANGE;
        m_end = m_beg + KGE_REL_RANGE < rows_total ? m_beg + KGE_REL_RANGE : rows_total;
        out += (int64_t)group * N;               // group g owns columns [g N, (g + 1) N) of the output rows
    }
    if (m_beg >= m_end) return;                  // uniform over the block
    const int32_t n_tiles = (int32_t)((m_end - m_beg + RT - 1) / RT);
    const bool cols = 32 * w < N;                // this wavefront has output columns (uniform per wavefront)

    // the relation's matrix: this wavefront's 32 columns as row operands, all K
    bf16x8 wreg[KS];
    {
        const uint16_t *Wr = Wk + (int64_t)group * w_stride;
        const int32_t n = 32 * w + lrow;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (n < N) v = *reinterpret_cast<const u32x4 *>(Wr + (int64_t)n * K + ks * 16 + half * 8);
            wreg[ks] = __builtin_bit_cast(bf16x8, v);
        }
    }

    // this thread's chunks of a tile: row t / CPR + p RPP, chunk t % CPR
    const int crow = t / CPR;
    const uint32_t cbyte = (uint32_t)(t % CPR) * 16u;
    int32_t ai[NP];
    u32x4 R[NP];
    auto tile_rows = [&](int32_t ti) __attribute__((always_inline)) {
        const int64_t m0 = m_beg + (int64_t)ti * RT;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int64_t r = m0 + crow + p * RPP, rc = r < m_end ? r : m_end - 1;   // past the range: its last row again
            ai[p] = aidx ? aidx[rc] : (int32_t)rc;
        }
    };
    auto tile_load = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const char *ap = reinterpret_cast<const char *>(A) + (int64_t)ai[p] * lda * 2;
            R[p] = *reinterpret_cast<const u32x4 *>(ap + cbyte);
        }
    };
    auto tile_to_lds = [&](uint16_t *buf) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < NP; ++p)
            *reinterpret_cast<u32x4 *>(reinterpret_cast<char *>(buf) + (size_t)(crow + p * RPP) * pitch * 2 + cbyte) = R[p];
    };

    tile_rows(0);
    tile_load();
    if (n_tiles > 1) tile_rows(1);
    tile_to_lds(buf0);                           // waits for tile 0
    if (n_tiles > 1) tile_load();                // tile 1 in flight
    if (n_tiles > 2) tile_rows(2);
    __syncthreads();

    const int NC8 = N / 8;                       // 16-byte chunks per output row
    const int srow = t / NC8, c8 = t - srow * NC8; // this thread's first staged row and its chunk of every row
    for (int32_t ti = 0; ti < n_tiles; ++ti) {
        uint16_t *cur = (ti & 1) ? buf1 : buf0, *nxt = (ti & 1) ? buf0 : buf1;
        floatx16 acc[4];
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[rb][v] = 0.f;
        if (cols) {
            const uint16_t *ab = cur + (size_t)lrow * pitch + half * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8 af[4];
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
                    af[rb] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(ab + (size_t)rb * 32 * pitch + ks * 16));
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
                    acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[ks], af[rb], acc[rb], 0, 0, 0);
            }
        }
        __syncthreads();                         // tile ti consumed; the other buffer's staged rows have left
        if (ti + 1 < n_tiles) {
            tile_to_lds(nxt);                    // waits for tile ti + 1 (issued a tile ago)
            if (ti + 2 < n_tiles) {
                tile_load();                     // tile ti + 2 in flight
                if (ti + 3 < n_tiles) tile_rows(ti + 3);
            }
        }
        // register v of lane l: row l % 32 of the row block, column 8 (v / 4) + 4 (l / 32) + v % 4 of the 32
        if (cols) {
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<uint2 *>(cur + (size_t)(rb * 32 + lrow) * pitch + 32 * w + 8 * q + 4 * half) =
                        make_uint2(pack2(acc[rb][4 * q], acc[rb][4 * q + 1]), pack2(acc[rb][4 * q + 2], acc[rb][4 * q + 3]));
        }
        __syncthreads();                         // staged rows and the next tile are in LDS
        const int64_t m0 = m_beg + (int64_t)ti * RT;
        for (int row = srow; row < RT; row += RNT / NC8) {      // NC8 divides the block size: 4, 8, .. 32
            if (m0 + row < m_end) {
                const u32x4 v = *reinterpret_cast<const u32x4 *>(cur + (size_t)row * pitch + c8 * 8);
                *reinterpret_cast<u32x4 *>(out + (m0 + row) * ldo + c8 * 8) = v;
            }
        }
    }
}

template <int NP>
int launch_np(const kge_partition *p, int32_t n_groups, int64_t rows_total, const void *A, int64_t lda,
              const int32_t *aidx, const void *Wk, int32_t N, void *out, int64_t ldo, hipStream_t st)
{
    const int32_t K = 32 * NP;
    const int32_t pitch = (K > N ? K : N) + 8;
    const size_t lds = (size_t)2 * RT * pitch * 2;
    static bool attr_set = false;
    if (!attr_set) {      // the largest this instantiation can ask for (N = 256)
        KGE_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_rel_rows_bf16<NP>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)((size_t)2 * RT * (256 + 8) * 2)));
        attr_set = true;
    }
    const int64_t blocks = p ? p->n_relr : n_groups * cdiv(rows_total, KGE_REL_RANGE);
    KGE_REQUIRE(blocks < (1ll << 31), KGE_ERANGE, "per-run product: too many blocks");
    k_rel_rows_bf16<NP><<<(unsigned)blocks, RNT, lds, st>>>(
        reinterpret_cast<const uint16_t *>(A), lda, aidx, reinterpret_cast<const uint16_t *>(Wk), (int64_t)N * K, N,
        reinterpret_cast<uint16_t *>(out), ldo, p ? p->relr_rel : nullptr, p ? p->relr_beg : nullptr,
        p ? p->relr_end : nullptr, n_groups, rows_total, pitch);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

}  // namespace

bool rel_rows_bf16_supported(int32_t K, int32_t N)
{
    return (K == 64 || K == 128 || K == 256) && N >= 32 && N <= 256 && N % 32 == 0;
}

// out[s] = A[aidx ? aidx[s] : s] * Wk[rel(s)]^T for every run s;  A rows `lda` elements apart (16-byte aligned),
// Wk: bf16 [2R][N][K], out: bf16 [S][N].  Shapes outside rel_rows_bf16_supported are the caller's to route elsewhere.
int launch_rel_rows_bf16(const kge_partition *p, const void *A, int64_t lda, const int32_t *aidx, const void *Wk,
                         int32_t K, int32_t N, void *out, hipStream_t st)
{
    KGE_REQUIRE(rel_rows_bf16_supported(K, N), KGE_EINVAL, "per-run product: shape not supported by this kernel");
    KGE_REQUIRE(lda % 8 == 0 && ((uintptr_t)A % 16) == 0 && ((uintptr_t)Wk % 16) == 0 && ((uintptr_t)out % 16) == 0,
                KGE_EINVAL, "per-run product: operands must be 16-byte aligned");
    if (p->n_relr == 0) return KGE_OK;
    switch (K) {
    case 64: return launch_np<2>(p, 0, 0, A, lda, aidx, Wk, N, out, N, st);
    case 128: return launch_np<4>(p, 0, 0, A, lda, aidx, Wk, N, out, N, st);
    default: return launch_np<8>(p, 0, 0, A, lda, aidx, Wk, N, out, N, st);
    }
}

// out[i][g N .. (g + 1) N) = A[i] * Wk[g]^T for every row i < rows and every matrix g < n_groups (the basis
// projections of Eq. 2: A = the layer input, Wk[g] = V_g^T):  A: bf16 [rows][K], Wk: bf16 [n_groups][N][K],
// out: bf16 [rows][n_groups N].
int launch_all_rows_bf16(const void *A, int64_t rows, const void *Wk, int32_t n_groups, int32_t K, int32_t N,
                         void *out, hipStream_t st)
{
    KGE_REQUIRE(rel_rows_bf16_supported(K, N), KGE_EINVAL, "projection: shape not supported by this kernel");
    KGE_REQUIRE(((uintptr_t)A % 16) == 0 && ((uintptr_t)Wk % 16) == 0 && ((uintptr_t)out % 16) == 0, KGE_EINVAL,
                "projection: operands must be 16-byte aligned");
    KGE_REQUIRE(rows < (1ll << 31), KGE_ERANGE, "projection: too many rows");
    if (rows == 0 || n_groups == 0) return KGE_OK;
    const int64_t ldo = (int64_t)n_groups * N;
    switch (K) {
    case 64: return launch_np<2>(nullptr, n_groups, rows, A, K, nullptr, Wk, N, out, ldo, st);
    case 128: return launch_np<4>(nullptr, n_groups, rows, A, K, nullptr, Wk, N, out, ldo, st);
    default: return launch_np<8>(nullptr, n_groups, rows, A, K, nullptr, Wk, N, out, ldo, st);
    }
}
