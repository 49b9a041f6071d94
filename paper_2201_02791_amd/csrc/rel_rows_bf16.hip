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
//  * a block (16 wavefronts, one block per compute unit) takes a range of up to KGE_REL_RANGE runs of ONE relation.
//    Its wavefronts have two roles.  Eight MULTIPLY: wavefront w keeps the relation's 32 output columns
//    [32 w, 32 w + 32) in REGISTERS for the whole range as matrix-core operands (K / 16 operands of 8 bf16 per
//    lane, 64 registers at K = 256), so the matrix is read once per range (3 % of a full range's traffic) instead
//    of once per row tile.  Eight MOVE rows: global memory -> LDS and LDS -> global memory;
//  * rows go through LDS in tiles of 64: two row buffers and two buffers of staged results.  In step s (one
//    barrier per step) the multiplying wavefronts form tile s out of one row buffer - operands swapped, W as the
//    row operand, so that a lane ends up with 4 consecutive output columns of a row per register quad - round it
//    to bf16 in registers and stage it by 8-byte LDS writes, while the moving wavefronts write tile s + 1 into
//    the other row buffer, issue the loads of tile s + 5 and store the staged tile s - 1 as 16-byte, row-contiguous
//    stores.  Loading, multiplying and storing overlap instead of taking turns (taking turns, with all
//    wavefronts doing everything, was 5.35 ms per launch at 25 M runs; this form 5.03 ms, the speed of a plain
//    device copy of the same bytes);
//  * the moving wavefronts are four groups of two; group g owns the tiles j = g (mod 4) and keeps exactly one of
//    them in flight in its registers.  A wavefront's outstanding memory operations retire in order and the
//    compiler waits for all of them before the first use of any (measured: a ring of three tiles per wavefront
//    drained to zero at every step), so tiles in flight are spread over wavefronts, not over a wavefront's
//    registers: four tiles, 128 KB per compute unit, always on their way;
//  * LDS buffers are addressed as offsets from one base: a table of LDS pointers loses the address space, every
//    access becomes a flat one, and a flat access waits on the memory counter as well;
//  * what bounds it when the rows come from cache (the basis projections): the multiplying wavefronts read every
//    row tile eight times (4 KB of LDS reads per row) and the LDS delivers 64 bytes per clock per compute unit
//    (measured with a read-only loop of the same access pattern: 1.78 us per 64-row tile, twice the matrix
//    cores' 0.9 us).  Two column blocks per wavefront would halve that but need 128 operand registers, i.e. one
//    multiplying wavefront per SIMD: measured slower (5.9 against 5.0 ms); storing results from registers in
//    8-byte pieces instead of staging them: 6.5 ms.
#include "common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int RT = 64;           // rows per tile
constexpr int CW = 8;            // wavefronts that multiply (each owns 32 output columns)
constexpr int MW = 8;            // wavefronts that move rows: global -> LDS and LDS -> global
constexpr int RNT = 64 * (CW + MW);   // threads per block
constexpr int MT = 64 * MW;      // threads of the moving wavefronts
constexpr int MG = 4;            // groups of moving wavefronts = row tiles in flight
constexpr int GT = MT / MG;      // threads of a group

__device__ __forceinline__ uint32_t pack2(float lo, float hi)   // two fp32 -> packed bf16x2, nearest even
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float floatx2_t __attribute__((ext_vector_type(2)));
    const floatx2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// NP = K / 32 (a tile is 64 rows of K / 8 = 4 NP chunks of 16 bytes, moved by 512 threads: NP / 2 chunks each)
template <int NP>
__global__ __launch_bounds__(RNT) void k_rel_rows_bf16(
    const uint16_t *__restrict__ A, int64_t lda, const int32_t *__restrict__ aidx,
    const uint16_t *__restrict__ Wk, int64_t w_stride, int32_t N, uint16_t *__restrict__ out, int64_t ldo,
    const int32_t *__restrict__ r_rel, const int32_t *__restrict__ r_beg, const int32_t *__restrict__ r_end,
    int32_t n_groups, int64_t rows_total)   // without a range list: block i takes range i / n_groups of group i % n_groups
{
    constexpr int K = 32 * NP, KS = 2 * NP;      // contraction width, matrix-core steps of 16
    constexpr int CPR = K / 8;                   // 16-byte chunks per row
    constexpr int RPP = GT / CPR;                // rows per pass of a group of moving wavefronts
    constexpr int NPG = RT * CPR / GT;           // 16-byte chunks per moving thread and tile
    constexpr int PA = K + 8;                    // LDS row pitch of a row tile, elements
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int PS = N + 8;                        // LDS row pitch of a staged result tile
    // two row-tile buffers, then two staged-result buffers; addressed as offsets from the one LDS base (a table of
    // pointers would lose the address space and turn every access into a flat one, which waits on both counters)
    uint16_t *lds = reinterpret_cast<uint16_t *>(smem);
    auto abuf = [&](int i) __attribute__((always_inline)) { return lds + (i & 1) * (RT * PA); };
    auto sbuf = [&](int i) __attribute__((always_inline)) { return lds + 2 * RT * PA + (i & 1) * (RT * PS); };

    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
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

    // Step s = 0 .. n_tiles, one barrier each:
    //   multiplying wavefronts: tile s out of abuf(s), results (bf16) into sbuf(s)
    //   moving wavefronts:      tile s + 1 (in a group's registers since step s - 3) into abuf(s + 1), the loads of
    //                           tile s + 5 issued, the staged results of tile s - 1 from sbuf(s - 1) to memory
    // abuf(s + 1) was last read in step s - 1 and sbuf(s) in step s - 1 (tile s - 2): a barrier lies between.
    if (w >= CW) {
        // ------------------------------------------------------------------ the moving wavefronts
        // MG groups of two wavefronts; group g owns the tiles j = g (mod MG): it keeps exactly one of them in
        // flight in its registers, so "wait for my tile" is a plain wait for all of the wavefront's own loads
        // (the counter of outstanding memory operations is per wavefront and retires in order), and the block
        // always has MG tiles on their way.  The staged results of a tile are stored by the group two ahead.
        const int mt = t - 64 * CW, g = mt / GT, gt = mt % GT;
        const int crow = gt / CPR;
        const uint32_t cbyte = (uint32_t)(gt % CPR) * 16u;
        int32_t ai[NPG];
        u32x4 R[NPG];
        auto tile_rows = [&](int32_t ti) __attribute__((always_inline)) {
            const int32_t m0 = (int32_t)m_beg + ti * RT + crow, last = (int32_t)m_end - 1;   // rows are < 2^31
#pragma unroll
            for (int p = 0; p < NPG; ++p) {
                const int32_t r = m0 + p * RPP, rc = r < last ? r : last;          // past the range: its last row again
                ai[p] = aidx ? aidx[rc] : rc;
            }
        };
        auto tile_load = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int p = 0; p < NPG; ++p) {
                const char *ap = reinterpret_cast<const char *>(A) + (int64_t)ai[p] * lda * 2;
                R[p] = *reinterpret_cast<const u32x4 *>(ap + cbyte);
            }
        };
        auto tile_to_lds = [&](uint16_t *buf) __attribute__((always_inline)) {
#pragma unroll
            for (int p = 0; p < NPG; ++p)
                *reinterpret_cast<u32x4 *>(reinterpret_cast<char *>(buf) + (size_t)(crow + p * RPP) * PA * 2 + cbyte) = R[p];
        };
        const int NC8 = N / 8;                   // 16-byte chunks per output row (4, 8, .. 32: divides GT)
        const int srow = gt / NC8, c8 = gt - srow * NC8;

        // before step 0: tile 0 in LDS; tiles 1 .. MG in flight, tile j in group j % MG; each group knows the rows
        // of the tile it loads next
        if (g < n_tiles) { tile_rows(g); tile_load(); }
        if (g == 0) {
            if (MG < n_tiles) tile_rows(MG);
            tile_to_lds(abuf(0));                // waits for tile 0
            if (MG < n_tiles) { tile_load(); if (2 * MG < n_tiles) tile_rows(2 * MG); }
        } else if (g + MG < n_tiles) {
            tile_rows(g + MG);
        }
        __syncthreads();
        for (int32_t s = 0; s <= n_tiles; ++s) {
            if ((s + 1) % MG == g && s + 1 < n_tiles) {
                tile_to_lds(abuf(s + 1));        // waits for tile s + 1 (issued MG steps ago) and for the rows of tile s + 1 + MG
                if (s + 1 + MG < n_tiles) {
                    tile_load();                 // tile s + 1 + MG in flight
                    if (s + 1 + 2 * MG < n_tiles) tile_rows(s + 1 + 2 * MG);
                }
            }
            if ((s + MG - 1) % MG == g && s >= 1) {
                const uint16_t *sb = sbuf(s - 1);
                const int64_t m0 = m_beg + (int64_t)(s - 1) * RT;
                for (int row = srow; row < RT; row += GT / NC8) {
                    if (m0 + row < m_end) {
                        const u32x4 v = *reinterpret_cast<const u32x4 *>(sb + (size_t)row * PS + c8 * 8);
                        __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(out + (m0 + row) * ldo + c8 * 8));
                    }
                }
            }
            __syncthreads();
        }
        return;
    }
    // ---------------------------------------------------------------------- the multiplying wavefronts
    const int lrow = lane & 31, half = lane >> 5;
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
    __syncthreads();
    for (int32_t s = 0; s <= n_tiles; ++s) {
        if (s < n_tiles && cols) {
            floatx16 acc[2];
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[rb][v] = 0.f;
            const uint16_t *ab = abuf(s) + lrow * PA + half * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8 af[2];
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
                    af[rb] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(ab + rb * 32 * PA + ks * 16));
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
                    acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[ks], af[rb], acc[rb], 0, 0, 0);
            }
            // register v of lane l: row l % 32 of the row block, column 8 (v / 4) + 4 (l / 32) + v % 4 of the 32
            uint16_t *sb = sbuf(s);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<uint2 *>(sb + (size_t)(rb * 32 + lrow) * PS + 32 * w + 8 * q + 4 * half) =
                        make_uint2(pack2(acc[rb][4 * q], acc[rb][4 * q + 1]), pack2(acc[rb][4 * q + 2], acc[rb][4 * q + 3]));
        }
        __syncthreads();
    }
}

struct RangeList { int32_t n; const int32_t *rel, *beg, *end; };

template <int NP>
int launch_np(const RangeList *p, int32_t n_groups, int64_t rows_total, const void *A, int64_t lda,
              const int32_t *aidx, const void *Wk, int32_t N, void *out, int64_t ldo, hipStream_t st)
{
    const int32_t K = 32 * NP;
    const size_t lds = (size_t)2 * RT * (K + 8 + N + 8) * 2;
    static bool attr_set = false;
    if (!attr_set) {      // the largest this instantiation can ask for (N = 256)
        KGE_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_rel_rows_bf16<NP>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)((size_t)2 * RT * (K + 8 + 256 + 8) * 2)));
        attr_set = true;
    }
    const int64_t blocks = p ? p->n : n_groups * cdiv(rows_total, KGE_REL_RANGE);
    KGE_REQUIRE(blocks < (1ll << 31), KGE_ERANGE, "per-run product: too many blocks");
    k_rel_rows_bf16<NP><<<(unsigned)blocks, RNT, lds, st>>>(
        reinterpret_cast<const uint16_t *>(A), lda, aidx, reinterpret_cast<const uint16_t *>(Wk), (int64_t)N * K, N,
        reinterpret_cast<uint16_t *>(out), ldo, p ? p->rel : nullptr, p ? p->beg : nullptr,
        p ? p->end : nullptr, n_groups, rows_total);
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
// by_dst_slab: walk the ranges in the order of the destination slabs (for rows gathered by destination)
int launch_rel_rows_bf16(const kge_partition *p, const void *A, int64_t lda, const int32_t *aidx, const void *Wk,
                         int32_t K, int32_t N, void *out, hipStream_t st, bool by_dst_slab)
{
    KGE_REQUIRE(rel_rows_bf16_supported(K, N), KGE_EINVAL, "per-run product: shape not supported by this kernel");
    KGE_REQUIRE(lda % 8 == 0 && ((uintptr_t)A % 16) == 0 && ((uintptr_t)Wk % 16) == 0 && ((uintptr_t)out % 16) == 0,
                KGE_EINVAL, "per-run product: operands must be 16-byte aligned");
    if (p->n_relr == 0) return KGE_OK;
    const RangeList plain{p->n_relr, p->relr_rel, p->relr_beg, p->relr_end};
    const RangeList slabs{p->n_rels, p->rels_rel, p->rels_beg, p->rels_end};
    const RangeList *rl = by_dst_slab ? &slabs : &plain;
    switch (K) {
    case 64: return launch_np<2>(rl, 0, 0, A, lda, aidx, Wk, N, out, N, st);
    case 128: return launch_np<4>(rl, 0, 0, A, lda, aidx, Wk, N, out, N, st);
    default: return launch_np<8>(rl, 0, 0, A, lda, aidx, Wk, N, out, N, st);
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
