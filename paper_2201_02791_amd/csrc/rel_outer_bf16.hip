// The relation matrices' gradient of a layer that applies W_r per (relation, destination) run (Eq. 1-2
// regrouped): C_r = sum over the runs s of relation r of x_s^T g_s, with x_s the run's mean input row and g_s the
// output gradient row of its destination; bf16 rows in, fp32 accumulate, fp32 out, for layer widths of 128 or 256.
//
//   C[rel] (DI x DO) += sum_{s in [beg, end)} X[xidx[s]][0..DI)^T  G[gidx[s]][0..DO)
//
// The kernel only reads: a stream of run means and gathered rows of G (1 KB per run at 256 x 256, intensity 128
// flop/B, under the bf16 ridge).  Row gathers of this size run at 6.5 to 7 TB/s on this chip when nothing else
// is in their way, so the kernel is built to keep them in flight without spending registers or issue slots of the
// wavefronts that multiply:
//
//  * a block (12 wavefronts, one block per compute unit) takes one chunk of one relation's runs and holds the whole
//    DI x DO result in the accumulators of its eight MULTIPLYING wavefronts (4 x 2 of them, 64 x 128 each at
//    256 x 256: 128 accumulator registers per lane), so every row is read once and the chunk ends in one atomic
//    accumulation into C[rel];
//  * rows reach LDS in tiles of 32 runs without passing through registers: the four MOVING wavefronts issue
//    global -> LDS loads (16 bytes per lane, a wavefront instruction fills 1 KB of consecutive LDS: two rows of 256
//    elements) with the row indices read through the scalar cache, so a tile in flight costs them nothing but the
//    instruction.  Four tile buffers: one being multiplied, up to three on their way (96 KB per compute unit);
//  * the contraction runs over the rows, so both matrix-core operands are read from LDS with the transposing read
//    (ds_read_b64_tr_b16).  A global -> LDS load cannot pad rows, and rows 256 or 512 bytes apart would put the
//    four rows of one transposing read in the same banks; instead the 16-byte chunks of row i are stored XOR-ed
//    with 4 (i mod 4) - the lane that fills LDS slot c of row i fetches chunk c ^ 4 (i mod 4) - and the readers
//    apply the same XOR, which makes the reads conflict-free;
//  * one barrier per tile.  A moving wavefront waits with s_waitcnt vmcnt(n) until the tile that is read next has
//    landed (its loads retire in order, n = the loads of the younger tiles), the barrier publishes it; rows past
//    the end of the chunk are fetched from its last row and overwritten with zeros in LDS before that barrier.
#include "common.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int RT = 32;           // runs per tile
constexpr int NB = 4;            // tile buffers
constexpr int CW = 8;            // multiplying wavefronts, 4 (rows of C) x 2 (columns of C)
constexpr int MW = 4;            // moving wavefronts, 8 rows of a tile each
constexpr int ONT = 64 * (CW + MW);

// s_waitcnt with only the vector-memory counter set (gfx9 encoding: vmcnt in bits 3:0 and 15:14, the other
// counters at their maxima = no wait)
#define KGE_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0f70)

__device__ __forceinline__ void block_barrier()
{
    // the plain barrier instruction: the waits that make a tile visible are placed by hand (the vector-memory
    // counter for the global -> LDS loads, the LDS counter for the zero fill), and a fence would drain the
    // moving wavefronts' younger tiles as well.  Every wavefront's own LDS accesses are complete before it arrives.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xc07f);          // lgkmcnt(0): this wavefront's LDS reads and writes are done
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <int DI, int DO>
__global__ __launch_bounds__(ONT) void k_rel_outer_bf16(
    const uint16_t *__restrict__ X, int64_t ldx, const int32_t *__restrict__ xidx,
    const uint16_t *__restrict__ G, int64_t ldg, const int32_t *__restrict__ gidx,
    const int32_t *__restrict__ c_rel, const int32_t *__restrict__ c_beg, const int32_t *__restrict__ c_end,
    float *__restrict__ C, int32_t n_groups, int32_t rows_total, int32_t chunk_rows, float *__restrict__ C_last)
{
    constexpr int BX = 2 * DI, BG = 2 * DO;              // bytes of a row of X, of G
    constexpr int LX = BX / 16, LG = BG / 16;            // lanes (16-byte chunks) per row
    constexpr int RX = 64 / LX, RG = 64 / LG;            // rows per global -> LDS instruction
    constexpr int TB = RT * (BX + BG);                   // bytes of a tile buffer: the X rows, then the G rows
    constexpr int NI = 8 / RX + 8 / RG;                  // global -> LDS instructions per moving wavefront and tile
    constexpr int MI = DI / 128, NJ = DO / 64;           // 32 x 32 blocks per multiplying wavefront: MI x NJ
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);
    int32_t m_beg, m_end, rel;
    if (c_beg) {
        m_beg = c_beg[blockIdx.x]; m_end = c_end[blockIdx.x]; rel = c_rel[blockIdx.x];
    } else {
        // without a chunk list: every group (a block of DO columns of G's rows) over every chunk of all rows, the
        // groups of one chunk next to each other in the grid, so that the chunk's rows of X come from HBM once
        rel = (int32_t)(blockIdx.x % (uint32_t)n_groups);
        m_beg = (int32_t)(blockIdx.x / (uint32_t)n_groups) * chunk_rows;
        m_end = m_beg + chunk_rows < rows_total ? m_beg + chunk_rows : rows_total;
        G += (int64_t)rel * DO;
    }
    if (m_beg >= m_end) return;                          // uniform over the block
    const int32_t n_tiles = (m_end - m_beg + RT - 1) / RT;

    if (w >= CW) {
        // ------------------------------------------------------------------ the moving wavefronts
        const int mw = w - CW;                           // rows [8 mw, 8 mw + 8) of every tile
        const int lrx = lane / LX, cx = lane % LX, lrg = lane / LG, cg = lane % LG;
        auto issue = [&](int32_t ti) __attribute__((always_inline)) {
            const int32_t r0 = m_beg + ti * RT + 8 * mw, last = m_end - 1;
            int32_t xi[8], gi[8];                        // uniform: scalar loads
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int32_t r = r0 + q < last ? r0 + q : last;       // past the chunk: its last run again
                xi[q] = xidx ? xidx[r] : r;
                gi[q] = gidx ? gidx[r] : r;
            }
            unsigned char *bx = smem + (ti & (NB - 1)) * TB + 8 * mw * BX;
            unsigned char *bg = smem + (ti & (NB - 1)) * TB + RT * BX + 8 * mw * BG;
#pragma unroll
            for (int q = 0; q < 8; q += RX) {
                int32_t idx = xi[q];
#pragma unroll
                for (int k = 1; k < RX; ++k) idx = lrx == k ? xi[q + k] : idx;
                const int sw = ((q + lrx) & 3) << 2;     // row (8 mw + q + lrx) mod 4, in chunks of 16 bytes
                const char *src = reinterpret_cast<const char *>(X) + (int64_t)idx * ldx * 2 + ((cx ^ sw) << 4);
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                                 (__attribute__((address_space(3))) void *)(bx + q * BX), 16, 0, 0);
            }
#pragma unroll
            for (int q = 0; q < 8; q += RG) {
                int32_t idx = gi[q];
#pragma unroll
                for (int k = 1; k < RG; ++k) idx = lrg == k ? gi[q + k] : idx;
                const int sw = ((q + lrg) & 3) << 2;
                const char *src = reinterpret_cast<const char *>(G) + (int64_t)idx * ldg * 2 + ((cg ^ sw) << 4);
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                                 (__attribute__((address_space(3))) void *)(bg + q * BG), 16, 0, 0);
            }
        };
        // tile ti has landed once at most `younger` tiles issued after it are outstanding; then its rows past the
        // end of the chunk (the last tile only) become zeros
        auto land = [&](int32_t ti, int32_t younger) __attribute__((always_inline)) {
            if (younger >= 2) KGE_WAIT_VM(2 * NI);
            else if (younger == 1) KGE_WAIT_VM(NI);
            else KGE_WAIT_VM(0);
            const int32_t valid = m_end - m_beg - ti * RT;            // rows of the tile inside the chunk
            if (valid < RT) {
                unsigned char *bx = smem + (ti & (NB - 1)) * TB, *bg = bx + RT * BX;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int row = 8 * mw + q;
                    if (row >= valid) {
                        if (lane < LX) *reinterpret_cast<u32x4 *>(bx + row * BX + lane * 16) = u32x4{0u, 0u, 0u, 0u};
                        if (lane < LG) *reinterpret_cast<u32x4 *>(bg + row * BG + lane * 16) = u32x4{0u, 0u, 0u, 0u};
                    }
                }
            }
        };
        // before step 0: tiles 0 .. 2 issued, tile 0 landed
        const int32_t pro = n_tiles < NB - 1 ? n_tiles : NB - 1;
        for (int32_t ti = 0; ti < pro; ++ti) issue(ti);
        land(0, pro - 1);
        block_barrier();
        for (int32_t s = 0; s < n_tiles; ++s) {
            // buffer (s + 3) mod 4 held tile s - 1: read in step s - 1, a barrier ago
            if (s + NB - 1 < n_tiles) issue(s + NB - 1);
            if (s + 1 < n_tiles) {
                const int32_t issued = s + NB < n_tiles ? s + NB : n_tiles;
                land(s + 1, issued - (s + 2));
            }
            block_barrier();
        }
        return;
    }
    // ---------------------------------------------------------------------- the multiplying wavefronts
    const int wm = w >> 1, wn = w & 1;
    floatx16 acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    // transposing read: as an addressing lane of its group of 16, a lane points at row (lane % 16) / 4 of the four
    // rows of the group and at 4 of its 16 columns; lanes 32 .. 63 take the second half of the 16 rows of a step
    const int l16 = lane & 15, kr0 = 8 * (lane >> 5) + (l16 >> 2);
    const int cb = (16 * ((lane >> 4) & 1) + 4 * (l16 & 3)) * 2;     // byte offset of the lane's columns in a 32-column block
    const int sw = ((l16 >> 2) & 3) << 6;                             // the row's XOR, in bytes (rows kr0, kr0 + 4, + 16 ...)
    auto frag = [&](const unsigned char *tile, int rowbytes, int kr, int colbyte) __attribute__((always_inline)) {
        const unsigned char *p = tile + kr * rowbytes + ((colbyte ^ sw) + cb);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)p);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(p + 4 * rowbytes));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    block_barrier();
    for (int32_t s = 0; s < n_tiles; ++s) {
        const unsigned char *bx = smem + (s & (NB - 1)) * TB, *bg = bx + RT * BX;
#pragma unroll
        for (int ks = 0; ks < RT; ks += 16) {
            bf16x8 af[MI], bf[NJ];
#pragma unroll
            for (int i = 0; i < MI; ++i) af[i] = frag(bx, BX, ks + kr0, (wm * MI + i) * 64);
#pragma unroll
            for (int j = 0; j < NJ; ++j) bf[j] = frag(bg, BG, ks + kr0, (wn * NJ + j) * 64);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        block_barrier();
    }
    // register v of lane l: row 8 (v / 4) + 4 (l / 32) + v % 4 and column l % 32 of the 32 x 32 block
    float *Cr = (C_last && rel == n_groups - 1) ? C_last : C + (int64_t)rel * DI * DO;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = (wm * MI + i) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int n = (wn * NJ + j) * 32 + (lane & 31);
                unsafeAtomicAdd(Cr + (int64_t)m * DO + n, acc[i][j][v]);
            }
}

struct OuterArgs {
    const void *X; int64_t ldx; const int32_t *xidx; const void *G; int64_t ldg; const int32_t *gidx;
    const int32_t *c_rel, *c_beg, *c_end; int64_t blocks; float *C;
    int32_t n_groups, rows_total, chunk_rows; float *C_last;
};

template <int DI, int DO>
int launch_shape(const OuterArgs &a, hipStream_t st)
{
    constexpr size_t lds = (size_t)NB * RT * 2 * (DI + DO);
    static bool attr_set = false;
    if (!attr_set) {
        KGE_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_rel_outer_bf16<DI, DO>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set = true;
    }
    KGE_REQUIRE(a.blocks < (1ll << 31), KGE_ERANGE, "outer-product sums: too many blocks");
    k_rel_outer_bf16<DI, DO><<<(unsigned)a.blocks, ONT, lds, st>>>(
        reinterpret_cast<const uint16_t *>(a.X), a.ldx, a.xidx, reinterpret_cast<const uint16_t *>(a.G), a.ldg, a.gidx,
        a.c_rel, a.c_beg, a.c_end, a.C, a.n_groups, a.rows_total, a.chunk_rows, a.C_last);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

int launch_any(const OuterArgs &a, int32_t d_in, int32_t d_out, hipStream_t st)
{
    KGE_REQUIRE(rel_outer_bf16_supported(d_in, d_out), KGE_EINVAL, "outer-product sums: shape not supported by this kernel");
    KGE_REQUIRE(a.ldx % 8 == 0 && a.ldg % 8 == 0 && a.ldx >= d_in && a.ldg >= d_out && ((uintptr_t)a.X % 16) == 0 &&
                    ((uintptr_t)a.G % 16) == 0,
                KGE_EINVAL, "outer-product sums: rows must be 16-byte aligned");
    if (d_in == 256) {
        if (d_out == 256) return launch_shape<256, 256>(a, st);
        return launch_shape<256, 128>(a, st);
    }
    if (d_out == 256) return launch_shape<128, 256>(a, st);
    return launch_shape<128, 128>(a, st);
}

}  // namespace

bool rel_outer_bf16_supported(int32_t d_in, int32_t d_out)
{
    return (d_in == 128 || d_in == 256) && (d_out == 128 || d_out == 256);
}

// C[r] (d_in x d_out fp32, zeroed by the caller) += sum over the runs s of relation r of X[xidx ? xidx[s] : s]^T
// G[seg_dst[s]];  X rows `ldx` and G rows `ldg` elements apart, both 16-byte aligned.
int launch_rel_outer_rows_bf16(const kge_partition *p, const void *X, int64_t ldx, const int32_t *xidx, const void *G,
                               int64_t ldg, int32_t d_in, int32_t d_out, float *C, hipStream_t st)
{
    if (p->n_relc == 0) return KGE_OK;
    const OuterArgs a{X, ldx, xidx, G, ldg, p->seg_dst, p->relc_rel, p->relc_beg, p->relc_end, p->n_relc, C, 0, 0, 0, nullptr};
    return launch_any(a, d_in, d_out, st);
}

// C[g] (d_in x d_out fp32, zeroed by the caller) += X^T Y_g for every column block g < n_groups of Y's rows
// (Y: bf16 [rows][ldy], block g = columns [g d_out, (g + 1) d_out)); the last block's sum goes to C_last when that is
// non-null (the weight gradients of Eq. 2: X = the layer input, Y = [dP | G], C = dV, C_last = dW_0).
int launch_col_blocks_outer_bf16(const void *X, int64_t rows, const void *Y, int64_t ldy, int32_t n_groups,
                                 int32_t d_in, int32_t d_out, float *C, float *C_last, hipStream_t st)
{
    if (rows == 0 || n_groups == 0) return KGE_OK;
    KGE_REQUIRE(rows < (1ll << 31) - 65536 && ldy >= (int64_t)n_groups * d_out, KGE_ERANGE, "outer-product sums: bad row count or pitch");
    // every chunk ends in one atomic accumulation of a whole d_in x d_out tile: long chunks, as long as about two
    // blocks per compute unit are left
    int32_t chunk = 8192;
    while (chunk > 2048 && cdiv(rows, chunk) * n_groups < 512) chunk /= 2;
    const OuterArgs a{X, d_in, nullptr, Y, ldy, nullptr, nullptr, nullptr, nullptr, cdiv(rows, chunk) * n_groups, C,
                      n_groups, (int32_t)rows, chunk, C_last};
    return launch_any(a, d_in, d_out, st);
}
