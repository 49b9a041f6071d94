// The three dense contractions of the encoder (see gemm.hip) for workloads that keep messages
// in bf16, on v_mfma_f32_32x32x16_bf16 (fp32 accumulation).
//
// Every operand is a plain row-major bf16 matrix by the time it reaches a GEMM: small
// conversion kernels write a bf16 copy of the layer input, of [V_1..V_B | W_0] (row-major and
// transposed), and append the upstream gradient G to the dP buffer, so that X = [dP | G] is one
// matrix.  The GEMM loaders are then bare 16-byte loads.
//
//   project      [P | Self] = Hbf  (N x K)  *  WbfT^T   both operands k-contiguous
//   input_grad   dH         = X    (N x nc) *  Wbf^T    both operands k-contiguous
//   weight_grad  d[V | W0]  = Hbf^T * X                 both operands k-strided (k = vertex); formed as (X^T Hbf)^T
//
// and for layers that apply W_r per (relation, destination) run:
//
//   rel_outer    C_r = sum_{runs s of r} Zbf[s]^T Gbf[dst(s)]   k-strided (k = run), grouped by relation,
//                                                        B rows picked through the run -> destination list
//
// Block tile 128 x 256 x 32 (or x 64), 4 wavefronts in a 2 x 2 grid, each owning 64 x 128 = 2 x 4 MFMA
// tiles (128 accumulator registers, two blocks per CU).  k-contiguous operands: LDS holds A as [m][k] and B
// as [n][k], k contiguous, rows padded to 80 (176) bytes so the 16-byte operand reads of a half-wavefront
// touch every bank once; a lane feeds the matrix core 8 consecutive k values of one row.  k-strided operands
// stay k-major in LDS ([k][m], [k][n], as they lie in memory) and the operands are fetched with the
// transposing LDS read of gfx950.  The next tile's global loads are issued before the MFMA loop of the
// current tile.  bf16 outputs go through LDS so that they are written as 16-byte vectors, row-contiguous.
#include "common.h"
#include <type_traits>

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int TM = 128, TN = 256, TK = 32, NT = 256;

__device__ __forceinline__ uint32_t pack2(float lo, float hi)   // two fp32 -> packed bf16x2, nearest even
{
    // one v_cvt_pk_bf16_f32 on gfx950
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float floatx2_t __attribute__((ext_vector_type(2)));
    const floatx2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Row-major bf16 matrix, rows `ld` elements apart.  `idx` (optional): logical row r is stored row idx[r].
struct MatBF {
    const uint16_t *p; int64_t rows; int32_t cols; int64_t ld; const int32_t *idx;
};

struct EpiProjectStaged {     // columns < bd -> P (bf16), the rest -> Self (fp32); through LDS
    static constexpr bool staged = true, packed = false, swapped = false;
    uint16_t *P; float *Self; int64_t rows; int32_t d_out, bd;
    __device__ __forceinline__ void bind(int32_t) {}
    __device__ __forceinline__ void store8(int64_t m, int32_t n, const float4 &x, const float4 &y) const
    {
        if (m >= rows || n >= bd + d_out) return;
        if (n < bd) {
            *reinterpret_cast<uint4 *>(P + m * bd + n) =
                make_uint4(pack2(x.x, x.y), pack2(x.z, x.w), pack2(y.x, y.y), pack2(y.z, y.w));
        } else {
            float *q = Self + m * d_out + (n - bd);
            *reinterpret_cast<float4 *>(q) = x;
            *reinterpret_cast<float4 *>(q + 4) = y;
        }
    }
    __device__ __forceinline__ void store(int64_t, int32_t, float) const {}
};
// d[V | W0] = H^T X accumulated with atomics, computed as (X^T H)^T: A = X (its columns are the tile's rows),
// B = H.  Every column block of X is then read by one block only (X is the big operand, (B+1) d_out columns; H
// has d_in), and with the matrix-core operands swapped as well a lane's neighbours hold neighbouring columns of
// X, so the atomics of a wavefront instruction stay contiguous.
struct EpiWeightGradAtomicT {
    static constexpr bool staged = false, packed = false, swapped = true;
    float *dV, *dW0; int32_t d_in, d_out, B;
    __device__ __forceinline__ void bind(int32_t) {}
    __device__ __forceinline__ void store(int64_t xc, int32_t hc, float v) const   // column of X, column of H
    {
        const int32_t bd = B * d_out;
        if (xc >= bd + d_out || hc >= d_in) return;
        const int32_t b = (int32_t)xc / d_out, c = (int32_t)xc - b * d_out;
        float *dst = b < B ? dV + ((int64_t)b * d_in + hc) * d_out + c : dW0 + (int64_t)hc * d_out + c;
        unsafeAtomicAdd(dst, v);
    }
    __device__ __forceinline__ void store8(int64_t, int32_t, const float4 &, const float4 &) const {}
};
struct EpiRowMajorF32 {
    static constexpr bool staged = false, packed = false, swapped = false;
    float *out; int64_t rows; int32_t cols;
    __device__ __forceinline__ void bind(int32_t) {}
    __device__ __forceinline__ void store(int64_t m, int32_t n, float v) const
    {
        if (m < rows && n < cols) out[m * cols + n] = v;
    }
    __device__ __forceinline__ void store8(int64_t, int32_t, const float4 &, const float4 &) const {}
};
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));     // 16 bytes as a plain vector value

// out[m][n] as bf16, rows below `rows` only.  `packed`: the kernel forms the product transposed (operands
// swapped), so that a lane's accumulators hold 4 consecutive columns of one row; they are rounded to bf16 in
// registers, staged through LDS by 8-byte writes and leave as 16-byte row-contiguous stores.
struct EpiRowsBF16Staged {
    static constexpr bool staged = true, packed = true, swapped = true;
    uint16_t *out; int64_t rows; int32_t cols;
    __device__ __forceinline__ void bind(int32_t) {}
    __device__ __forceinline__ void store_packed(int64_t m, int32_t n, const u32x4 &v) const    // 8 columns from n
    {
        if (m >= rows || n >= cols) return;
        *reinterpret_cast<u32x4 *>(out + m * cols + n) = v;
    }
    __device__ __forceinline__ void store8(int64_t, int32_t, const float4 &, const float4 &) const {}
    __device__ __forceinline__ void store(int64_t, int32_t, float) const {}
};
struct EpiRelOuterAtomic {    // C[group] (d_in x d_out) accumulates the chunks of one relation
    static constexpr bool staged = false, packed = false, swapped = false;
    float *C; int32_t d_in, d_out; int32_t group;
    __device__ __forceinline__ void bind(int32_t g) { group = g; }
    __device__ __forceinline__ void store(int64_t m, int32_t n, float v) const
    {
        if (m < d_in && n < d_out) unsafeAtomicAdd(C + ((int64_t)group * d_in + m) * d_out + n, v);
    }
    __device__ __forceinline__ void store8(int64_t, int32_t, const float4 &, const float4 &) const {}
};

// KC = true : C[m][n] = sum_k A[m][k] B[n][k]   (k-contiguous operands)
// KC = false: C[m][n] = sum_k A[k][m] B[k][n]   (k-strided operands: the contraction index is the row of both)
// Split s contracts [s*kchunk, min((s+1)*kchunk, K)), or, in a grouped launch (g_beg non-null),
// [g_beg[s], g_end[s]) with the epilogue bound to group g_id[s].
// TNt: columns of the block tile, 256 (a wavefront owns 64 x 128: 128 accumulator registers, two blocks
// per CU) or 128 (64 x 64: four blocks per CU, for contractions too short to hide their own latency).
// TKt: contraction depth of a tile, 32 or (k-contiguous operands only) 64: with 64 a row's piece of a
// tile is a whole 128-byte line, and one tile instead of two is in flight in registers.
// k-strided operands (TR in the code): tiles go to LDS as they lie in memory, k-major, by 16-byte loads and stores, and
// the matrix-core operands are fetched with the transposing LDS read of gfx950 (ds_read_b64_tr_b16: within 16
// lanes, lane l receives the l-th 16-bit column of the 4 x 16 block whose four rows lanes 0-3, 4-7, 8-11 and
// 12-15 address 4 columns at a time).  No transposes in registers, a quarter of the load instructions.  The
// launcher checks that columns and pitches are multiples of 8 elements (bf16 layers have such widths).
// MT (k-contiguous operands with a tile list only): a block takes `tpb` consecutive row tiles of the list
// (`tiles_m` then counts such groups and `n_mt` the tiles), and the first loads of the next tile are issued in
// place of the refills that the current tile's last steps have no use for, so that they are in flight while the
// current tile's results go out.  Its loads carry no clamps: the launcher checks that the contraction is a whole
// number of PF * TKt deep rounds over all of A's columns, that B is un-indexed with a multiple of RPP rows in one
// column tile, and that A's (indexed) rows are below 2^31.
template <bool KC, class EPI, int TNt = TN, int TKt = TK, bool MT = false>
__global__ __launch_bounds__(NT, TNt == TN ? 2 : 4) void k_gemm_bf16(MatBF A, MatBF B, EPI epi, int64_t K, int64_t kchunk,
                                                     int32_t tiles_m, int32_t tiles_n, int32_t n_splits,
                                                     const int32_t *__restrict__ g_id,
                                                     const int32_t *__restrict__ g_beg,
                                                     const int32_t *__restrict__ g_end,
                                                     const int32_t *__restrict__ mt_id,
                                                     const int32_t *__restrict__ mt_beg,
                                                     const int32_t *__restrict__ mt_end, int64_t b_group_stride,
                                                     int32_t tpb, int32_t n_mt)
{
    constexpr int NJ = TNt / 64;                 // 32-column MFMA tiles per wavefront
    constexpr int LDKt = TKt == 32 ? 40 : 88;    // LDS row pitch in elements: 80 / 176 bytes, so that the 16-byte
                                                 // operand reads of 8 consecutive rows fall in 8 different bank groups
    constexpr int TPR = TKt / 8, RPP = NT / TPR; // k-contiguous loads: threads per row, rows per pass
    constexpr int PF = TKt == TK ? 2 : 1;        // tiles in flight in registers
    static_assert(KC || TKt == TK, "k-strided operands use the 32-deep tile");
    static_assert(KC || !MT, "several row tiles per block: k-contiguous operands only");
    constexpr bool TR = !KC;
    // TR: LDS rows of TM + 32 and TNt + 32 elements (pitches of 64 bytes modulo 256: the four rows that 16 lanes
    // read at once fall in four different quarters of the banks)
    constexpr int PA = TM + 32, PB = TNt + 32;
    constexpr int LRA = TM / 8, LRB = TNt / 8;             // lanes per tile row, 8 elements each
    constexpr int RA = NT / LRA, RB = NT / LRB;            // tile rows per pass of the block
    constexpr int NLA = TR ? TK / RA : 1, NLB = TR ? TK / RB : 1;   // loads per thread and tile
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t (*As)[LDKt] = reinterpret_cast<uint16_t (*)[LDKt]>(smem);
    uint16_t (*Bs)[LDKt] = reinterpret_cast<uint16_t (*)[LDKt]>(smem + TM * LDKt * 2);

    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int wm = w >> 1, wn = w & 1;
    // block id -> (split, row tile, column tile).  Workgroup i is dispatched to XCD i % 8, each with
    // its own L2.  The (split x row tile, column tile) space is cut into patches of 64 tiles (8 x 8 when there are
    // at least 8 column tiles); a patch goes
    // to one XCD and the 64 blocks that XCD runs at a time are one patch, so every A row tile and B
    // column tile that enters an L2 is used by 8 blocks.
    const int64_t rows_total = (int64_t)n_splits * tiles_m;
    const int pn = tiles_n >= 8 ? 8 : (tiles_n >= 4 ? 4 : (tiles_n >= 2 ? 2 : 1)), pm = 64 / pn;   // patch shape
    const int64_t patches_n = (tiles_n + pn - 1) / pn;
    const int64_t q = blockIdx.x / 8, xcd = blockIdx.x % 8;
    const int64_t patch = (q / 64) * 8 + xcd;
    const int r64 = (int)(q % 64);
    const int64_t prow = (patch / patches_n) * pm + r64 / pn;
    const int32_t tn = (int32_t)((patch % patches_n) * pn + r64 % pn);
    if (prow >= rows_total || tn >= tiles_n) return;          // padding blocks of the last patches
    const int32_t tm = (int32_t)(prow % tiles_m);
    const int64_t bid = prow / tiles_m;                        // split index
    // row tiles: tm * TM, or, with a tile list (mt_beg non-null), rows [mt_beg[tm], mt_end[tm]) of group
    // mt_id[tm] (at most TM rows): A is cut at the tile's end, B is the group's matrix, and the
    // epilogue must not write past the tile (its own row bound is set by the launcher's EPI type)
    int64_t m0 = (int64_t)tm * TM;
    int64_t m_end = A.rows;
    const int32_t t_first = MT ? tm * tpb : tm;                                  // first (only) tile of the list
    const int32_t t_cnt = MT ? (n_mt - t_first < tpb ? n_mt - t_first : tpb) : 1;
    const uint16_t *Bp = B.p;
    if (mt_beg) {
        m0 = mt_beg[t_first];
        m_end = mt_end[t_first];
        if (KC) A.rows = m_end;
        Bp = B.p + (int64_t)mt_id[t_first] * b_group_stride;
    }
    const int32_t n0 = tn * TNt;
    int64_t kbeg = bid * kchunk;
    int64_t kend = (kbeg + kchunk < K) ? kbeg + kchunk : K;
    if (g_beg) { kbeg = g_beg[bid]; kend = g_end[bid]; epi.bind(g_id[bid]); }

    floatx16 acc[2][NJ];

    // Two tiles are in flight in registers while a third is multiplied out of LDS (24 registers per
    // tile, 16-byte octets), so that nothing waits for a load before the matrix-core loop.  Rows picked
    // through an index list have their indices fetched one tile earlier still, which keeps the row loads
    // themselves independent.
    struct Regs {
        u32x4 a[KC ? TM / RPP : NLA], b[KC ? TNt / RPP : NLB];
        uint32_t keep;      // which of a[] are inside the contraction range: applied when the tile goes to LDS, so
                            // that nothing touches the loaded registers (and waits for them) before that
    };
    Regs rg[PF];
    // KC = false: stored rows of A and of B for this thread's loads of the tile that is loaded next (16 or 32
    // lanes share a row).  A k past the range's end takes the range's last row instead (kend <= rows of both
    // operands) and clears its bit in kmask: every load is then unconditional - no divergent branch per load -
    // and only A's octets are zeroed for such a k, which makes the product vanish whatever finite row B repeats.
    // Two sets of them, used in turn: the rows of tile j + 3 are fetched (into the set tile j + 1 no longer needs)
    // AHEAD of the loads of tile j + 2.  A wavefront's memory operations retire in order, so waiting for indices
    // that were issued behind a tile's loads would wait for those loads too, and nothing would stay in flight
    // across a step.
    struct RowSet { int32_t tai[NLA], tbi[NLB]; uint32_t kmask; };
    RowSet rs[2];
    rs[0].kmask = rs[1].kmask = 0u;
    uint16_t *As2 = reinterpret_cast<uint16_t *>(smem), *Bs2 = As2 + TK * PA;

    auto load_rows = [&](int64_t k0, RowSet &S) __attribute__((always_inline)) {
        if constexpr (TR) {
            S.kmask = 0u;
#pragma unroll
            for (int i = 0; i < NLA; ++i) {
                const int64_t rl = k0 + t / LRA + RA * i, rcl = rl < kend ? rl : kend - 1;
                S.tai[i] = A.idx ? A.idx[rcl] : (int32_t)rcl;
                S.kmask |= (rl < kend ? 1u : 0u) << i;
            }
#pragma unroll
            for (int i = 0; i < NLB; ++i) {
                const int64_t rl = k0 + t / LRB + RB * i, rcl = rl < kend ? rl : kend - 1;
                S.tbi[i] = B.idx ? B.idx[rcl] : (int32_t)rcl;
            }
        }
    };
    // k-contiguous operands: the stored rows of this thread's tile rows (through the index lists), fetched
    // once.  Rows past an operand's end repeat its last row: they only feed outputs the epilogue drops, and
    // every load stays unconditional.
    constexpr int NAR = KC ? TM / RPP : 1;
    using arow_t = typename std::conditional<MT, int32_t, int64_t>::type;   // MT: rows of a list-indexed operand, < 2^31
    arow_t arow[NAR], arow_n[MT ? NAR : 1];
    int64_t bcrow[KC ? TNt / RPP : 1];
    int64_t m0_n = 0, m_end_n = 0;               // MT: the tile after the current one
    const uint16_t *Bp_n = Bp;
    auto a_rows = [&](int64_t mb, int64_t rows, arow_t *out) __attribute__((always_inline)) {
#pragma unroll
        for (int ps = 0; ps < NAR; ++ps) {
            const int64_t r = mb + t / TPR + ps * RPP, rc = r < rows ? r : rows - 1;
            out[ps] = A.idx ? (arow_t)A.idx[rc] : (arow_t)rc;
        }
    };
    if constexpr (KC) {
        a_rows(m0, A.rows, arow);
#pragma unroll
        for (int ps = 0; ps < TNt / RPP; ++ps) {
            const int64_t r = n0 + t / TPR + ps * RPP, rc = r < B.rows ? r : B.rows - 1;
            bcrow[ps] = B.idx ? (int64_t)B.idx[rc] : rc;
        }
    }
    auto load_tile = [&](int64_t k0, Regs &R, const arow_t *arow, const uint16_t *Bp, const RowSet &S) __attribute__((always_inline)) {
        if constexpr (MT) {
            // the launcher guarantees whole tiles along k, an un-indexed B and B.rows a multiple of RPP: no clamps.
            // B rows: one 32-bit lane offset behind a scalar base per pass; A rows: the address is rebuilt from
            // the 32-bit row at every load (kept opaque, or the 64-bit addresses of both tiles would stay live)
            const uint32_t ko2 = (uint32_t)(t % TPR) * 16u;
#pragma unroll
            for (int ps = 0; ps < NAR; ++ps) {
                arow_t r = arow[ps];
                asm volatile("" : "+v"(r));
                const char *ap = reinterpret_cast<const char *>(A.p) + ((int64_t)r * A.ld + k0) * 2;
                R.a[ps] = *reinterpret_cast<const u32x4 *>(ap + ko2);
            }
            const uint32_t voff = (uint32_t)(t / TPR) * (uint32_t)B.ld * 2u + ko2;
#pragma unroll
            for (int ps = 0; ps < TNt / RPP; ++ps) {
                const int64_t prow = ps * RPP < B.rows ? ps * RPP : 0;
                const char *bb = reinterpret_cast<const char *>(Bp) + (prow * B.ld + k0) * 2;
                R.b[ps] = *reinterpret_cast<const u32x4 *>(bb + voff);
            }
        } else if constexpr (KC) {
            // an octet past the contraction range reads octet 0 instead, and A's copy of it is zeroed
            const int ko = (t % TPR) * 8;
            const bool kok = k0 + ko < kend && k0 + ko < A.cols;
            const int64_t kc = kok ? k0 + ko : 0;
#pragma unroll
            for (int ps = 0; ps < TM / RPP; ++ps)
                R.a[ps] = *reinterpret_cast<const u32x4 *>(A.p + (int64_t)arow[ps] * A.ld + kc);
            R.keep = kok ? 1u : 0u;
#pragma unroll
            for (int ps = 0; ps < TNt / RPP; ++ps) R.b[ps] = *reinterpret_cast<const u32x4 *>(Bp + bcrow[ps] * B.ld + kc);
        } else if constexpr (TR) {
            // 8 consecutive columns of one row per load; an octet past the matrix reads its last octet instead
            const int32_t ca0 = (int32_t)m0 + (t % LRA) * 8, ca = ca0 + 8 <= A.cols ? ca0 : A.cols - 8;
            const int32_t cb0 = n0 + (t % LRB) * 8, cb = cb0 + 8 <= B.cols ? cb0 : B.cols - 8;
#pragma unroll
            for (int i = 0; i < NLA; ++i)
                R.a[i] = *reinterpret_cast<const u32x4 *>(A.p + (int64_t)S.tai[i] * A.ld + ca);
            R.keep = S.kmask;
#pragma unroll
            for (int i = 0; i < NLB; ++i) R.b[i] = *reinterpret_cast<const u32x4 *>(Bp + (int64_t)S.tbi[i] * B.ld + cb);
        }
    };
    auto store_tile = [&](Regs &R) __attribute__((always_inline)) {
        if constexpr (KC) {
            const int row = t / TPR, ko = (t % TPR) * 8;
#pragma unroll
            for (int ps = 0; ps < TM / RPP; ++ps)
                *reinterpret_cast<u32x4 *>(&As[row + ps * RPP][ko]) = (MT || R.keep) ? R.a[ps] : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int ps = 0; ps < TNt / RPP; ++ps) *reinterpret_cast<u32x4 *>(&Bs[row + ps * RPP][ko]) = R.b[ps];
        } else if constexpr (TR) {
#pragma unroll
            for (int i = 0; i < NLA; ++i)
                *reinterpret_cast<u32x4 *>(&As2[(t / LRA + RA * i) * PA + (t % LRA) * 8]) =
                    (R.keep >> i) & 1u ? R.a[i] : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < NLB; ++i)
                *reinterpret_cast<u32x4 *>(&Bs2[(t / LRB + RB * i) * PB + (t % LRB) * 8]) = R.b[i];
        }
    };
    auto mma_tile = [&]() __attribute__((always_inline)) {
        if constexpr (TR) {
            typedef short s16x4 __attribute__((ext_vector_type(4)));
            // lane -> (row lane % 32 of the 32-row operand tile, k-group lane / 32); as an addressing lane of its
            // group of 16 it points at k-row (lane % 16) / 4 of the group's four and at columns 4 (lane % 4) ...
            const int l16 = lane & 15, kr0 = 8 * (lane >> 5) + (l16 >> 2), mc = 16 * ((lane >> 4) & 1) + 4 * (l16 & 3);
            auto frag = [&](const uint16_t *tile, int pitch, int kr, int col) __attribute__((always_inline)) {
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (s16x4 __attribute__((address_space(3))) *)(tile + kr * pitch + col));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (s16x4 __attribute__((address_space(3))) *)(tile + (kr + 4) * pitch + col));
                return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            };
#pragma unroll
            for (int ks = 0; ks < TKt; ks += 16) {
                bf16x8 af[2], bfr[NJ];
#pragma unroll
                for (int i = 0; i < 2; ++i) af[i] = frag(As2, PA, ks + kr0, wm * 64 + i * 32 + mc);
#pragma unroll
                for (int j = 0; j < NJ; ++j) bfr[j] = frag(Bs2, PB, ks + kr0, wn * (TNt / 2) + j * 32 + mc);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        acc[i][j] = EPI::swapped ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0)
                                                 : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
            }
            return;
        }
#pragma unroll
        for (int ks = 0; ks < TKt; ks += 16) {
            const int kc = ks + 8 * (lane >> 5);
            bf16x8 af[2], bfr[NJ];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                af[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&As[wm * 64 + i * 32 + (lane & 31)][kc]));
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                bfr[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&Bs[wn * (TNt / 2) + j * 32 + (lane & 31)][kc]));
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = EPI::swapped ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0)
                                            : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
    };
    // one step of the pipeline: tile k0 (held in R) goes to LDS and is multiplied; R is refilled with tile
    // k0 + PF TK, or (MT) with the same-numbered early tile of the block's next row tile
    bool has_next = false;
    const int64_t kwrap = (kend - kbeg + TKt - 1) / TKt * TKt;   // MT: a whole number of PF-tile rounds (kbeg = 0)
    // S: the rows of the tile that refills R (fetched a step ago); Sn: where the rows of the tile after it go
    auto step = [&](int64_t k0, Regs &R, RowSet &S, RowSet &Sn) __attribute__((always_inline)) {
        __syncthreads();                 // previous tile fully consumed
        store_tile(R);
        __syncthreads();
        const int64_t kn = k0 + PF * TKt;
        if (kn < kend) { load_rows(kn + TKt, Sn); load_tile(kn, R, arow, Bp, S); }
        else if (MT && has_next) load_tile(kn - kwrap, R, arow_n, Bp_n, S);
        mma_tile();
    };

    // The same step where the refill is known to lie inside the range: no condition around the loads, so that the
    // compiler can count the memory operations issued after the tile it is about to use and waits for that tile
    // only (behind a condition it has to assume the fewest and waits for everything in flight).
    auto step_full = [&](int64_t k0, Regs &R, RowSet &S, RowSet &Sn) __attribute__((always_inline)) {
        __syncthreads();
        store_tile(R);
        __syncthreads();
        load_rows(k0 + (PF + 1) * TKt, Sn);
        load_tile(k0 + PF * TKt, R, arow, Bp, S);
        mma_tile();
    };
    const bool long_range = PF == 2 && !MT && kend - kbeg >= 4 * TKt;    // uniform over the block
    if (long_range) {
        load_rows(kbeg, rs[0]);
        load_rows(kbeg + TKt, rs[1]);
        load_tile(kbeg, rg[0], arow, Bp, rs[0]);
        load_rows(kbeg + 2 * TKt, rs[0]);
        load_tile(kbeg + TKt, rg[1], arow, Bp, rs[1]);
    } else if (kbeg < kend) {
        load_rows(kbeg, rs[0]);
        load_rows(kbeg + TKt, rs[1]);
        load_tile(kbeg, rg[0], arow, Bp, rs[0]);
        if (PF == 2 && kbeg + TKt < kend) { load_rows(kbeg + 2 * TKt, rs[0]); load_tile(kbeg + TKt, rg[1], arow, Bp, rs[1]); }
    }
    for (int32_t ti = 0; ti < t_cnt; ++ti) {
    if constexpr (MT) {
        has_next = ti + 1 < t_cnt;
        if (has_next) {                  // the next tile's rows, fetched a whole tile ahead of their loads
            m0_n = mt_beg[t_first + ti + 1];
            m_end_n = mt_end[t_first + ti + 1];
            Bp_n = B.p + (int64_t)mt_id[t_first + ti + 1] * b_group_stride;
            a_rows(m0_n, m_end_n, arow_n);
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    if constexpr (PF == 2) {
        int64_t k0 = kbeg;
        if (long_range) {
            for (; k0 + 4 * TKt <= kend; k0 += 2 * TKt) {     // both refills of the pair lie inside the range
                step_full(k0, rg[0], rs[0], rs[1]);
                step_full(k0 + TKt, rg[1], rs[1], rs[0]);
            }
        }
        for (; k0 < kend; k0 += 2 * TKt) {
            step(k0, rg[0], rs[0], rs[1]);
            if (k0 + TKt < kend) step(k0 + TKt, rg[1], rs[1], rs[0]);
        }
    } else {
        for (int64_t k0 = kbeg; k0 < kend; k0 += TKt) step(k0, rg[0], rs[0], rs[0]);
    }
    // D register v of lane l: row 8*(v/4) + 4*(l/32) + v%4, column l%32 of its 32x32 tile
    if constexpr (EPI::packed) {
        // transposed product: register v of lane l is row l%32, column 8*(v/4) + 4*(l/32) + v%4 of the tile
        constexpr int SP = TNt / 2 + 8;            // staged row pitch, bf16 elements (16-byte multiple)
        uint16_t *stage = reinterpret_cast<uint16_t *>(smem) + w * 32 * SP;     // 32 rows per wavefront
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            __syncthreads();             // operand tiles (or the previous row group) no longer needed
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<uint2 *>(&stage[(lane & 31) * SP + j * 32 + 8 * q + 4 * (lane >> 5)]) =
                        make_uint2(pack2(acc[i][j][4 * q], acc[i][j][4 * q + 1]),
                                   pack2(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]));
            __syncthreads();
            constexpr int LPRW = NJ * 4;             // lanes across a wavefront's row of NJ * 32 columns, 8 each
#pragma unroll
            for (int it = 0; it < 32 / (64 / LPRW); ++it) {
                const int row = it * (64 / LPRW) + lane / LPRW, c8 = (lane % LPRW) * 8;
                const u32x4 v = *reinterpret_cast<const u32x4 *>(&stage[row * SP + c8]);
                if (m0 + wm * 64 + i * 32 + row < m_end || !mt_beg)
                    epi.store_packed(m0 + wm * 64 + i * 32 + row, n0 + wn * (TNt / 2) + c8, v);
            }
        }
    } else if (EPI::staged) {
        constexpr int ELD = TNt / 2;               // floats per staged row: one wavefront's columns
        float *stage = reinterpret_cast<float *>(smem) + w * 32 * ELD;   // 32 rows x 128 columns per wavefront
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            __syncthreads();             // operand tiles (or the previous row group) no longer needed
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    stage[(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * ELD + j * 32 + (lane & 31)] = acc[i][j][v];
            __syncthreads();
            constexpr int LPRW = NJ * 4;             // lanes across a wavefront's row of NJ * 32 columns, 8 each
#pragma unroll
            for (int it = 0; it < 32 / (64 / LPRW); ++it) {
                const int row = it * (64 / LPRW) + lane / LPRW, c8 = (lane % LPRW) * 8;
                const float4 x = *reinterpret_cast<const float4 *>(&stage[row * ELD + c8]);
                const float4 y = *reinterpret_cast<const float4 *>(&stage[row * ELD + c8 + 4]);
                if (m0 + wm * 64 + i * 32 + row < m_end || !mt_beg)
                    epi.store8(m0 + wm * 64 + i * 32 + row, n0 + wn * (TNt / 2) + c8, x, y);
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    // swapped operands: the lane runs along the tile's rows and the registers along its columns
                    const int rr = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3), cc = lane & 31;
                    const int row = wm * 64 + i * 32 + (EPI::swapped ? cc : rr);
                    const int col = wn * (TNt / 2) + j * 32 + (EPI::swapped ? rr : cc);
                    if (m0 + row < m_end || !mt_beg) epi.store(m0 + row, n0 + col, acc[i][j][v]);
                }
    }
    if constexpr (MT) {
        if (has_next) {
            m0 = m0_n; m_end = m_end_n; Bp = Bp_n;
#pragma unroll
            for (int ps = 0; ps < NAR; ++ps) arow[ps] = arow_n[ps];
        }
    }
    }   // row tiles of the block
}

// ---- conversion kernels
__global__ void k_cvt_rows(const float4 *__restrict__ src, int64_t n4, uint2 *__restrict__ dst)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n4; i += stride) {
        const float4 x = src[i];
        dst[i] = make_uint2(pack2(x.x, x.y), pack2(x.z, x.w));
    }
}

// G (fp32 [N][d_out]) -> columns [bd, bd + d_out) of X (bf16 [N][nc])
__global__ void k_append_g(const float4 *__restrict__ G, int64_t N, int32_t d_out, int32_t bd, int32_t nc,
                           uint16_t *__restrict__ X)
{
    const int d4 = d_out >> 2;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x, n4 = N * d4;
    for (; i < n4; i += stride) {
        const int64_t r = i / d4;
        const int c = (int)(i - r * d4) * 4;
        const float4 x = G[i];
        *reinterpret_cast<uint2 *>(X + r * nc + bd + c) = make_uint2(pack2(x.x, x.y), pack2(x.z, x.w));
    }
}

// The activation's backward pass with both outputs: G = dH (masked by Hout > 0 for ReLU) in fp32, and its bf16
// copy behind the B d_out columns of dP in X (one pass over dH and Hout instead of a second one over G)
__global__ void k_act_backward_append(const float4 *__restrict__ dH, const float4 *__restrict__ Hout, int act,
                                      int64_t N, int32_t d_out, int32_t bd, int32_t nc, float4 *__restrict__ G,
                                      uint16_t *__restrict__ X)
{
    const int d4 = d_out >> 2;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x, n4 = N * d4;
    for (; i < n4; i += stride) {
        const int64_t r = i / d4;
        const int c = (int)(i - r * d4) * 4;
        float4 g = dH[i];
        if (act == KGE_ACT_RELU) {
            const float4 h = Hout[i];
            g.x = h.x > 0.f ? g.x : 0.f; g.y = h.y > 0.f ? g.y : 0.f;
            g.z = h.z > 0.f ? g.z : 0.f; g.w = h.w > 0.f ? g.w : 0.f;
        }
        G[i] = g;
        *reinterpret_cast<uint2 *>(X + r * nc + bd + c) = make_uint2(pack2(g.x, g.y), pack2(g.z, g.w));
    }
}

// [V_1 .. V_B | W0] (fp32) -> Wbf [d_in][nc] and WbfT [nc][d_in], bf16
__global__ void k_cvt_weights(const float *__restrict__ V, const float *__restrict__ W0, int32_t d_in,
                              int32_t d_out, int32_t B, uint16_t *__restrict__ Wbf, uint16_t *__restrict__ WbfT)
{
    const int32_t nc = (B + 1) * d_out;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)d_in * nc) return;
    const int32_t k = (int32_t)(idx / nc), n = (int32_t)(idx - (int64_t)k * nc);
    const int32_t b = n / d_out, c = n - b * d_out;
    const float v = b < B ? V[((int64_t)b * d_in + k) * d_out + c] : W0[(int64_t)k * d_out + c];
    const uint16_t h = (uint16_t)(pack2(v, 0.f) & 0xffffu);
    Wbf[idx] = h;
    WbfT[(int64_t)n * d_in + k] = h;
}

template <bool KC, class EPI, int TNt = TN, int TKt = TK, bool MT = false>
int launch_gemm(const MatBF &A, const MatBF &B, const EPI &epi, int64_t K, int64_t kchunk, int32_t tiles_m,
                int32_t tiles_n, int64_t splits, hipStream_t st, const int32_t *g_id = nullptr,
                const int32_t *g_beg = nullptr, const int32_t *g_end = nullptr, const int32_t *mt_id = nullptr,
                const int32_t *mt_beg = nullptr, const int32_t *mt_end = nullptr, int64_t b_group_stride = 0,
                int32_t tpb = 1)
{
    const int32_t n_mt = tiles_m;                 // MT: tiles in the list; tiles_m becomes groups of tpb
    if (MT) {
        constexpr int PFt = TKt == TK ? 2 : 1, RPPt = NT / (TKt / 8);
        KGE_REQUIRE(tpb >= 1 && mt_beg && !g_beg && splits == 1 && tiles_n == 1 && !B.idx && K == A.cols &&
                        K % (PFt * TKt) == 0 && B.rows % RPPt == 0 && B.rows <= TNt && A.rows < 0x7fffffffLL,
                    KGE_EINVAL, "shape not supported by the multi-tile row product");
        tiles_m = (int32_t)cdiv(n_mt, tpb);
    }
    const int pn = tiles_n >= 8 ? 8 : (tiles_n >= 4 ? 4 : (tiles_n >= 2 ? 2 : 1)), pm = 64 / pn;
    const int64_t n_patches = cdiv(splits * tiles_m, pm) * cdiv(tiles_n, pn);
    const int64_t blocks = cdiv(n_patches, 8) * 8 * 64;
    KGE_REQUIRE(blocks < 0x7fffffffLL, KGE_ERANGE, "grid too large");
    constexpr bool TR = !KC;
    if (TR)
        KGE_REQUIRE(A.cols >= 8 && B.cols >= 8 && A.cols % 8 == 0 && B.cols % 8 == 0 && A.ld % 8 == 0 && B.ld % 8 == 0 &&
                        reinterpret_cast<uintptr_t>(A.p) % 16 == 0 && reinterpret_cast<uintptr_t>(B.p) % 16 == 0 &&
                        b_group_stride % 8 == 0,
                    KGE_EINVAL, "shape not supported by the 16-byte k-strided loader");
    const size_t lds_main = TR ? (size_t)TK * (TM + 32 + TNt + 32) * 2 : (size_t)(TM + TNt) * (TKt == 32 ? 40 : 88) * 2, lds_epi = EPI::packed ? (size_t)4 * 32 * (TNt / 2 + 8) * 2 : (size_t)4 * 32 * (TNt / 2) * 4;
    const size_t lds = EPI::staged ? (lds_epi > lds_main ? lds_epi : lds_main) : lds_main;
    static bool attr_set = false;
    if (!attr_set) {
        KGE_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_bf16<KC, EPI, TNt, TKt, MT>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set = true;
    }
    k_gemm_bf16<KC, EPI, TNt, TKt, MT><<<(unsigned)blocks, NT, lds, st>>>(A, B, epi, K, kchunk, tiles_m, tiles_n,
                                                                (int32_t)splits, g_id, g_beg, g_end, mt_id, mt_beg, mt_end,
                                                                b_group_stride, tpb, n_mt);
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

}  // namespace

int launch_cvt_rows_bf16(const float *src, int64_t n, void *dst, hipStream_t st)
{
    if (n == 0) return KGE_OK;
    int64_t n4 = n / 4, blocks = cdiv(n4, 256);
    if (blocks > 65536) blocks = 65536;
    KGE_PROF("cvt_rows", st);
    k_cvt_rows<<<(unsigned)blocks, 256, 0, st>>>(reinterpret_cast<const float4 *>(src), n4, reinterpret_cast<uint2 *>(dst));
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

int launch_append_g_bf16(const float *G, int64_t N, int32_t d_out, int32_t B, void *X, hipStream_t st)
{
    if (N == 0) return KGE_OK;
    int64_t blocks = cdiv(N * (d_out / 4), 256);
    if (blocks > 65536) blocks = 65536;
    KGE_PROF("append_g", st);
    k_append_g<<<(unsigned)blocks, 256, 0, st>>>(reinterpret_cast<const float4 *>(G), N, d_out, B * d_out,
                                                 (B + 1) * d_out, reinterpret_cast<uint16_t *>(X));
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

int launch_act_backward_append_bf16(const float *dHout, const float *Hout, int act, int64_t N, int32_t d_out, int32_t B,
                                    float *G, void *X, hipStream_t st)
{
    const int64_t n4 = N * (d_out / 4);
    if (n4 == 0) return KGE_OK;
    int64_t blocks = cdiv(n4, 256);
    if (blocks > 65536) blocks = 65536;
    KGE_PROF("act_bwd", st);
    k_act_backward_append<<<(unsigned)blocks, 256, 0, st>>>(reinterpret_cast<const float4 *>(dHout),
                                                            reinterpret_cast<const float4 *>(Hout), act, N, d_out,
                                                            B * d_out, (B + 1) * d_out, reinterpret_cast<float4 *>(G),
                                                            reinterpret_cast<uint16_t *>(X));
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

int launch_cvt_weights_bf16(const float *V, const float *W0, int32_t d_in, int32_t d_out, int32_t B, void *Wbf,
                            void *WbfT, hipStream_t st)
{
    const int64_t n = (int64_t)d_in * (B + 1) * d_out;
    KGE_PROF("cvt_weights", st);
    k_cvt_weights<<<(unsigned)cdiv(n, 256), 256, 0, st>>>(V, W0, d_in, d_out, B, reinterpret_cast<uint16_t *>(Wbf),
                                                         reinterpret_cast<uint16_t *>(WbfT));
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

// [P | Self] = Hbf * [V | W0]      Hbf: bf16 [N][d_in]; WbfT: bf16 [nc][d_in]
static int project_gemm(const void *Hbf, int64_t N, int32_t d_in, int32_t d_out, int32_t B, const void *WbfT, void *P,
                        float *Self, const char *prof_name, hipStream_t st);

int launch_project_bf16(const void *Hbf, int64_t N, int32_t d_in, int32_t d_out, int32_t B, const void *WbfT,
                        void *P, float *Self, hipStream_t st)
{
    if (N == 0) return KGE_OK;
    if (B > 0 && rel_rows_bf16_supported(d_in, d_out)) {
        // the B basis projections: every V_b held in registers while the input rows stream past (rel_rows_bf16.hip);
        // the self-loop product (fp32 out) stays on the GEMM
        int rc;
        {
            KGE_PROF("project", st);
            rc = launch_all_rows_bf16(Hbf, N, WbfT, B, d_in, d_out, P, st);
        }
        if (rc != KGE_OK || !Self) return rc;
        return project_gemm(Hbf, N, d_in, d_out, 0, reinterpret_cast<const uint16_t *>(WbfT) + (int64_t)B * d_out * d_in,
                            nullptr, Self, "project_self", st);
    }
    return project_gemm(Hbf, N, d_in, d_out, B, WbfT, P, Self, "project", st);
}

static int project_gemm(const void *Hbf, int64_t N, int32_t d_in, int32_t d_out, int32_t B, const void *WbfT, void *P,
                        float *Self, const char *prof_name, hipStream_t st)
{
    const int32_t nc = (B + 1) * d_out;
    const int32_t tiles_m = (int32_t)cdiv(N, TM), tiles_n = (int32_t)cdiv(nc, TN);
    MatBF A{reinterpret_cast<const uint16_t *>(Hbf), N, d_in, d_in, nullptr};
    MatBF Bm{reinterpret_cast<const uint16_t *>(WbfT), nc, d_in, d_in, nullptr};
    EpiProjectStaged ep{reinterpret_cast<uint16_t *>(P), Self, N, d_out, B * d_out};
    KGE_PROF(prof_name, st);
    return launch_gemm<true, EpiProjectStaged, TN, 64>(A, Bm, ep, d_in, cdiv(d_in, TK) * TK, tiles_m, tiles_n, 1, st);
}

// d[V | W0] = Hbf^T X     X: bf16 [N][nc] = [dP | G]
int launch_weight_grad_bf16(const void *Hbf, int64_t N, int32_t d_in, int32_t d_out, int32_t B, const void *X,
                            float *dV, float *dW0, hipStream_t st)
{
    int rc = launch_fill_zero(dV, sizeof(float) * (size_t)B * d_in * d_out, st);
    if (rc != KGE_OK) return rc;
    rc = launch_fill_zero(dW0, sizeof(float) * (size_t)d_in * d_out, st);
    if (rc != KGE_OK) return rc;
    if (N == 0) return KGE_OK;
    const int32_t nc = (B + 1) * d_out;
    if (rel_outer_bf16_supported(d_in, d_out)) {     // the row-streaming kernel of rel_outer_bf16.hip
        KGE_PROF("weight_grad", st);
        return launch_col_blocks_outer_bf16(Hbf, N, X, nc, B + 1, d_in, d_out, dV, dW0, st);
    }
    // X as the row operand: 128 of its columns per block against all (up to 256) columns of H at a time
    const int32_t tiles_m = (int32_t)cdiv(nc, TM), tiles_n = (int32_t)cdiv(d_in, TN);
    int64_t splits = cdiv(2048, (int64_t)tiles_m * tiles_n);
    int64_t kchunk = cdiv(cdiv(N, splits), TK) * TK;
    if (kchunk < 8 * TK) kchunk = 8 * TK;
    splits = cdiv(N, kchunk);
    MatBF Xm{reinterpret_cast<const uint16_t *>(X), N, nc, nc, nullptr};
    MatBF Hm{reinterpret_cast<const uint16_t *>(Hbf), N, d_in, d_in, nullptr};
    EpiWeightGradAtomicT ep{dV, dW0, d_in, d_out, B};
    KGE_PROF("weight_grad", st);
    return launch_gemm<false, EpiWeightGradAtomicT>(Xm, Hm, ep, N, kchunk, tiles_m, tiles_n, splits, st);
}

// dH = X [V | W0]^T        Wbf: bf16 [d_in][nc]
int launch_input_grad_bf16(const void *X, int64_t N, int32_t d_in, int32_t d_out, int32_t B, const void *Wbf,
                           float *dH, hipStream_t st)
{
    if (N == 0) return KGE_OK;
    const int32_t nc = (B + 1) * d_out;
    const int32_t tiles_m = (int32_t)cdiv(N, TM), tiles_n = (int32_t)cdiv(d_in, TN);
    MatBF A{reinterpret_cast<const uint16_t *>(X), N, nc, nc, nullptr};
    MatBF Bm{reinterpret_cast<const uint16_t *>(Wbf), d_in, nc, nc, nullptr};
    EpiRowMajorF32 ep{dH, N, d_in};
    KGE_PROF("input_grad", st);
    return launch_gemm<true, EpiRowMajorF32, TN, 64>(A, Bm, ep, nc, cdiv(nc, TK) * TK, tiles_m, tiles_n, 1, st);
}

// C[r] (d_in x d_out, fp32, zeroed here) = sum_{runs s of relation r} Zbf[s]^T Gbf[seg_dst[s]]
// Gbf: bf16 rows of d_out elements, `ldg` elements apart (the G block appended behind dP)
int launch_rel_outer_bf16(const kge_partition *p, const void *Zbf, const int32_t *zrow, const void *Gbf, int64_t ldg,
                          int32_t d_in, int32_t d_out, float *C, hipStream_t st)
{
    const int64_t R2 = 2 * (int64_t)p->n_relations;
    int rc = launch_fill_zero(C, sizeof(float) * (size_t)R2 * d_in * d_out, st);
    if (rc != KGE_OK) return rc;
    if (p->n_seg == 0 || p->n_relc == 0) return KGE_OK;
    if (rel_outer_bf16_supported(d_in, d_out)) {     // the row-streaming kernel of rel_outer_bf16.hip
        KGE_PROF("rel_outer", st);
        return launch_rel_outer_rows_bf16(p, Zbf, d_in, zrow, Gbf, ldg, d_in, d_out, C, st);
    }
    const int32_t tiles_m = (int32_t)cdiv(d_in, TM), tiles_n = (int32_t)cdiv(d_out, TN);
    MatBF A{reinterpret_cast<const uint16_t *>(Zbf), p->n_seg, d_in, d_in, zrow};
    MatBF Bm{reinterpret_cast<const uint16_t *>(Gbf), p->n_seg, d_out, ldg, p->seg_dst};
    EpiRelOuterAtomic ep{C, d_in, d_out, 0};
    KGE_PROF("rel_outer", st);
    return launch_gemm<false, EpiRelOuterAtomic>(A, Bm, ep, p->n_seg, 0, tiles_m, tiles_n, p->n_relc, st,
                                                 p->relc_rel, p->relc_beg, p->relc_end);
}

// Wb[r][k][n] and WbT[r][n][k] = bf16(sum_b a[r][b] V[b][k][n]): Eq. 2 written out for every relation, summed in
// fp32 in the order of b and rounded once, in the two orientations the per-run products read; the fp32 matrices
// are never stored.  One block: a 32 x 32 tile of (k, n) for RB relations.  A thread owns four neighbouring n of
// one k (one 16-byte load of V per basis, served by L2: the blocks that share a tile are neighbours in the
// grid); the coefficients are uniform over the block and come through scalar loads.  The transposed copy goes
// through LDS.  d_in and d_out are multiples of 4 here.
template <int RB>
__global__ __launch_bounds__(256) void k_relation_weights_bf16(const float *__restrict__ a, int32_t R2, int32_t B,
                                                               const float *__restrict__ V, int32_t d_in,
                                                               int32_t d_out, uint16_t *__restrict__ Wb,
                                                               uint16_t *__restrict__ WbT)
{
    constexpr int PT = 36;                       // tile pitch in elements: rows 8-byte aligned
    __shared__ uint16_t tile[RB][32][PT];
    const int r0 = blockIdx.x * RB;
    const int tiles_n = (d_out + 31) >> 5;
    const int k0 = (int)(blockIdx.y / tiles_n) * 32, n0 = (int)(blockIdx.y % tiles_n) * 32;
    const int kk = threadIdx.x >> 3, c4 = (threadIdx.x & 7) * 4;
    const int64_t dd = (int64_t)d_in * d_out;
    const bool in = k0 + kk < d_in && n0 + c4 < d_out;
    const float *vp = V + (in ? (int64_t)(k0 + kk) * d_out + n0 + c4 : 0);
    const float *ar[RB];
#pragma unroll
    for (int j = 0; j < RB; ++j) ar[j] = a + (int64_t)min(r0 + j, R2 - 1) * B;
    float4 acc[RB];
#pragma unroll
    for (int j = 0; j < RB; ++j) acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    int b = 0;
    for (; b + 4 <= B; b += 4) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4 *>(vp + (b + u) * dd);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                const float c = ar[j][b + u];
                acc[j].x = fmaf(c, v[u].x, acc[j].x); acc[j].y = fmaf(c, v[u].y, acc[j].y);
                acc[j].z = fmaf(c, v[u].z, acc[j].z); acc[j].w = fmaf(c, v[u].w, acc[j].w);
            }
    }
    for (; b < B; ++b) {
        const float4 v = *reinterpret_cast<const float4 *>(vp + b * dd);
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            const float c = ar[j][b];
            acc[j].x = fmaf(c, v.x, acc[j].x); acc[j].y = fmaf(c, v.y, acc[j].y);
            acc[j].z = fmaf(c, v.z, acc[j].z); acc[j].w = fmaf(c, v.w, acc[j].w);
        }
    }
#pragma unroll
    for (int j = 0; j < RB; ++j) {
        const uint2 h = make_uint2(pack2(acc[j].x, acc[j].y), pack2(acc[j].z, acc[j].w));
        if (in && r0 + j < R2)
            *reinterpret_cast<uint2 *>(Wb + (int64_t)(r0 + j) * dd + (int64_t)(k0 + kk) * d_out + n0 + c4) = h;
        *reinterpret_cast<uint2 *>(&tile[j][kk][c4]) = h;
    }
    __syncthreads();
    // transposed: this thread now owns four neighbouring k (c4 ..) of one n (kk)
    if (n0 + kk < d_out && k0 + c4 < d_in) {
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            if (r0 + j >= R2) break;
            const uint32_t e0 = tile[j][c4][kk], e1 = tile[j][c4 + 1][kk], e2 = tile[j][c4 + 2][kk],
                           e3 = tile[j][c4 + 3][kk];
            *reinterpret_cast<uint2 *>(WbT + (int64_t)(r0 + j) * dd + (int64_t)(n0 + kk) * d_in + k0 + c4) =
                make_uint2(e0 | (e1 << 16), e2 | (e3 << 16));
        }
    }
}

// The relation matrices of Eq. 2 straight to bf16: Wb [2R][d_in][d_out] and WbT [2R][d_out][d_in]
int launch_relation_weights_bf16(const float *a, int32_t R2, int32_t B, const float *V, int32_t d_in, int32_t d_out,
                                 void *Wb, void *WbT, hipStream_t st)
{
    if (R2 == 0) return KGE_OK;
    constexpr int RB = 16;
    const int64_t tiles = cdiv(d_in, 32) * cdiv(d_out, 32);
    KGE_REQUIRE(d_in % 4 == 0 && d_out % 4 == 0 && tiles <= 65535, KGE_EINVAL,
                "relation weights in bf16: widths must be multiples of 4");
    dim3 grid((unsigned)cdiv(R2, RB), (unsigned)tiles, 1);
    KGE_PROF("rel_weights", st);
    k_relation_weights_bf16<RB><<<grid, 256, 0, st>>>(a, R2, B, V, d_in, d_out, reinterpret_cast<uint16_t *>(Wb),
                                                     reinterpret_cast<uint16_t *>(WbT));
    KGE_LAUNCH_CHECK();
    return KGE_OK;
}

// The per-run products take the kernel of rel_rows_bf16.hip when it supports the layer's widths (64, 128 or 256
// in, a multiple of 32 up to 256 out); the rest runs here as a grouped GEMM over row tiles of the run list.
// Row tiles that one block takes in turn (the next tile's first loads overlap the current tile's stores);
// measured at 25 M runs, d = 256: 1 -> 6.4 ms, 2 -> 6.3, 4 and 8 -> 6.2 (the other kernel: 5.3).
constexpr int32_t ROW_TILES_PER_BLOCK = 4;

// U[s] = Zbf[s] Wrel[rel(s)]   bf16 in, bf16 out; WbT: bf16 [2R][d_out][d_in]
int launch_apply_relation_weights_bf16(const kge_partition *p, const void *Zbf, const int32_t *zrow, const void *WbT,
                                       int32_t d_in, int32_t d_out, void *U, hipStream_t st)
{
    if (p->n_relt == 0) return KGE_OK;
    const int32_t tiles_n = (int32_t)cdiv(d_out, TN);
    MatBF A{reinterpret_cast<const uint16_t *>(Zbf), p->n_seg, d_in, d_in, zrow};
    MatBF Bm{reinterpret_cast<const uint16_t *>(WbT), d_out, d_in, d_in, nullptr};
    EpiRowsBF16Staged ep{reinterpret_cast<uint16_t *>(U), p->n_seg, d_out};
    KGE_PROF("apply_rel", st);
    if (rel_rows_bf16_supported(d_in, d_out))
        return launch_rel_rows_bf16(p, Zbf, d_in, zrow, WbT, d_in, d_out, U, st);
    if (tiles_n == 1 && d_in % 64 == 0 && d_out % 32 == 0)   // several row tiles per block, the next one's first loads under the current one's stores
        return launch_gemm<true, EpiRowsBF16Staged, TN, 64, true>(A, Bm, ep, d_in, cdiv(d_in, TK) * TK, p->n_relt, tiles_n, 1,
                                                                  st, nullptr, nullptr, nullptr, p->relt_rel, p->relt_beg,
                                                                  p->relt_end, (int64_t)d_in * d_out, ROW_TILES_PER_BLOCK);
    return launch_gemm<true, EpiRowsBF16Staged, TN, 64>(A, Bm, ep, d_in, cdiv(d_in, TK) * TK, p->n_relt, tiles_n, 1, st, nullptr,
                                                nullptr, nullptr, p->relt_rel, p->relt_beg, p->relt_end,
                                                (int64_t)d_in * d_out);
}

// dZ[s] = Gbf[dst(s)] Wrel[rel(s)]^T   Gbf rows of d_out elements, ldg apart; Wb: bf16 [2R][d_in][d_out]
int launch_apply_relation_weights_t_bf16(const kge_partition *p, const void *Gbf, int64_t ldg, const void *Wb,
                                         int32_t d_in, int32_t d_out, void *dZ, hipStream_t st)
{
    if (p->n_relt == 0) return KGE_OK;
    const int32_t tiles_n = (int32_t)cdiv(d_in, TN);
    MatBF A{reinterpret_cast<const uint16_t *>(Gbf), p->n_seg, d_out, ldg, p->seg_dst};
    MatBF Bm{reinterpret_cast<const uint16_t *>(Wb), d_in, d_out, d_out, nullptr};
    EpiRowsBF16Staged ep{reinterpret_cast<uint16_t *>(dZ), p->n_seg, d_in};
    KGE_PROF("apply_rel_t", st);
    if (rel_rows_bf16_supported(d_out, d_in))
        return launch_rel_rows_bf16(p, Gbf, ldg, p->seg_dst, Wb, d_out, d_in, dZ, st, true);
    if (tiles_n == 1 && d_out % 64 == 0 && d_in % 64 == 0)   // two tiles in flight: the contraction must be whole pairs of them
        return launch_gemm<true, EpiRowsBF16Staged, TN, 64, true>(A, Bm, ep, d_out, cdiv(d_out, TK) * TK, p->n_relt, tiles_n, 1,
                                                                  st, nullptr, nullptr, nullptr, p->relt_rel, p->relt_beg,
                                                                  p->relt_end, (int64_t)d_in * d_out, ROW_TILES_PER_BLOCK);
    return launch_gemm<true, EpiRowsBF16Staged>(A, Bm, ep, d_out, cdiv(d_out, TK) * TK, p->n_relt, tiles_n, 1, st, nullptr,
                                                nullptr, nullptr, p->relt_rel, p->relt_beg, p->relt_end,
                                                (int64_t)d_in * d_out);
}
