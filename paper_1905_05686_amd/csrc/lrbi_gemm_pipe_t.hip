// Transposed masked product on the matrix cores, dX = (W o I_a)^T dY (the backward pass through the masking layer,
// Sec. 2: the decoded index acts as a binary mask on W, gradients flow through the kept weights only), in the
// software-pipelined form of the forward tile kernel: both operands go from global memory straight into an LDS ring
// (f16 / bf16, fp32 accumulate), for tile shapes that line up with the blocking (c % 128 == 0, r % 128 == 0,
// k <= 64, no cut-off tiles).
//
// One workgroup of eight wavefronts owns 128 rows of dX (128 columns of W) x 128 batch columns and walks the rows of
// W (the reduction range, possibly one slice of it) in slabs of 64.  What differs from the forward kernel:
//   * A slab of W is 64 rows x 128 columns, row-major as it lies in memory: the same image as the forward kernel's X
//     slab, and so is the slab of dY (64 rows x 128 batch columns).  Both MFMA operands need 8 consecutive reduction
//     steps of one column: both come out of LDS with the transposing read.
//   * The mask is needed transposed: the 16 bytes a lane holds of W for one MFMA are 8 consecutive ROWS of one column
//     of W.  Per panel of 512 rows the kernel forms, for each of its 128 columns j and each 128-row unit, the 128
//     mask bits of those rows: the OR, over the ranks l with (I_z)_{l j} = 1, of column l of I_p (Eq. 3 read along
//     a column).  Column l of I_p as a bit string over 128 rows is gathered bit by bit from the rows' I_p words (they
//     sit in LDS, as in the forward kernel; the bit strings take their place); the ranks of column j are gathered
//     from the I_z rows in LDS the same way.
// The pipeline (four stages, loads three slabs ahead, waits by count, one barrier per slab), the way the mask is
// applied to the operand (select on the bit pattern), the sum of the two halves of every slab through LDS and the
// output through per-wave LDS strips are the forward kernel's.
#include "lrbi_internal.hpp"
#include "lrbi_lds_dma.hpp"
#include "lrbi_mfma_common.hpp"

namespace lrbi {

static constexpr int PT_THREADS = 512;
static constexpr int PT_BJ = 128, PT_BQ = 128;
static constexpr int PT_STAGE_BYTES = 32768; // W: 64 rows x 256 bytes, then dY: 64 rows x 256 bytes
static constexpr int PT_STAGE_Y = 16384;
static constexpr int PT_NS = 4;
static constexpr int PT_MT_ROW = 72;                      // bytes per column of W of a mask panel: 64 + 8
static constexpr int PT_MT_BYTES = PT_BJ * PT_MT_ROW;
static constexpr int PT_FZ_ROWS = FAST_MAX_K;
static constexpr int PT_FZ_ROW_BYTES = PANEL_WORDS * 4;   // 64: four units x four words

// HALF (tile widths that are an odd multiple of 64, e.g. the 576-column tiles of Table 2): the workgroup's 128
// columns may lie in two tile columns, so the I_p words are kept per 64-column half (8 KB instead of 4 KB) and the
// ranks of every column, 4 KB, take the place of the I_z slices once those have been read (one more barrier).
template <bool HALF = false> struct SmemPipeT {
    static constexpr size_t mt_off = (size_t)PT_NS * PT_STAGE_BYTES;
    static constexpr size_t fz_off = mt_off + 2 * PT_MT_BYTES;
    static constexpr size_t fip_off = fz_off + PT_FZ_ROWS * PT_FZ_ROW_BYTES;
    static constexpr size_t sel_off = HALF ? fz_off : fip_off + 128 * PANEL_UNITS * 2 * 4; // (I_p words: 4 KB; later its columns as bits)
    static constexpr size_t bytes = HALF ? fip_off + 128 * PANEL_UNITS * 2 * 2 * 4
                                         : sel_off + PANEL_UNITS * 128 * 8; // the ranks of every column, per unit
};
static_assert(SmemPipeT<true>::bytes <= 160 * 1024 && SmemPipeT<false>::bytes <= 160 * 1024, "LDS of a compute unit");
static_assert(PT_FZ_ROWS * PT_FZ_ROW_BYTES == PANEL_UNITS * 128 * 8, "the ranks of the columns fit where the I_z slices were");

template <typename Tag, bool SPLIT, bool HALF = false>
__global__ __launch_bounds__(PT_THREADS) void mfma_gemm_pipe_t_kernel(
    Geom g, const uint16_t *__restrict__ W, int64_t ldw, const uint32_t *__restrict__ Ip,
    const uint32_t *__restrict__ Iz, const uint16_t *__restrict__ DY, int64_t lddy, int N,
    uint16_t *__restrict__ DX, int64_t lddx, float *__restrict__ P, int64_t ldp, int jblocks, int qblocks,
    int64_t iper, int xcd_remap, int y_vec_ok)
{
    constexpr int NS = PT_NS;
    constexpr int FN = PT_BQ / 32;
    using S = SmemPipeT<HALF>;

    extern __shared__ uint4 lrbi_dyn_smem[];
    unsigned char *smem = (unsigned char *)lrbi_dyn_smem;
    unsigned char *Mt = smem + S::mt_off;              // [2][128 columns of W][PT_MT_ROW]: mask bytes along the rows
    uint32_t *Fz = (uint32_t *)(smem + S::fz_off);     // [4 units][4 words][64 ranks]: I_z under the workgroup's 128 columns
    uint32_t *Fip = (uint32_t *)(smem + S::fip_off);   // [4 units][2 words][128 rows] of I_p; then [4][64 ranks][4]: its columns as bits
    uint2 *Sel = (uint2 *)(smem + S::sel_off);         // [4 units][128 columns]: the ranks of a column of I_z (unit's tile)

    int64_t bid = blockIdx.x;
    if (xcd_remap) {
        const int64_t per = gridDim.x / 8;
        bid = (bid % 8) * per + bid / 8;
    }
    const int qi = (int)(bid % qblocks);
    const int ji = (int)((bid / qblocks) % jblocks);
    const int slice = (int)(bid / ((int64_t)qblocks * jblocks));
    const int j0 = ji * PT_BJ;
    const int q0 = qi * PT_BQ;
    const int64_t ibeg = (int64_t)slice * iper;
    const int64_t iend = (ibeg + iper < g.m) ? ibeg + iper : g.m;
    const int nslabs = (int)((iend - ibeg) / BK); // whole slabs only: m % 128 == 0, iper % 128 == 0
    const int last = nslabs - 1;
    const int npanels = (nslabs + PANEL_SLABS - 1) / PANEL_SLABS;
    const int tj = j0 / g.c;                       // the workgroup's columns lie inside one tile column (c % 128 == 0)
    const int coff = j0 - tj * g.c;
    const int tjb = (j0 + 64) / g.c;               // HALF: tile column and offset of the upper 64 columns
    const int coffb = j0 + 64 - tjb * g.c;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = wave >> 2; // which half of every slab's 16-row steps
    const int wq = wave & 3;  // which 32 columns of W (rows of dX)
    const int l32 = lane & 31, lg = lane >> 5;

    // ---- global -> LDS: both slabs are 64 rows of 256 bytes; piece p of row q is stored at slot p ^ (2 (q & 3)); a
    // load instruction fills 4 rows; wavefront w issues the chunks w and w + 8
    uint32_t wvo[2], yvo[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int chunk = wave + 8 * i;
        const int xr = chunk * 4 + (lane >> 4);
        const int xp = (lane & 15) ^ (2 * (xr & 3));
        wvo[i] = (uint32_t)((xr * ldw + xp * 8) * 2);
        int nn = xp * 8;
        if (q0 + nn + 8 > N) nn = N - 8 - q0; // piece beyond N: fetch a valid piece instead, its columns are dropped
        yvo[i] = (uint32_t)((xr * lddy + nn) * 2);
    }
    const uint16_t *wbase = W + ibeg * ldw + j0;
    const uint16_t *ybase = DY + ibeg * lddy + q0;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    auto issue_piece = [&](int slab, int stage, auto i_c) {
        constexpr int i = decltype(i_c)::value;
        const uint32_t sb = lds0 + (uint32_t)stage * PT_STAGE_BYTES + (uint32_t)wave * 1024u;
        if constexpr (i < 2) load_to_lds16(sb + i * 8192u, wbase + (int64_t)slab * BK * ldw, wvo[i]);
        else load_to_lds16(sb + PT_STAGE_Y + (i - 2) * 8192u, ybase + (int64_t)slab * BK * lddy, yvo[i - 2]);
    };

    // ---- operand reads (transposing read): 16-lane group G = lane / 16 serves columns 16 (G % 2) .. + 15 of a
    // 32-column block and reduction group G / 2; lane d of the group addresses row d / 4, columns 4 (d % 4).
    // Block a sits 64 (a ^ t) bytes further, t = bit 2 of the row's swizzle.  This wavefront's steps are 2 kg + j.
    const int d16 = lane & 15, G16 = lane >> 4;
    uint32_t xfe, xfo; // blocks a = 0, 2 (+128) and a = 1, 3 (+128) of a slab image, step j = 0 (+4096 for j = 1)
    {
        const int q = 8 * (G16 >> 1) + (d16 >> 2);
        const int sw = 2 * (q & 3);
        const int p = (2 * (G16 & 1) + ((d16 & 3) >> 1)) ^ (sw & 2);
        const int t = (sw >> 2) & 1;
        const uint32_t base = (uint32_t)(kg * 8192 + q * 256 + p * 16 + 8 * (d16 & 1));
        xfe = base + 64u * t;
        xfo = base + 64u * (1 - t);
    }
    const uint32_t wta = ((wq & 1) ? xfo : xfe) + (uint32_t)((wq >> 1) * 128); // the W block of this wavefront
    // mask bytes of this lane's column of W: 8 bytes per slab, of which this wavefront's steps use bytes 4 kg + 2 j + lg
    const uint32_t mta = (uint32_t)((wq * 32 + l32) * PT_MT_ROW);

    u32x4 wf[2][2], yf[2][FN]; // W operands [slab parity][j]; dY operands [j][block]
    auto read_w = [&](int stage, auto par_c, auto j_c) {
        constexpr int par = decltype(par_c)::value, j = decltype(j_c)::value;
        const unsigned char *p = smem + stage * PT_STAGE_BYTES + wta + j * 4096;
        const u32x2 lo = lds_read_tr16_v((const uint16_t *)p);
        const u32x2 hi = lds_read_tr16_v((const uint16_t *)(p + 1024));
        wf[par][j] = u32x4{lo.x, lo.y, hi.x, hi.y};
    };
    auto read_y = [&](int stage, auto j_c, auto a_c) {
        constexpr int j = decltype(j_c)::value, a = decltype(a_c)::value;
        const unsigned char *p = smem + stage * PT_STAGE_BYTES + PT_STAGE_Y + ((a & 1) ? xfo : xfe) + (a >> 1) * 128 + j * 4096;
        const u32x2 lo = lds_read_tr16_v((const uint16_t *)p);
        const u32x2 hi = lds_read_tr16_v((const uint16_t *)(p + 1024));
        yf[j][a] = u32x4{lo.x, lo.y, hi.x, hi.y};
    };
    f32x16 acc[FN];
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][v] = 0.f;
    auto mma = [&](auto par_c, auto j_c, auto a_c) {
        constexpr int par = decltype(par_c)::value, j = decltype(j_c)::value, a = decltype(a_c)::value;
        acc[a] = mfma_32x32x16(Tag{}, yf[j][a], wf[par][j], acc[a]);
    };
    // mask of a W operand: m holds this wavefront's two mask bytes of the slab, step j's at bits 16 j
    auto mask_lo = [&](auto par_c, auto j_c, uint32_t m) -> uint32_t {
        constexpr int par = decltype(par_c)::value, j = decltype(j_c)::value;
        const uint32_t bits8 = (m >> (16 * j)) & 0xFFu;
        const uint32_t y = bits8 | (bits8 << 15);
        wf[par][j].x = select2(wf[par][j].x, y & 0x00010001u);
        wf[par][j].y = select2(wf[par][j].y, (y >> 2) & 0x00010001u);
        return y;
    };
    auto mask_hi = [&](auto par_c, auto j_c, uint32_t y) {
        constexpr int par = decltype(par_c)::value, j = decltype(j_c)::value;
        wf[par][j].z = select2(wf[par][j].z, (y >> 4) & 0x00010001u);
        wf[par][j].w = select2(wf[par][j].w, (y >> 6) & 0x00010001u);
    };
    auto fetch_mask = [&](int slab) -> u32x2 {
        const unsigned char *p = Mt + ((slab / PANEL_SLABS) & 1) * PT_MT_BYTES + (slab % PANEL_SLABS) * 8 + mta;
        return *reinterpret_cast<const u32x2 *>(p);
    };
    auto my_bytes = [&](u32x2 mk) -> uint32_t { return (kg ? mk.y : mk.x) >> (8 * lg); };

    // ---- factor slices of one panel (512 rows of W = four units of 128 rows): global -> LDS, word by word, in the
    // order the gathers below want them: I_z as [unit][word of the 128 columns][rank] (a lane then reads four ranks of
    // its word per 16-byte read), I_p as [unit][word][row].  Sixteen load instructions each, two per wavefront.
    // (cti, roff): tile row and row offset inside it of the next panel's first unit; a unit lies inside one tile
    // (r % 128 == 0).  Ranks at or beyond k fetch rank 0 instead and are masked out; units beyond the reduction range
    // fetch the range's first unit and are never used; with one I_p word per row the second word repeats the first.
    int cti = (int)(ibeg / g.r), roff = (int)(ibeg - (ibeg / g.r) * g.r);
    int64_t crow = ibeg;
    const uint32_t zb_first = (uint32_t)(((((int64_t)cti * g.tile_cols + tj) * g.k) * (int64_t)g.izw + (coff >> 5)) * 4);
    const uint32_t pb_first = (uint32_t)(((((int64_t)cti * g.tile_cols + tj) * g.r + roff) * (int64_t)g.ipw) * 4);
    const uint32_t fz_lane = (uint32_t)(((lane < g.k) ? lane : 0) * g.izw * 4);
    int leaders = 1; // bit u: unit u of the panel whose factors were asked for last is the first one of its tile row
    auto load_factors = [&]() {
        uint32_t zb[PANEL_UNITS], pb[PANEL_UNITS];
        leaders = 1;
#pragma unroll
        for (int u = 1; u < PANEL_UNITS; ++u)
            if ((roff + 128 * u) % g.r == 0) leaders |= 1 << u;
        if constexpr (HALF) {
            // the same images with the upper two words of a column's I_z row and a second set of I_p words taken from
            // the upper half's tile: I_z 16 instructions as below, I_p [unit][half][word][row]: 32, four per wavefront
            uint32_t zc[PANEL_UNITS], pc[PANEL_UNITS];
#pragma unroll
            for (int u = 0; u < PANEL_UNITS; ++u) {
                const bool ok = crow < iend;
                const int64_t ta = (int64_t)cti * g.tile_cols + tj, tb = (int64_t)cti * g.tile_cols + tjb;
                zb[u] = ok ? (uint32_t)(((ta * g.k) * (int64_t)g.izw + (coff >> 5)) * 4) : zb_first;
                pb[u] = ok ? (uint32_t)(((ta * g.r + roff) * (int64_t)g.ipw) * 4) : pb_first;
                zc[u] = ok ? (uint32_t)(((tb * g.k) * (int64_t)g.izw + (coffb >> 5)) * 4) : zb_first;
                pc[u] = ok ? (uint32_t)(((tb * g.r + roff) * (int64_t)g.ipw) * 4) : pb_first;
                crow += 128;
                roff += 128;
                if (roff >= g.r) {
                    roff = 0;
                    ++cti;
                }
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int q = wave * 2 + i; // uniform
                const int u = q >> 2, w = q & 3;
                const uint32_t za = u == 0 ? zb[0] : (u == 1 ? zb[1] : (u == 2 ? zb[2] : zb[3]));
                const uint32_t zu = u == 0 ? zc[0] : (u == 1 ? zc[1] : (u == 2 ? zc[2] : zc[3]));
                load_to_lds4(lds0 + (uint32_t)S::fz_off + (uint32_t)q * 256u, Iz,
                             ((w & 2) ? zu : za) + fz_lane + (uint32_t)((w & 1) * 4));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int q = wave * 4 + i; // uniform
                const int u = q >> 3, h = (q >> 2) & 1, iw = ((q >> 1) & 1) < g.ipw ? ((q >> 1) & 1) : 0, row = (q & 1) * 64 + lane;
                const uint32_t pa = u == 0 ? pb[0] : (u == 1 ? pb[1] : (u == 2 ? pb[2] : pb[3]));
                const uint32_t pu = u == 0 ? pc[0] : (u == 1 ? pc[1] : (u == 2 ? pc[2] : pc[3]));
                load_to_lds4(lds0 + (uint32_t)S::fip_off + (uint32_t)q * 256u, Ip, (h ? pu : pa) + (uint32_t)((row * g.ipw + iw) * 4));
            }
            return;
        }
#pragma unroll
        for (int u = 0; u < PANEL_UNITS; ++u) {
            const bool ok = crow < iend;
            const int64_t t = (int64_t)cti * g.tile_cols + tj;
            zb[u] = ok ? (uint32_t)(((t * g.k) * (int64_t)g.izw + (coff >> 5)) * 4) : zb_first;
            pb[u] = ok ? (uint32_t)(((t * g.r + roff) * (int64_t)g.ipw) * 4) : pb_first;
            crow += 128;
            roff += 128;
            if (roff >= g.r) {
                roff = 0;
                ++cti;
            }
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int q = wave * 2 + i; // uniform
            {
                const int u = q >> 2, w = q & 3;
                const uint32_t zsel = u == 0 ? zb[0] : (u == 1 ? zb[1] : (u == 2 ? zb[2] : zb[3]));
                load_to_lds4(lds0 + (uint32_t)S::fz_off + (uint32_t)q * 256u, Iz, zsel + fz_lane + (uint32_t)(w * 4));
            }
            {
                const int u = q >> 2, iw = ((q >> 1) & 1) < g.ipw ? ((q >> 1) & 1) : 0, row = (q & 1) * 64 + lane;
                const uint32_t psel = u == 0 ? pb[0] : (u == 1 ? pb[1] : (u == 2 ? pb[2] : pb[3]));
                load_to_lds4(lds0 + (uint32_t)S::fip_off + (uint32_t)q * 256u, Ip, psel + (uint32_t)((row * g.ipw + iw) * 4));
            }
        }
    };
    // Eq. 3 along the columns of W for one panel, in three steps with a workgroup barrier between them (the factor
    // slices have landed and are visible when the first one runs):
    //  1. lane (unit, rank l, 32-row chunk) gathers bit l of the chunk's 32 I_p words into one word: 32 rows of column
    //     l of I_p (a second word for rank l + 32 when k > 32);
    //  2. (nobody reads the I_p words any more) the gathered words are stored over them as [unit][rank][16 bytes];
    //     in the same step, lane (unit, column j) gathers the ranks of column j, bit j of the I_z rows, for the units
    //     that start a tile row (the units behind them share its I_z);
    //  3. lane (column j, unit): the mask bits of the unit's 128 rows are the OR of the bit strings of the column's
    //     ranks.
    // In the slab loop the three steps ride on the barriers of three consecutive iterations; only the first panel,
    // in the prologue, pays for barriers of its own.  Bits at or beyond k are zero in the packed factors.
    uint32_t tw0 = 0u, tw1 = 0u, tw2 = 0u, tw3 = 0u, csel0 = 0u, csel1 = 0u;
    auto panel_step1 = [&]() {
        const int u = tid >> 7, l = (tid >> 2) & 31, c = tid & 3;
        if constexpr (HALF) { // both halves' I_p words: [unit][half][word][row]
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint4 *src = (const uint4 *)(Fip + ((u * 2 + h) * 2) * 128 + c * 32);
                uint32_t t0 = 0u, t1 = 0u;
#pragma unroll
                for (int i4 = 0; i4 < 8; ++i4) {
                    const uint4 v = src[i4];
                    t0 |= (((v.x >> l) & 1u) | (((v.y >> l) & 1u) << 1) | (((v.z >> l) & 1u) << 2) | (((v.w >> l) & 1u) << 3)) << (4 * i4);
                }
                if (g.k > 32) {
#pragma unroll
                    for (int i4 = 0; i4 < 8; ++i4) {
                        const uint4 v = src[32 + i4];
                        t1 |= (((v.x >> l) & 1u) | (((v.y >> l) & 1u) << 1) | (((v.z >> l) & 1u) << 2) | (((v.w >> l) & 1u) << 3)) << (4 * i4);
                    }
                }
                if (h == 0) {
                    tw0 = t0;
                    tw1 = t1;
                } else {
                    tw2 = t0;
                    tw3 = t1;
                }
            }
            return;
        }
        const uint4 *src = (const uint4 *)(Fip + (u * 2) * 128 + c * 32); // rows 32 c .. + 31 of the unit, word 0
        uint32_t t0 = 0u, t1 = 0u;
#pragma unroll
        for (int i4 = 0; i4 < 8; ++i4) {
            const uint4 v = src[i4];
            t0 |= (((v.x >> l) & 1u) | (((v.y >> l) & 1u) << 1) | (((v.z >> l) & 1u) << 2) | (((v.w >> l) & 1u) << 3)) << (4 * i4);
        }
        if (g.k > 32) {
#pragma unroll
            for (int i4 = 0; i4 < 8; ++i4) {
                const uint4 v = src[32 + i4]; // word 1 of the same rows: 128 words further
                t1 |= (((v.x >> l) & 1u) | (((v.y >> l) & 1u) << 1) | (((v.z >> l) & 1u) << 2) | (((v.w >> l) & 1u) << 3)) << (4 * i4);
            }
        }
        tw0 = t0;
        tw1 = t1;
    };
    auto panel_step2 = [&]() {
        const int u = tid >> 7, l = (tid >> 2) & 31, c = tid & 3;
        if constexpr (HALF) { // [unit][half][rank][16 bytes]
            Fip[((u * 2) * FAST_MAX_K + l) * 4 + c] = tw0;
            Fip[((u * 2 + 1) * FAST_MAX_K + l) * 4 + c] = tw2;
            if (g.k > 32) {
                Fip[((u * 2) * FAST_MAX_K + 32 + l) * 4 + c] = tw1;
                Fip[((u * 2 + 1) * FAST_MAX_K + 32 + l) * 4 + c] = tw3;
            }
            return;
        }
        Fip[(u * FAST_MAX_K + l) * 4 + c] = tw0;
        if (g.k > 32) Fip[(u * FAST_MAX_K + 32 + l) * 4 + c] = tw1;
    };
    auto panel_step3 = [&]() { // lane (unit, column); only the first unit of every tile row under the panel gathers
        const int u = tid >> 7, col = tid & 127;
        if (!((leaders >> u) & 1)) return; // uniform over the wavefront
        const uint4 *fz = (const uint4 *)(Fz + (u * 4 + (col >> 5)) * 64); // this column's word of every rank
        const int sh = col & 31;
        uint32_t sel0 = 0u, sel1 = 0u; // the ranks of this column
#pragma unroll
        for (int l4 = 0; l4 < 8; ++l4) {
            const uint4 v = fz[l4];
            sel0 |= (((v.x >> sh) & 1u) | (((v.y >> sh) & 1u) << 1) | (((v.z >> sh) & 1u) << 2) | (((v.w >> sh) & 1u) << 3)) << (4 * l4);
        }
        if (g.k > 32) {
#pragma unroll
            for (int l4 = 0; l4 < 8; ++l4) {
                const uint4 v = fz[8 + l4];
                sel1 |= (((v.x >> sh) & 1u) | (((v.y >> sh) & 1u) << 1) | (((v.z >> sh) & 1u) << 2) | (((v.w >> sh) & 1u) << 3)) << (4 * l4);
            }
        }
        // slots of ranks at or beyond k hold a stand-in (rank 0)
        if (g.k < 32) sel0 &= (1u << g.k) - 1u;
        if (g.k <= 32) sel1 = 0u;
        else if (g.k < 64) sel1 &= (1u << (g.k - 32)) - 1u;
        if constexpr (HALF) { // kept in registers: the words go where the I_z slices are, behind the next barrier
            csel0 = sel0;
            csel1 = sel1;
        } else {
            Sel[u * 128 + col] = make_uint2(sel0, sel1);
        }
    };
    auto panel_step3b = [&]() { // HALF only
        const int u = tid >> 7, col = tid & 127;
        if (!((leaders >> u) & 1)) return;
        Sel[u * 128 + col] = make_uint2(csel0, csel1);
    };
    auto panel_step4 = [&](int panel) { // lane (column, unit): OR of the bit strings of the column's ranks
        const int col = tid >> 2, u = tid & 3;
        const int lead = 31 - __builtin_clz((uint32_t)(leaders & ((2 << u) - 1))); // the unit that gathered for u's tile row
        const uint2 sel01 = Sel[lead * 128 + col];
        const uint4 *ipt = (const uint4 *)Fip + (HALF ? u * 2 + (col >> 6) : u) * FAST_MAX_K;
        uint4 a = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int iw = 0; iw < 2; ++iw) {
            uint32_t sel = iw ? sel01.y : sel01.x;
            while (sel) { // two ranks per round: their reads are in flight together
                const int la = __builtin_ctz(sel) + 32 * iw;
                sel &= sel - 1u;
                uint4 z = ipt[la];
                if (sel) {
                    const int lb = __builtin_ctz(sel) + 32 * iw;
                    sel &= sel - 1u;
                    const uint4 y = ipt[lb];
                    z = make_uint4(z.x | y.x, z.y | y.y, z.z | y.z, z.w | y.w);
                }
                a = make_uint4(a.x | z.x, a.y | z.y, a.z | z.z, a.w | z.w);
            }
        }
        unsigned char *out = Mt + (panel & 1) * PT_MT_BYTES + col * PT_MT_ROW + u * 16;
        *reinterpret_cast<uint2 *>(out) = make_uint2(a.x, a.y);
        *reinterpret_cast<uint2 *>(out + 8) = make_uint2(a.z, a.w);
    };

    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
#define LRBI_SB() __builtin_amdgcn_sched_barrier(0)
#define LRBI_BARRIER()                                             \
    do {                                                           \
        LRBI_SB();                                                 \
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");         \
        __builtin_amdgcn_s_barrier();                              \
        LRBI_SB();                                                 \
    } while (0)

    // ---- prologue: the factor slices of panel 0 first, then slabs 0 .. NS - 2 (the last one's dY half follows in the
    // first iteration); the panel is decoded as soon as the factor slices are in, slab 0 is waited for after that
    load_factors();
    constexpr int kProloguePieces = (NS - 2) * 4 + 2;
    static_for<NS - 1>([&](auto sc) {
        constexpr int st = decltype(sc)::value;
        const int sl0 = st < last ? st : last;
        issue_piece(sl0, st, I0{});
        issue_piece(sl0, st, I1{});
        if constexpr (st != NS - 2) {
            issue_piece(sl0, st, I2{});
            issue_piece(sl0, st, I3{});
        }
    });
    wait_loads<kProloguePieces>();
    __syncthreads();
    panel_step1();
    __syncthreads();
    panel_step2();
    panel_step3();
    __syncthreads();
    if constexpr (HALF) {
        panel_step3b();
        __syncthreads();
    }
    panel_step4(0);
    wait_loads<kProloguePieces - 4>(); // slab 0
    __syncthreads();
    uint32_t mcur = my_bytes(fetch_mask(0));
    read_w(0, I0{}, I0{});
    read_w(0, I0{}, I1{});
    read_y(0, I0{}, I0{});
    read_y(0, I0{}, I1{});
    read_y(0, I0{}, I2{});
    read_y(0, I0{}, I3{});
    {
        const uint32_t y = mask_lo(I0{}, I0{}, mcur);
        mask_hi(I0{}, I0{}, y);
    }

    // ---- main loop, unrolled by NS: the schedule of the forward kernel (loads spread over the iteration)
    for (int s0 = 0; s0 < nslabs; s0 += NS) {
        static_for<NS>([&](auto sc) {
            constexpr int st = decltype(sc)::value;
            constexpr int st1 = (st + 1) % NS;
            constexpr int stn = (st + NS - 1) % NS;
            constexpr int stp = (st + NS - 2) % NS;
            using Par = std::integral_constant<int, st & 1>;
            using Nxt = std::integral_constant<int, (st & 1) ^ 1>;
            const int s = s0 + st;
            if (s < nslabs) {
                uint32_t y;
                u32x2 mk;
                const int sl = s + NS - 1 < last ? s + NS - 1 : last;
                const int sp = s + NS - 2 < last ? s + NS - 2 : last;
                // first step
                mma(Par{}, I0{}, I0{}); read_y(st, I1{}, I0{}); y = mask_lo(Par{}, I1{}, mcur);
                mma(Par{}, I0{}, I1{}); read_y(st, I1{}, I1{}); mask_hi(Par{}, I1{}, y);
                issue_piece(sp, stp, I2{});
                mma(Par{}, I0{}, I2{}); read_y(st, I1{}, I2{});
                mk = fetch_mask(s + 1 < last ? s + 1 : last);
                mma(Par{}, I0{}, I3{}); read_y(st, I1{}, I3{});
                issue_piece(sp, stp, I3{});
                const int ps = s % PANEL_SLABS;
                const int np = s / PANEL_SLABS + 1;
                if (ps == 0 && np < npanels) load_factors();
                wait_loads<(NS - 3) * 4>();
                LRBI_BARRIER();
                // second step
                mma(Par{}, I1{}, I0{}); read_y(st1, I0{}, I0{}); read_w(st1, Nxt{}, I0{}); read_w(st1, Nxt{}, I1{});
                issue_piece(sl, stn, I0{});
                mma(Par{}, I1{}, I1{}); read_y(st1, I0{}, I1{}); mcur = my_bytes(mk);
                issue_piece(sl, stn, I1{});
                mma(Par{}, I1{}, I2{}); read_y(st1, I0{}, I2{}); y = mask_lo(Nxt{}, I0{}, mcur);
                mma(Par{}, I1{}, I3{}); read_y(st1, I0{}, I3{}); mask_hi(Nxt{}, I0{}, y);
                // mask of the next panel: its factor slices, asked for at slab 0, were waited for by every wavefront in
                // front of slab 1's barrier; the three steps follow the barriers of slabs 1, 2 and 3; first read at slab 7
                if (np < npanels) {
                    if (ps == 1) panel_step1();
                    else if (ps == 2) {
                        panel_step2();
                        panel_step3();
                    } else if (ps == 3) {
                        if constexpr (HALF) panel_step3b();
                        else panel_step4(np);
                    } else if (HALF && ps == 4) panel_step4(np); // (written behind slab 4's barrier, first read at slab 7)
                }
            }
        });
    }
#undef LRBI_SB
#undef LRBI_BARRIER
    wait_loads<0>();
    __syncthreads();

    // ---- the two halves of every slab: wavefronts 4 .. 7 hand their sums to wavefronts 0 .. 3 through LDS
    {
        float *red = (float *)smem + (size_t)wq * (FN * 16 * 64) + lane;
        if (kg == 1) {
#pragma unroll
            for (int a = 0; a < FN; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v) red[(a * 16 + v) * 64] = acc[a][v];
        }
        __syncthreads();
        if (kg == 1) return;
#pragma unroll
        for (int a = 0; a < FN; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][v] += red[(a * 16 + v) * 64];
    }

    // ---- epilogue: lane holds, per 32-column block a, batch columns 8 (v / 4) + 4 lg + (v % 4) of row l32 of dX
    const int64_t row0 = (int64_t)j0 + wq * 32;
    if (SPLIT) {
        constexpr int RS = 128 * 4 + 16;
        unsigned char *strip = smem + 65536 + wq * (32 * RS);
#pragma unroll
        for (int a = 0; a < FN; ++a)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4)
                *reinterpret_cast<float4 *>(strip + l32 * RS + (a * 32 + 8 * v4 + 4 * lg) * 4) =
                    make_float4(acc[a][4 * v4 + 0], acc[a][4 * v4 + 1], acc[a][4 * v4 + 2], acc[a][4 * v4 + 3]);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int rr = 2 * i + lg, col = q0 + 4 * l32;
            const float4 o = *reinterpret_cast<const float4 *>(strip + rr * RS + l32 * 16);
            if (col < ldp) *reinterpret_cast<float4 *>(P + ((int64_t)slice * g.n + row0 + rr) * ldp + col) = o;
        }
    } else {
        constexpr int RS = 128 * 2 + 8;
        unsigned char *strip = smem + 65536 + wq * (32 * RS);
#pragma unroll
        for (int a = 0; a < FN; ++a)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                uint16_t o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = cvt_store(Tag{}, acc[a][4 * v4 + e]);
                *reinterpret_cast<uint2 *>(strip + l32 * RS + (a * 32 + 8 * v4 + 4 * lg) * 2) = *reinterpret_cast<uint2 *>(o);
            }
        const int l16 = lane & 15, rq = lane >> 4;
        const bool y16 = y_vec_ok && (((uintptr_t)DX & 15) == 0) && (lddx % 8 == 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int rr = 4 * i + rq, col = q0 + 8 * l16;
            const uint2 lo = *reinterpret_cast<const uint2 *>(strip + rr * RS + l16 * 16);
            const uint2 hi = *reinterpret_cast<const uint2 *>(strip + rr * RS + l16 * 16 + 8);
            uint16_t *yp = DX + (row0 + rr) * lddx + col;
            if (y16 && col + 7 < N) {
                *reinterpret_cast<uint4 *>(yp) = make_uint4(lo.x, lo.y, hi.x, hi.y);
            } else {
                const uint32_t w4[4] = {lo.x, lo.y, hi.x, hi.y};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (col + e < N) yp[e] = (uint16_t)(w4[e >> 1] >> (16 * (e & 1)));
            }
        }
    }
}

// true when the pipelined transposed kernel serves this call: aligned tile shapes, dY readable in 16-byte pieces, a
// batch wide enough for its 128-column blocks to pay (above 32 columns: HBM-cold 4096 x 9216 at 64 columns 29.3
// against 35.4 us on the staged kernel, 4096 x 4096 18.0 against 21.7 us), offsets that fit the kernel's 32-bit per-lane byte offsets
bool pipe_t_ok(const Geom &g, const void *dW, int64_t ldw, const void *dIz, const void *dDY, int64_t lddy, int64_t N)
{
    if ((g.r % 128) != 0 || g.k > FAST_MAX_K || g.ragged) return false;
    if ((g.c % 128) != 0 && ((g.c % 64) != 0 || (g.n % 128) != 0)) return false; // 64 (2 j + 1): gathered per half
    if ((((uintptr_t)dDY & 15) != 0) || (lddy % 8 != 0) || (N % 8 != 0) || N <= 32) return false;
    if ((((uintptr_t)dW & 15) != 0) || (ldw % 8 != 0)) return false;
    if (((uintptr_t)dIz & 15) != 0) return false;
    if (ldw > (1 << 22) || lddy > (1 << 22)) return false;
    const int64_t tiles = (int64_t)g.tile_rows * g.tile_cols;
    if (tiles * g.k * g.izw * 4 >= (int64_t)1 << 31 || tiles * g.r * g.ipw * 4 >= (int64_t)1 << 31) return false;
    return true;
}

// slices over the rows of W for the pipelined transposed kernel: one workgroup per compute unit at most, at least
// eight slabs per slice, no more slices than the caller's workspace was sized for
int pipe_t_slices(const Geom &g, int64_t N, int max_slices, int64_t *iper)
{
    const int64_t tiles = (g.n / PT_BJ) * ((N + PT_BQ - 1) / PT_BQ);
    const int64_t units = g.m / 128; // slices are cut at multiples of 128 rows
    int64_t want = 256 / (tiles > 0 ? tiles : 1);
    if (want > units / 4) want = units / 4;
    if (want > max_slices) want = max_slices;
    if (want < 1) want = 1;
    const int64_t per = (units + want - 1) / want;
    *iper = per * 128;
    return (int)((units + per - 1) / per);
}

template <typename Tag>
static int launch_pipe_t_dtype(const Geom &g, int slices, int64_t iper, const void *dW, int64_t ldw, const uint32_t *dIp,
                               const uint32_t *dIz, const void *dDY, int64_t lddy, int64_t N, void *dDX, int64_t lddx,
                               void *dWorkspace, hipStream_t stream)
{
    const int64_t jblocks = g.n / PT_BJ, qblocks = (N + PT_BQ - 1) / PT_BQ;
    const int64_t blocks = jblocks * qblocks * slices;
    if (blocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    const int y_vec_ok = (((uintptr_t)dDX & 7) == 0) && (lddx % 4 == 0);
    const int xcd_remap = (blocks % 8 == 0) ? 1 : 0;
    const int64_t ldp = (N + 3) / 4 * 4;
    const bool half = (g.c % 128) != 0;
    const size_t smem = half ? SmemPipeT<true>::bytes : SmemPipeT<false>::bytes;
    auto kern = slices > 1 ? (half ? mfma_gemm_pipe_t_kernel<Tag, true, true> : mfma_gemm_pipe_t_kernel<Tag, true>)
                           : (half ? mfma_gemm_pipe_t_kernel<Tag, false, true> : mfma_gemm_pipe_t_kernel<Tag, false>);
    LRBI_SET_MAX_LDS(kern, smem);
    LRBI_LAUNCH(kern, dim3((unsigned)blocks), dim3(PT_THREADS), smem, stream, g, (const uint16_t *)dW, ldw, dIp, dIz,
                (const uint16_t *)dDY, lddy, (int)N, (uint16_t *)dDX, lddx, (float *)dWorkspace, ldp, (int)jblocks,
                (int)qblocks, iper, xcd_remap, y_vec_ok);
    return LRBI_OK;
}

// the product alone; with more than one slice the caller adds the partial planes [slice][n][ldp]
int launch_pipe_t_gemm(const Geom &g, int slices, int64_t iper, lrbi_dtype dt, const void *dW, int64_t ldw,
                       const uint32_t *dIp, const uint32_t *dIz, const void *dDY, int64_t lddy, int64_t N, void *dDX,
                       int64_t lddx, void *dWorkspace, hipStream_t stream)
{
    if (dt == LRBI_F16)
        return launch_pipe_t_dtype<F16Tag>(g, slices, iper, dW, ldw, dIp, dIz, dDY, lddy, N, dDX, lddx, dWorkspace, stream);
    if (dt == LRBI_BF16)
        return launch_pipe_t_dtype<BF16Tag>(g, slices, iper, dW, ldw, dIp, dIz, dDY, lddy, N, dDX, lddx, dWorkspace, stream);
    return LRBI_ERR_DTYPE;
}

} // namespace lrbi
