// Fused masked product on the matrix cores, tile kernel with both operands loaded straight into LDS
// (f16 / bf16, fp32 accumulate): Y = (W o I_a) X with the mask of Eq. 3 rebuilt inside the kernel, for tile shapes
// that line up with the kernel's blocking (c % 128 == 0, r % 128 == 0, k <= 64, no edge tiles).
//
// One workgroup of eight wavefronts (two per SIMD) owns a 128 x 128 tile of Y and walks the reduction range in
// slabs of 64 columns of W.  Wavefront (kg, wq) owns rows 32 wq .. + 31 of the tile for the 16-column steps
// 2 kg and 2 kg + 1 of every slab; the two halves' sums are added through LDS at the end (fixed order).
//   * Both operands of a slab go from global memory straight into LDS (the load-to-LDS form of the global
//     load: no registers, no LDS store instructions, no vector-ALU work), three slabs ahead of the arithmetic,
//     into a ring of four stages.  A lane may fetch any 16-byte piece, but lands it at (stage base + 16 lane):
//     the pieces are fetched in a permuted order, so that the linear image in LDS is the swizzled layout in
//     which the operand reads below hit every bank once (no padding).
//   * The mask is applied where a W operand leaves LDS: the 16 bytes a lane holds for one MFMA are 8
//     consecutive weights of one row, their 8 mask bits one byte of that row's mask.  Pruned weights are zeroed by a
//     packed 16-bit integer multiply by 0 / 1 (a select on the bit pattern: nothing stored under a 0 bit, NaN
//     and Inf included, reaches the product).
//   * The mask itself is rebuilt one panel (512 columns) at a time, one panel ahead, from the panel's slices of
//     the factors (also loaded straight into LDS): mask row = OR of the I_z rows that the row's I_p word selects
//     (Eq. 3).
//   * X stays in its natural [k][n] order in LDS and is read with the transposing LDS read of gfx950.
//   * One workgroup barrier per slab, without a drain of the loads in flight: what must have landed is waited
//     for by count.  Two wavefronts per SIMD: measured, one wavefront per SIMD cannot keep enough 8-byte LDS
//     reads in flight (68 against 160 bytes per clock and compute unit).
//   * The output tile leaves through LDS as 16-byte pieces of whole rows.
#include "lrbi_internal.hpp"
#include "lrbi_lds_dma.hpp"
#include "lrbi_mfma_common.hpp"

namespace lrbi {

static constexpr int PIPE_THREADS = 512;
static constexpr int PIPE_BM = 128, PIPE_BN = 128;
static constexpr int STAGE_BYTES = 32768; // W: 128 rows x 128 bytes, then X: 64 rows x 256 bytes
static constexpr int STAGE_X = 16384;
static constexpr int MT_ROW = 72;                    // bytes per row of a mask panel: 64 + 8 (conflict-free 8-byte reads)
static constexpr int MT_BYTES = PIPE_BM * MT_ROW;    // one mask panel
static constexpr int FZ_ROWS = FAST_MAX_K + 1;       // I_z rows under a panel; row 64 stays zero
static constexpr int FZ_ROW_BYTES = PANEL_WORDS * 4; // 64

template <int NS, bool HALF = false> struct SmemDma {
    static constexpr size_t mt_off = (size_t)NS * STAGE_BYTES;
    static constexpr size_t fz_off = mt_off + 2 * MT_BYTES;
    static constexpr size_t fip_off = fz_off + FZ_ROWS * FZ_ROW_BYTES;
    static constexpr size_t bytes = fip_off + PIPE_BM * PANEL_UNITS * (HALF ? 2 : 1) * 2 * 4;
};
static_assert(SmemDma<4, true>::bytes <= 160 * 1024, "LDS of a compute unit");


// CONV: X is not a matrix in memory but a zero-padded activation [B][H + 2][Wd + 2][C] (channels fastest), and column
// (b, oh, ow) of the product's X holds, at reduction index (kh * 3 + kw) * C + ci, the value act[b][oh + kh][ow + kw][ci]
// (a 3 x 3 convolution with padding 1 written as a product, the unfolded matrix never materialised).  A slab of 64
// reduction indices is then 64 consecutive channels of one tap: 128 contiguous bytes per column, which go into the
// stage in the same swizzled row-major image as W's rows and come out with the same 16-byte operand reads.
// EMIT: the mask bytes that the kernel rebuilds anyway also go to global memory, in the layout of the stand-alone
// decode (one bit per weight, rows of `mask_pitch16` 16-byte pieces): every (row, 128-column unit) of the mask is
// formed by exactly one workgroup of the first column block, so the decode costs one 16-byte store per lane and
// panel instead of a kernel of its own.
// HALF: tile widths that are an odd multiple of 64 (the paper's 576-column tiles, Table 2): a 128-column unit may
// then lie across two tile columns, so the factor slices are gathered, and Eq. 3 is evaluated, per 64-column half
// unit, each with the I_p word and the I_z words of its own tile.  Everything behind the mask bytes is the same.
template <typename Tag, int NS, bool SPREAD, bool SPLIT, bool CONV, bool EMIT = false, bool HALF = false>
__global__ __launch_bounds__(PIPE_THREADS) void mfma_gemm_pipe_kernel(
    Geom g, const uint16_t *__restrict__ W, int64_t ldw, const uint32_t *__restrict__ Ip,
    const uint32_t *__restrict__ Iz, const uint16_t *__restrict__ X, int64_t ldx, int N,
    uint16_t *__restrict__ Y, int64_t ldy, float *__restrict__ P, int64_t ldp, int mblocks, int nblocks,
    int64_t kper, int xcd_remap, int y_vec_ok, ConvGeom cg, uint4 *__restrict__ mask_out, int64_t mask_pitch16)
{
    static_assert(NS == 4, "LDS stages (an even number: the W operand registers alternate with the slab's parity)");
    static_assert(!SPREAD || NS == 4, "loads spread over the iteration land one iteration later: four stages");
    constexpr int FN = PIPE_BN / 32; // 32-column blocks of the wave tile
    static_assert(!(HALF && CONV), "half units: the plain product only");
    using S = SmemDma<NS, HALF>;

    extern __shared__ uint4 lrbi_dyn_smem[];
    unsigned char *smem = (unsigned char *)lrbi_dyn_smem;
    unsigned char *Mt = smem + S::mt_off;                // [2][128][MT_ROW]  mask bytes of two panels
    uint32_t *Fz = (uint32_t *)(smem + S::fz_off);       // [65][16]          I_z rows under the panel being decoded
    uint32_t *Fip = (uint32_t *)(smem + S::fip_off);     // [128][4][2]       I_p words per row and 128-column unit
                                                         // (HALF: [128][8][2], per 64-column half unit)

    int64_t bid = blockIdx.x;
    if (xcd_remap) {
        const int64_t per = gridDim.x / 8;
        bid = (bid % 8) * per + bid / 8;
    }
    const int ni = (int)(bid % nblocks);
    const int mi = (int)((bid / nblocks) % mblocks);
    const int slice = (int)(bid / ((int64_t)nblocks * mblocks));
    const int64_t m0 = (int64_t)mi * PIPE_BM;
    const int n0 = ni * PIPE_BN;
    const int kbeg = (int)(slice * kper);
    const int kend = (int)((kbeg + kper < g.n) ? kbeg + kper : g.n);
    const int nslabs = (kend - kbeg) / BK; // whole slabs only: n % 128 == 0, kper % 128 == 0
    const int last = nslabs - 1;
    const int npanels = (nslabs + PANEL_SLABS - 1) / PANEL_SLABS;
    const int ti = (int)(m0 / g.r); // the workgroup's rows lie inside one tile row (r % 128 == 0)
    const int il0 = (int)(m0 - (int64_t)ti * g.r);
    const int64_t trow = (int64_t)ti * g.tile_cols;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // 0 .. 7
    const int kg = wave >> 2;                                  // which half of every slab's 16-column steps
    const int wq = wave & 3;                                   // which 32 rows of the tile
    const int l32 = lane & 31, lg = lane >> 5;

    // ---- global -> LDS: per-lane byte offsets of the pieces this lane fetches (they never change)
    // W stage image: row-major 128-byte rows, piece p of row q stored at slot p ^ ((q >> 1) & 7).  A load
    // instruction fills 1 KiB = 8 rows; wavefront w issues the chunks w and w + 8.
    // X stage image: row-major 256-byte rows, piece p of row q stored at slot p ^ (2 (q & 3)); a load instruction
    // fills 4 rows; same chunk assignment.
    uint32_t wvo[2], xvo[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int chunk = wave + 8 * i;
        const int wr = chunk * 8 + (lane >> 3);
        const int wp = (lane & 7) ^ ((wr >> 1) & 7);
        wvo[i] = (uint32_t)((wr * ldw + wp * 8) * 2);
        if constexpr (CONV) {
            // same image as W: 8 columns of X (128 bytes of channels each) per instruction
            const int xr = chunk * 8 + (lane >> 3);
            const int xp = (lane & 7) ^ ((xr >> 1) & 7);
            int col = n0 + xr;
            if (col >= N) col = N - 1; // column beyond N: a valid column instead, it is dropped at the end
            const int hw = cg.H * cg.Wd;
            const int b = col / hw, rem = col - b * hw;
            const int oh = rem / cg.Wd, ow = rem - oh * cg.Wd;
            const int64_t pix = ((int64_t)b * (cg.H + 2) + oh) * (cg.Wd + 2) + ow; // tap (0, 0) of the column
            xvo[i] = (uint32_t)((pix * cg.cin + xp * 8) * 2);
        } else {
            const int xr = chunk * 4 + (lane >> 4);
            const int xp = (lane & 15) ^ (2 * (xr & 3));
            int nn = xp * 8;
            if (n0 + nn + 8 > N) nn = N - 8 - n0; // piece beyond N: fetch a valid piece instead, its columns are dropped
            xvo[i] = (uint32_t)((xr * ldx + nn) * 2);
        }
    }
    const uint16_t *wbase = W + m0 * ldw + kbeg;
    const uint16_t *xbase = CONV ? X : X + (int64_t)kbeg * ldx + n0;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    // piece i (0, 1: W chunks, 2, 3: X chunks) of a slab into a stage
    auto issue_piece = [&](int slab, int stage, auto i_c) {
        constexpr int i = decltype(i_c)::value;
        const uint32_t sb = lds0 + (uint32_t)stage * STAGE_BYTES + (uint32_t)wave * 1024u;
        if constexpr (i < 2) load_to_lds16(sb + i * 8192u, wbase + slab * BK, wvo[i]);
        else if constexpr (CONV) {
            // the slab's 64 reduction indices: channels ci0 .. ci0 + 63 of tap (kh, kw)
            const int kidx = kbeg + slab * BK;
            const int tap = kidx / cg.cin, ci0 = kidx - tap * cg.cin;
            const int kh = tap / 3, kw = tap - 3 * kh;
            load_to_lds16(sb + STAGE_X + (i - 2) * 8192u, xbase + ((kh * (cg.Wd + 2) + kw) * cg.cin + ci0), xvo[i - 2]);
        } else
            load_to_lds16(sb + STAGE_X + (i - 2) * 8192u, xbase + (int64_t)slab * BK * ldx, xvo[i - 2]);
    };

    // ---- operand reads: byte addresses inside a stage.  This wavefront's steps are kk = 2 kg + j, j = 0, 1.
    // W operand of step kk: row q = 32 wq + (lane % 32), piece 2 kk + (lane / 32)
    uint32_t wfa[2];
    {
        const int q = wq * 32 + l32;
        const int c7 = (q >> 1) & 7;
#pragma unroll
        for (int j = 0; j < 2; ++j) wfa[j] = (uint32_t)(q * 128 + (((2 * (2 * kg + j) + lg) ^ c7) * 16));
    }
    // X operand (transposing read): 16-lane group G = lane / 16 serves columns 16 (G % 2) .. + 15 of a
    // 32-column block and k group G / 2; lane d of the group addresses row d / 4, columns 4 (d % 4).
    // Block a sits 64 (a ^ t) bytes further, t = bit 2 of the row's swizzle.
    const int d16 = lane & 15, G16 = lane >> 4;
    uint32_t xfe, xfo; // blocks a = 0, 2 (+128) and a = 1, 3 (+128), step j = 0 (+4096 for j = 1)
    {
        const int q = 8 * (G16 >> 1) + (d16 >> 2); // row inside the step (+ 4 for the upper half)
        const int sw = 2 * (q & 3);
        const int p = (2 * (G16 & 1) + ((d16 & 3) >> 1)) ^ (sw & 2);
        const int t = (sw >> 2) & 1;
        const uint32_t base = (uint32_t)(STAGE_X + kg * 8192 + q * 256 + p * 16 + 8 * (d16 & 1));
        xfe = base + 64u * t;
        xfo = base + 64u * (1 - t);
    }
    // mask bytes of this lane's row: 8 bytes per slab, of which this wavefront's steps use bytes 4 kg + 2 j + lg
    const uint32_t mta = (uint32_t)((wq * 32 + l32) * MT_ROW);

    u32x4 wf[2][2], xf[2][FN]; // W operands [slab parity][j]; X operands [j][block]
    auto read_w = [&](int stage, auto par_c, auto j_c) {
        constexpr int par = decltype(par_c)::value, j = decltype(j_c)::value;
        wf[par][j] = *reinterpret_cast<const u32x4 *>(smem + stage * STAGE_BYTES + wfa[j]);
    };
    // CONV: X operand of step kk, block a: column q = 32 a + (lane % 32), piece 2 kk + (lane / 32), image as W's
    uint32_t xca[2];
    {
        const int c7 = (l32 >> 1) & 7; // (q >> 1) & 7 does not depend on the block
#pragma unroll
        for (int j = 0; j < 2; ++j) xca[j] = (uint32_t)(STAGE_X + l32 * 128 + (((2 * (2 * kg + j) + lg) ^ c7) * 16));
    }
    auto read_x = [&](int stage, auto j_c, auto a_c) {
        constexpr int j = decltype(j_c)::value, a = decltype(a_c)::value;
        if constexpr (CONV) {
            xf[j][a] = *reinterpret_cast<const u32x4 *>(smem + stage * STAGE_BYTES + xca[j] + a * 4096);
            return;
        }
        const unsigned char *p = smem + stage * STAGE_BYTES + ((a & 1) ? xfo : xfe) + (a >> 1) * 128 + j * 4096;
        const u32x2 lo = lds_read_tr16_v((const uint16_t *)p);
        const u32x2 hi = lds_read_tr16_v((const uint16_t *)(p + 1024));
        xf[j][a] = u32x4{lo.x, lo.y, hi.x, hi.y};
    };
    f32x16 acc[FN];
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][v] = 0.f;
    auto mma = [&](auto par_c, auto j_c, auto a_c) {
        constexpr int par = decltype(par_c)::value, j = decltype(j_c)::value, a = decltype(a_c)::value;
        acc[a] = mfma_32x32x16(Tag{}, xf[j][a], wf[par][j], acc[a]);
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
        const unsigned char *p = Mt + ((slab / PANEL_SLABS) & 1) * MT_BYTES + (slab % PANEL_SLABS) * 8 + mta;
        return *reinterpret_cast<const u32x2 *>(p);
    };
    auto my_bytes = [&](u32x2 mk) -> uint32_t { return (kg ? mk.y : mk.x) >> (8 * lg); };

    // ---- factor slices of one panel: global -> LDS (the same load-to-LDS form), then Eq. 3 for the panel.
    // (ctj, coff): tile column and column offset inside it of the next panel to be loaded; a 128-column unit
    // lies inside one tile (c % 128 == 0), so stepping by 128 lands exactly on tile borders.
    // I_z: wavefronts 0 .. 3 fetch ranks 16 w .. + 15, lane = (rank, unit): the unit's four words of that
    // rank's row.  Ranks at or beyond k fetch rank 0 instead: no I_p bit selects them (pad bits are zero).
    // Units beyond the reduction range fetch the range's first unit instead: their mask bytes are never read.
    // I_p: one word per lane, 256 bytes per instruction, two instructions per wavefront, image [row][unit][2];
    // with one word per row the second word's slot receives the first word again and is ignored below.
    int ctj = kbeg / g.c, coff = kbeg - (kbeg / g.c) * g.c, ccol = kbeg;
    const uint32_t zb_first = (uint32_t)((((trow + ctj) * g.k) * (int64_t)g.izw + (coff >> 5)) * 4);
    const uint32_t pb_first = (uint32_t)((((trow + ctj) * g.r + il0) * (int64_t)g.ipw) * 4);
    const int fz_l = wq * 16 + (lane >> 2);
    const uint32_t fz_lane = (uint32_t)(((fz_l < g.k) ? fz_l : 0) * g.izw * 4);
    const int fz_u = lane & 3;
    auto load_factors = [&]() {
        if constexpr (HALF) {
            // per half unit (64 columns, two words of an I_z row): one word per lane.  I_z: instruction q of 16
            // (two per wavefront) fills ranks 4 q .. + 3, lane = (rank, half unit, word); I_p: image
            // [row][half unit][2], four instructions per wavefront.
            constexpr int HU = 2 * PANEL_UNITS;
            uint32_t zb[HU], pb[HU];
#pragma unroll
            for (int h = 0; h < HU; ++h) {
                const bool ok = ccol < kend;
                zb[h] = ok ? (uint32_t)((((trow + ctj) * g.k) * (int64_t)g.izw + (coff >> 5)) * 4) : zb_first;
                pb[h] = ok ? (uint32_t)((((trow + ctj) * g.r + il0) * (int64_t)g.ipw) * 4) : pb_first;
                ccol += 64;
                coff += 64;
                if (coff >= g.c) {
                    coff = 0;
                    ++ctj;
                }
            }
            const int hu = (lane >> 1) & 7;
            const uint32_t zlo = (hu & 2) ? ((hu & 1) ? zb[3] : zb[2]) : ((hu & 1) ? zb[1] : zb[0]);
            const uint32_t zhi = (hu & 2) ? ((hu & 1) ? zb[7] : zb[6]) : ((hu & 1) ? zb[5] : zb[4]);
            const uint32_t plo = (hu & 2) ? ((hu & 1) ? pb[3] : pb[2]) : ((hu & 1) ? pb[1] : pb[0]);
            const uint32_t phi = (hu & 2) ? ((hu & 1) ? pb[7] : pb[6]) : ((hu & 1) ? pb[5] : pb[4]);
            const uint32_t zsel = (hu & 4) ? zhi : zlo, psel = (hu & 4) ? phi : plo;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int q = wave * 2 + i;
                const int rank = q * 4 + (lane >> 4);
                load_to_lds4(lds0 + (uint32_t)S::fz_off + (uint32_t)q * 256u, Iz,
                             zsel + (uint32_t)((((rank < g.k) ? rank : 0) * g.izw + (lane & 1)) * 4));
            }
            const int iw = (lane & 1) < g.ipw ? (lane & 1) : 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int q = wave * 4 + i;
                const int row = q * 4 + (lane >> 4);
                load_to_lds4(lds0 + (uint32_t)S::fip_off + (uint32_t)q * 256u, Ip, psel + (uint32_t)((row * g.ipw + iw) * 4));
            }
            return;
        }
        uint32_t zb[PANEL_UNITS], pb[PANEL_UNITS]; // byte offsets of each unit's tile slices (uniform)
#pragma unroll
        for (int u = 0; u < PANEL_UNITS; ++u) {
            const bool ok = ccol < kend;
            zb[u] = ok ? (uint32_t)((((trow + ctj) * g.k) * (int64_t)g.izw + (coff >> 5)) * 4) : zb_first;
            pb[u] = ok ? (uint32_t)((((trow + ctj) * g.r + il0) * (int64_t)g.ipw) * 4) : pb_first;
            ccol += 128;
            coff += 128;
            if (coff >= g.c) {
                coff = 0;
                ++ctj;
            }
        }
        if (kg == 0) {
            const uint32_t zsel = fz_u == 0 ? zb[0] : (fz_u == 1 ? zb[1] : (fz_u == 2 ? zb[2] : zb[3]));
            load_to_lds16(lds0 + (uint32_t)S::fz_off + (uint32_t)wq * 1024u, Iz, zsel + fz_lane);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int idx = (wave * 2 + i) * 64 + lane;
            const int row = idx >> 3, u = (idx >> 1) & 3, iw = (idx & 1) < g.ipw ? (idx & 1) : 0;
            const uint32_t psel = u == 0 ? pb[0] : (u == 1 ? pb[1] : (u == 2 ? pb[2] : pb[3]));
            load_to_lds4(lds0 + (uint32_t)S::fip_off + (uint32_t)(wave * 2 + i) * 256u, Ip,
                         psel + (uint32_t)((row * g.ipw + iw) * 4));
        }
    };
    // Eq. 3 for the panel.  A lane forms the 4 mask words of one row under one 128-column unit: it takes the row's
    // I_p word(s), picks the first two set ranks without looking at memory (rank 64 = the zero row when there are
    // fewer), and ORs their I_z pieces, both reads in flight together; rows with more set ranks (few: the factors
    // are sparse) loop over the rest.
    auto decode_panel = [&](int panel) {
        const int row = tid >> 2, u = tid & 3;
        unsigned char *out = Mt + (panel & 1) * MT_BYTES + row * MT_ROW + u * 16;
        const uint32_t *fp = Fip + (row * PANEL_UNITS + u) * (HALF ? 4 : 2);
        const uint32_t *fz = Fz + 4 * u;
        uint4 a;
        if constexpr (HALF) {
            // the unit's two halves, each from the I_p word(s) and the two I_z words of its own tile
            uint2 hv[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                unsigned long long sel = (unsigned long long)fp[2 * h];
                if (g.ipw > 1) sel |= (unsigned long long)fp[2 * h + 1] << 32;
                const uint32_t *fh = fz + 2 * h;
                const int l0 = sel ? __builtin_ctzll(sel) : FAST_MAX_K;
                sel &= sel - 1ull;
                const int l1 = sel ? __builtin_ctzll(sel) : FAST_MAX_K;
                sel &= sel - 1ull;
                const uint2 z0 = *reinterpret_cast<const uint2 *>(fh + l0 * PANEL_WORDS);
                const uint2 z1 = *reinterpret_cast<const uint2 *>(fh + l1 * PANEL_WORDS);
                uint2 o = make_uint2(z0.x | z1.x, z0.y | z1.y);
                while (sel) {
                    const int le = __builtin_ctzll(sel);
                    sel &= sel - 1ull;
                    const uint2 ze = *reinterpret_cast<const uint2 *>(fh + le * PANEL_WORDS);
                    o.x |= ze.x;
                    o.y |= ze.y;
                }
                hv[h] = o;
            }
            a = make_uint4(hv[0].x, hv[0].y, hv[1].x, hv[1].y);
        } else if (g.ipw == 1) { // ranks up to 32: one word
            uint32_t sel = fp[0];
            const int l0 = sel ? __builtin_ctz(sel) : FAST_MAX_K;
            sel &= sel - 1u;
            const int l1 = sel ? __builtin_ctz(sel) : FAST_MAX_K;
            sel &= sel - 1u;
            const uint4 z0 = *reinterpret_cast<const uint4 *>(fz + l0 * PANEL_WORDS);
            const uint4 z1 = *reinterpret_cast<const uint4 *>(fz + l1 * PANEL_WORDS);
            a = make_uint4(z0.x | z1.x, z0.y | z1.y, z0.z | z1.z, z0.w | z1.w);
            while (sel) {
                const int le = __builtin_ctz(sel);
                sel &= sel - 1u;
                const uint4 ze = *reinterpret_cast<const uint4 *>(fz + le * PANEL_WORDS);
                a.x |= ze.x;
                a.y |= ze.y;
                a.z |= ze.z;
                a.w |= ze.w;
            }
        } else {
            unsigned long long sel = (unsigned long long)fp[0] | ((unsigned long long)fp[1] << 32);
            const int l0 = sel ? __builtin_ctzll(sel) : FAST_MAX_K;
            sel &= sel - 1ull;
            const int l1 = sel ? __builtin_ctzll(sel) : FAST_MAX_K;
            sel &= sel - 1ull;
            const uint4 z0 = *reinterpret_cast<const uint4 *>(fz + l0 * PANEL_WORDS);
            const uint4 z1 = *reinterpret_cast<const uint4 *>(fz + l1 * PANEL_WORDS);
            a = make_uint4(z0.x | z1.x, z0.y | z1.y, z0.z | z1.z, z0.w | z1.w);
            while (sel) {
                const int le = __builtin_ctzll(sel);
                sel &= sel - 1ull;
                const uint4 ze = *reinterpret_cast<const uint4 *>(fz + le * PANEL_WORDS);
                a.x |= ze.x;
                a.y |= ze.y;
                a.z |= ze.z;
                a.w |= ze.w;
            }
        }
        *reinterpret_cast<uint2 *>(out) = make_uint2(a.x, a.y);
        *reinterpret_cast<uint2 *>(out + 8) = make_uint2(a.z, a.w);
        if constexpr (EMIT) {
            // units past the end of this workgroup's reduction range were formed from stand-in factors: not stored
            const int unit = kbeg / 128 + panel * PANEL_UNITS + u;
            if (ni == 0 && unit * 128 < kend) mask_out[(m0 + row) * mask_pitch16 + unit] = a;
        }
    };

    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
// nothing crosses this line when the compiler orders the instructions
#define LRBI_SB() __builtin_amdgcn_sched_barrier(0)
// workgroup barrier without the compiler's own "wait for every outstanding memory operation" in front of it (that
// wait would drain the slabs in flight); what has to be complete is waited for explicitly
#define LRBI_BARRIER()                                             \
    do {                                                           \
        LRBI_SB();                                                 \
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); /* this wavefront's LDS writes have landed */ \
        __builtin_amdgcn_s_barrier();                              \
        LRBI_SB();                                                 \
    } while (0)

    // ---- prologue: the factor slices of panel 0 first, then slabs 0 .. NS - 2; the panel is decoded as soon as the
    // factor slices are in (the slabs issued behind them stay in flight), and slab 0 is waited for after that
    if (tid < PANEL_WORDS) Fz[FAST_MAX_K * PANEL_WORDS + tid] = 0u;
    load_factors();
    constexpr int kProloguePieces = SPREAD ? (NS - 2) * 4 + 2 : (NS - 1) * 4; // slab copies of this wavefront behind them
    static_for<NS - 1>([&](auto sc) {
        constexpr int st = decltype(sc)::value;
        const int sl0 = st < last ? st : last;
        issue_piece(sl0, st, I0{});
        issue_piece(sl0, st, I1{});
        if constexpr (!(SPREAD && st == NS - 2)) { // SPREAD: the last slab's other half follows in the first iteration
            issue_piece(sl0, st, I2{});
            issue_piece(sl0, st, I3{});
        }
    });
    wait_loads<kProloguePieces>();
    __syncthreads();
    decode_panel(0);
    // slab 0 (EMIT: the panel's mask store is one more, younger, entry of the same in-order count)
    wait_loads<kProloguePieces - 4 + (EMIT ? 1 : 0)>();
    __syncthreads();
    // entry state of the loop: X operands of this wavefront's first step, its W operand masked, the second read
    uint32_t mcur = my_bytes(fetch_mask(0));
    read_w(0, I0{}, I0{});
    read_w(0, I0{}, I1{});
    read_x(0, I0{}, I0{});
    read_x(0, I0{}, I1{});
    read_x(0, I0{}, I2{});
    read_x(0, I0{}, I3{});
    {
        const uint32_t y = mask_lo(I0{}, I0{}, mcur);
        mask_hi(I0{}, I0{}, y);
    }

    // ---- main loop, unrolled by NS so that the stage of a slab is a compile-time constant.
    // Iteration s multiplies slab s out of stage s % NS: each wavefront its two 16-column steps.  After the
    // first step every wavefront waits until its own pieces of slab s + 1 have landed; the barrier makes the
    // whole slab visible and tells that nobody reads slab s - 1 any more; the second step then runs next to the
    // loads of slab s + NS - 1 into the stage slab s - 1 occupied and to the reads of slab s + 1's operands.
    for (int s0 = 0; s0 < nslabs; s0 += NS) {
        static_for<NS>([&](auto sc) {
            constexpr int st = decltype(sc)::value;       // stage of slab s
            constexpr int st1 = (st + 1) % NS;            // stage of slab s + 1
            constexpr int stn = (st + NS - 1) % NS;       // stage of slab s - 1 = stage of slab s + NS - 1
            constexpr int stp = (st + NS - 2) % NS;       // stage of slab s - 2 = stage of slab s + NS - 2
            using Par = std::integral_constant<int, st & 1>;        // register set of slab s's W operands
            using Nxt = std::integral_constant<int, (st & 1) ^ 1>;  // ... of slab s + 1's
            const int s = s0 + st;
            if (s < nslabs) {
                uint32_t y;
                u32x2 mk;
                const int sl = s + NS - 1 < last ? s + NS - 1 : last;
                const int sp = s + NS - 2 < last ? s + NS - 2 : last;
                // first step
                mma(Par{}, I0{}, I0{}); read_x(st, I1{}, I0{}); y = mask_lo(Par{}, I1{}, mcur);
                mma(Par{}, I0{}, I1{}); read_x(st, I1{}, I1{}); mask_hi(Par{}, I1{}, y);
                if constexpr (SPREAD) issue_piece(sp, stp, I2{});
                mma(Par{}, I0{}, I2{}); read_x(st, I1{}, I2{});
                mk = fetch_mask(s + 1 < last ? s + 1 : last); // mask bytes of the next slab
                mma(Par{}, I0{}, I3{}); read_x(st, I1{}, I3{});
                if constexpr (SPREAD) issue_piece(sp, stp, I3{});
                // factor slices of the next panel, requested at the panel's first slab: they have landed, for
                // every wavefront, behind the next iteration's wait and barrier
                const int ps = s % PANEL_SLABS;
                const int np = s / PANEL_SLABS + 1;
                if (ps == 0 && np < npanels) load_factors();
                // slab s + 1 has landed (four younger loads may still be in flight with four stages; EMIT: and the mask
                // store of the panel that the previous iteration turned into mask bytes)
                if (EMIT && ps == 3 && np < npanels) wait_loads<(NS - 3) * 4 + 1>();
                else wait_loads<(NS - 3) * 4>();
                LRBI_BARRIER();
                // second step
                mma(Par{}, I1{}, I0{}); read_x(st1, I0{}, I0{}); read_w(st1, Nxt{}, I0{}); read_w(st1, Nxt{}, I1{});
                issue_piece(sl, stn, I0{});
                mma(Par{}, I1{}, I1{}); read_x(st1, I0{}, I1{}); mcur = my_bytes(mk);
                issue_piece(sl, stn, I1{});
                mma(Par{}, I1{}, I2{}); read_x(st1, I0{}, I2{}); y = mask_lo(Nxt{}, I0{}, mcur);
                if constexpr (!SPREAD) issue_piece(sl, stn, I2{});
                mma(Par{}, I1{}, I3{}); read_x(st1, I0{}, I3{}); mask_hi(Nxt{}, I0{}, y);
                if constexpr (!SPREAD) issue_piece(sl, stn, I3{});
                // mask of the next panel, turned into mask bytes at the panel's slab 2; the first read of the new
                // mask bytes is at slab 7
                if (ps == 2 && np < npanels) decode_panel(np);
            }
        });
    }
#undef LRBI_SB
#undef LRBI_BARRIER
    wait_loads<0>(); // nothing may still be landing in LDS
    __syncthreads();

    // ---- the two halves of the reduction range: wavefronts 4 .. 7 hand their sums to wavefronts 0 .. 3 through LDS
    {
        float *red = (float *)smem + (size_t)wq * (FN * 16 * 64) + lane; // [wq][a][v][lane]; the stages are dead now
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

    // ---- epilogue: lane holds, per 32-column block a, columns n = 8 (v / 4) + 4 lg + (v % 4) of output row l32.
    // The wavefront's 32 x 128 block goes through its own strip of LDS (rounded to the output type first, or as
    // fp32 for a partial plane) and leaves as 16-byte pieces of whole rows.
    const int64_t row0 = m0 + wq * 32;
    if (SPLIT) {
        constexpr int RS = 128 * 4 + 16; // bytes per staged row
        unsigned char *strip = smem + 65536 + wq * (32 * RS);
#pragma unroll
        for (int a = 0; a < FN; ++a)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4)
                *reinterpret_cast<float4 *>(strip + l32 * RS + (a * 32 + 8 * v4 + 4 * lg) * 4) =
                    make_float4(acc[a][4 * v4 + 0], acc[a][4 * v4 + 1], acc[a][4 * v4 + 2], acc[a][4 * v4 + 3]);
        // (the strip is private to the wavefront: its own LDS operations complete in order)
#pragma unroll
        for (int i = 0; i < 16; ++i) { // 2 rows per instruction: 32 lanes x 16 bytes per row
            const int rr = 2 * i + lg, col = n0 + 4 * l32;
            const float4 o = *reinterpret_cast<const float4 *>(strip + rr * RS + l32 * 16);
            // (non-temporal: the planes are read once, by another kernel; measured 0.6-0.8 us of the call on a
            // 4096 x 9216 matrix at 128 columns, most of it the end of this kernel)
            typedef float nt_f4 __attribute__((ext_vector_type(4)));
            nt_f4 ov = {o.x, o.y, o.z, o.w};
            if (col < ldp) __builtin_nontemporal_store(ov, reinterpret_cast<nt_f4 *>(P + ((int64_t)slice * g.m + row0 + rr) * ldp + col));
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
        const bool y16 = y_vec_ok && (((uintptr_t)Y & 15) == 0) && (ldy % 8 == 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) { // 4 rows per instruction: 16 lanes x 16 bytes per row
            const int rr = 4 * i + rq, col = n0 + 8 * l16;
            const uint2 lo = *reinterpret_cast<const uint2 *>(strip + rr * RS + l16 * 16);
            const uint2 hi = *reinterpret_cast<const uint2 *>(strip + rr * RS + l16 * 16 + 8);
            uint16_t *yp = Y + (row0 + rr) * ldy + col;
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

// tile shapes the pipelined kernel's blocking lines up with: tile rows in blocks of 128, tile widths a multiple of
// 128, or of 64 (gathered per half unit) when the row length is still a multiple of 128
bool pipe_shape_ok(const Geom &g)
{
    if ((g.r % PIPE_BM) != 0 || g.k > FAST_MAX_K || g.ragged) return false;
    return (g.c % 128) == 0 || ((g.c % 64) == 0 && (g.n % 128) == 0);
}

// true when the pipelined kernel serves this call: aligned tile shapes, X readable in 16-byte pieces, offsets
// that fit the kernel's 32-bit per-lane byte offsets
bool pipe_ok(const Geom &g, const void *dIz, const void *dX, int64_t ldw, int64_t ldx, int64_t N)
{
    if (!pipe_shape_ok(g)) return false;
    if ((((uintptr_t)dX & 15) != 0) || (ldx % 8 != 0) || (N % 8 != 0) || N < 8) return false;
    if (((uintptr_t)dIz & 15) != 0) return false; // the I_z slices are fetched in 16-byte pieces
    if (ldw > (1 << 22) || ldx > (1 << 22)) return false;
    // byte offsets into the packed factors are kept in 32 bits
    const int64_t tiles = (int64_t)g.tile_rows * g.tile_cols;
    if (tiles * g.k * g.izw * 4 >= (int64_t)1 << 31 || tiles * g.r * g.ipw * 4 >= (int64_t)1 << 31) return false;
    return true;
}

template <typename Tag, int NS, bool SPREAD, bool CONV, bool EMIT = false, bool HALF = false>
static int launch_pipe_t(const Geom &g, const MfmaPlan &plan, const void *dW, int64_t ldw, const uint32_t *dIp,
                         const uint32_t *dIz, const void *dX, int64_t ldx, int64_t N, void *dY, int64_t ldy,
                         void *dWorkspace, const ConvGeom &cg, hipStream_t stream, MaskOut mo = {nullptr, 0})
{
    const int64_t mblocks = g.m / PIPE_BM;
    const int64_t nblocks = (N + PIPE_BN - 1) / PIPE_BN;
    const int64_t blocks = mblocks * nblocks * plan.splitk;
    if (blocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    const bool split = plan.splitk > 1 || plan.planes_only;
    const int y_vec_ok = (((uintptr_t)dY & 7) == 0) && (ldy % 4 == 0);
    const int xcd_remap = (blocks % 8 == 0) ? 1 : 0;
    const int64_t ldp = (N + 3) / 4 * 4;
    const size_t smem = SmemDma<NS, HALF>::bytes;
    auto kern = split ? mfma_gemm_pipe_kernel<Tag, NS, SPREAD, true, CONV, EMIT, HALF>
                      : mfma_gemm_pipe_kernel<Tag, NS, SPREAD, false, CONV, EMIT, HALF>;
    LRBI_SET_MAX_LDS(kern, smem);
    LRBI_LAUNCH(kern, dim3((unsigned)blocks), dim3(PIPE_THREADS), smem, stream, g, (const uint16_t *)dW, ldw, dIp, dIz,
                (const uint16_t *)dX, ldx, (int)N, (uint16_t *)dY, ldy, (float *)dWorkspace, ldp, (int)mblocks,
                (int)nblocks, plan.kper, xcd_remap, y_vec_ok, cg, (uint4 *)mo.ptr, mo.pitch16);
    return LRBI_OK;
}

// variant 0, 1: a slab's loads issued in a burst right after the barrier (longest time to land: weights streaming
// from HBM); 2: loads spread evenly over the iteration (operands coming from L2).
// The caller adds the partial planes when the plan is split.
int launch_pipe_gemm(const Geom &g, const MfmaPlan &plan, lrbi_dtype dt, int variant, const void *dW, int64_t ldw,
                     const uint32_t *dIp, const uint32_t *dIz, const void *dX, int64_t ldx, int64_t N, void *dY,
                     int64_t ldy, void *dWorkspace, hipStream_t stream, MaskOut mo)
{
    const ConvGeom none = {0, 0, 0};
    if (g.c % 128 != 0) { // half units: one variant per dtype (loads spread over the iteration), with or without the mask
#define LRBI_PIPE_ARGS g, plan, dW, ldw, dIp, dIz, dX, ldx, N, dY, ldy, dWorkspace, none, stream, mo
        if (dt == LRBI_F16)
            return mo.ptr ? launch_pipe_t<F16Tag, 4, true, false, true, true>(LRBI_PIPE_ARGS)
                          : launch_pipe_t<F16Tag, 4, true, false, false, true>(LRBI_PIPE_ARGS);
        if (dt == LRBI_BF16)
            return mo.ptr ? launch_pipe_t<BF16Tag, 4, true, false, true, true>(LRBI_PIPE_ARGS)
                          : launch_pipe_t<BF16Tag, 4, true, false, false, true>(LRBI_PIPE_ARGS);
#undef LRBI_PIPE_ARGS
        return LRBI_ERR_DTYPE;
    }
    if (mo.ptr) { // the mask as a by-product: one variant per dtype (loads spread over the iteration)
        if (dt == LRBI_F16)
            return launch_pipe_t<F16Tag, 4, true, false, true>(g, plan, dW, ldw, dIp, dIz, dX, ldx, N, dY, ldy, dWorkspace,
                                                               none, stream, mo);
        if (dt == LRBI_BF16)
            return launch_pipe_t<BF16Tag, 4, true, false, true>(g, plan, dW, ldw, dIp, dIz, dX, ldx, N, dY, ldy, dWorkspace,
                                                                none, stream, mo);
        return LRBI_ERR_DTYPE;
    }
#define LRBI_PIPE_ARGS g, plan, dW, ldw, dIp, dIz, dX, ldx, N, dY, ldy, dWorkspace, none, stream
    if (dt == LRBI_F16) {
        if (variant <= 1) return launch_pipe_t<F16Tag, 4, false, false>(LRBI_PIPE_ARGS);
        return launch_pipe_t<F16Tag, 4, true, false>(LRBI_PIPE_ARGS);
    }
    if (dt == LRBI_BF16) {
        if (variant <= 1) return launch_pipe_t<BF16Tag, 4, false, false>(LRBI_PIPE_ARGS);
        return launch_pipe_t<BF16Tag, 4, true, false>(LRBI_PIPE_ARGS);
    }
#undef LRBI_PIPE_ARGS
    return LRBI_ERR_DTYPE;
}

// true when the pipelined kernel serves the convolution form: aligned tile shapes, 64 channels or a multiple,
// the weight matrix's 9 * cin columns, offsets that fit the kernel's 32-bit per-lane byte offsets
bool pipe_conv_ok(const Geom &g, const ConvGeom &cg, int64_t batch, const void *dIz, const void *dAct, int64_t ldw)
{
    if ((g.c % 128) != 0 || (g.r % PIPE_BM) != 0 || g.k > FAST_MAX_K || g.ragged) return false;
    if (cg.cin <= 0 || cg.cin % 64 != 0 || cg.H <= 0 || cg.Wd <= 0 || batch <= 0) return false;
    if (g.n != (int64_t)9 * cg.cin) return false;
    if ((((uintptr_t)dAct | (uintptr_t)dIz) & 15) != 0) return false;
    if (ldw > (1 << 22)) return false;
    const int64_t act_bytes = batch * (cg.H + 2) * (int64_t)(cg.Wd + 2) * cg.cin * 2;
    if (act_bytes >= ((int64_t)1 << 32) || batch * cg.H * (int64_t)cg.Wd > 0x7FFFFF00) return false;
    const int64_t tiles = (int64_t)g.tile_rows * g.tile_cols;
    if (tiles * g.k * g.izw * 4 >= (int64_t)1 << 31 || tiles * g.r * g.ipw * 4 >= (int64_t)1 << 31) return false;
    return true;
}

// the convolution form (operands from L2: loads spread over the iteration); N = batch * H * Wd columns
int launch_pipe_conv(const Geom &g, const MfmaPlan &plan, lrbi_dtype dt, const ConvGeom &cg, const void *dW, int64_t ldw,
                     const uint32_t *dIp, const uint32_t *dIz, const void *dAct, int64_t N, void *dY, int64_t ldy,
                     void *dWorkspace, hipStream_t stream)
{
    if (dt == LRBI_F16)
        return launch_pipe_t<F16Tag, 4, true, true>(g, plan, dW, ldw, dIp, dIz, dAct, 0, N, dY, ldy, dWorkspace, cg, stream);
    if (dt == LRBI_BF16)
        return launch_pipe_t<BF16Tag, 4, true, true>(g, plan, dW, ldw, dIp, dIz, dAct, 0, N, dY, ldy, dWorkspace, cg, stream);
    return LRBI_ERR_DTYPE;
}

} // namespace lrbi
