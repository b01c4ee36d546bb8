// Mask decode to HBM: I_a,t = I_p,t (x) I_z,t for every tile (Eq. 3, Sec. 3.1),
// written as the one-bit-per-weight binary index form (Fig. 1).
//
// The kernel should be bound by HBM stores, so the integer work per 32-bit mask
// word is kept small and every load is taken off the path of the stores:
//   * a work item is a band of rows of one tile row times a span of columns
//     (at most 64 16-byte pieces, i.e. one wavefront across);
//   * for an item the workgroup holds in LDS (a) the "Z table": the I_z rows of
//     every tile under the span, shifted to their absolute bit position in the
//     mask row (Z[l] is the concatenation over tiles of row l of each tile's
//     I_z), so tile boundaries that fall inside a word are resolved once per
//     item and not once per mask row, and (b) the I_p words of the band's rows;
//   * a lane produces 128 mask bits at a time: it walks the SET bits of the I_p
//     word (about k*p of them) and ORs the matching 16-byte pieces of Z;
//   * consecutive lanes hold consecutive 16-byte pieces of one mask row, so the
//     stores are full-width and coalesced.
// Two kernels share that code.  The one-shot kernel takes one item per
// workgroup (small masks).  The streaming kernel is persistent: one workgroup of
// 1024 lanes per compute unit walks many items with the two LDS tables double
// buffered, and the global loads of the next item's factors are in flight while
// the current item's rows are decoded and stored, so stores never wait for loads.
#include <stdlib.h>

#include "lrbi_internal.hpp"
#include "lrbi_lds_dma.hpp"

namespace lrbi {

static constexpr int kDecodeThreads = 256;
// masks too small for the streaming kernel: the span of an item is halved (down to 4 pieces = 64 bytes of a row)
// until there are this many items.  Measured on 4096 x 9216 with 576-column tiles, rank 32 / 64: 18.3 / 18.9 us at the
// widest span (288 items), 9.7 / 10.6 us with 512; 1024 and more cost the 300-column tiles of a 6000 x 3000 mask 3 us.
static constexpr int kSmallMaskItems = 512;
static constexpr int kSmallMaskMinShift = 2;
static constexpr int kStreamThreads = 1024;
static constexpr int kZTableBudgetBytes = 32 * 1024; // (k + 1) * span pieces * 16 bytes
static constexpr int kIpBudgetBytes = 12 * 1024;     // tiles under the span * (rows + 1) * ipw * 4 bytes
static constexpr int kMaxZPerLane = kZTableBudgetBytes / 16 / kStreamThreads;  // 16-byte pieces per lane and item
static constexpr int kMaxIpPerLane = kIpBudgetBytes / 4 / kStreamThreads;      // words per lane and item

// Fallback without LDS: every lane decodes its four words straight from global memory.
__global__ __launch_bounds__(kDecodeThreads) void decode_generic_kernel(Geom g, const uint32_t *__restrict__ Ip,
                                                                        const uint32_t *__restrict__ Iz,
                                                                        uint4 *__restrict__ mask,
                                                                        int64_t pitch16, int chunks)
{
    const int64_t e = (int64_t)blockIdx.x * kDecodeThreads + threadIdx.x;
    if (e >= g.m * (int64_t)chunks) return;
    const int64_t row = e / chunks;
    const int q = (int)(e - row * chunks);
    const int ti = (int)(row / g.r);
    const int il = (int)(row - (int64_t)ti * g.r);
    uint4 out;
    out.x = decode_word(g, Ip, Iz, ti, il, 4 * q + 0);
    out.y = decode_word(g, Ip, Iz, ti, il, 4 * q + 1);
    out.z = decode_word(g, Ip, Iz, ti, il, 4 * q + 2);
    out.w = decode_word(g, Ip, Iz, ti, il, 4 * q + 3);
    mask[row * pitch16 + q] = out;
}

// One 32-bit word of Z[l] at absolute word index w of the mask row (tile row ti); any c.
__device__ __forceinline__ uint32_t ztable_word(const Geom &g, const uint32_t *__restrict__ Iz, int ti, int l, int w)
{
    const int64_t j0 = (int64_t)w * 32;
    if (j0 >= g.n) return 0u;
    const int64_t j1 = (j0 + 32 < g.n) ? j0 + 32 : g.n;
    int tj = (int)(j0 / g.c);
    uint32_t acc = 0u;
    for (int64_t tbeg = (int64_t)tj * g.c; tbeg < j1; tbeg += g.c, ++tj) {
        const int64_t t = (int64_t)ti * g.tile_cols + tj;
        const int off = (int)(j0 - tbeg);
        const uint32_t valid = bit_range(off < 0 ? -off : 0, (g.c - off < 32) ? g.c - off : 32);
        acc |= iz_window(Iz + (t * g.k + l) * g.izw, g.izw, off) & valid;
    }
    return acc;
}

__device__ __forceinline__ uint4 or4(uint4 a, uint4 b)
{
    return make_uint4(a.x | b.x, a.y | b.y, a.z | b.z, a.w | b.w);
}

// OR of the Z-table pieces selected by the set bits of one I_p word.  The first two reads are
// issued back to back (their LDS latencies overlap); `zero_row` is an all-zero row of the table
// that absorbs the slots of words with fewer set bits.  Leftover bits take the loop.
__device__ __forceinline__ uint4 or_selected(uint4 acc, uint32_t sel, int l_base, const uint4 *__restrict__ Zq,
                                             int zshift, int zero_row)
{
    int l0 = zero_row, l1 = zero_row;
    if (sel) { l0 = __builtin_ctz(sel) + l_base; sel &= sel - 1u; }
    if (sel) { l1 = __builtin_ctz(sel) + l_base; sel &= sel - 1u; }
    const uint4 z0 = Zq[l0 << zshift], z1 = Zq[l1 << zshift];
    acc.x |= z0.x | z1.x;
    acc.y |= z0.y | z1.y;
    acc.z |= z0.z | z1.z;
    acc.w |= z0.w | z1.w;
    while (sel) {
        const int l = __builtin_ctz(sel) + l_base;
        sel &= sel - 1u;
        acc = or4(acc, Zq[l << zshift]);
    }
    return acc;
}

// Launch-time constants of the item decomposition.
struct DecodePlan {
    int chunks;             // 16-byte pieces per mask row
    int span_chunks;        // pieces per span (a power of two, so the table's row stride is a shift)
    int zshift;             // log2(span_chunks)
    int spans;              // spans per row
    int rows_per_band;
    int bands_per_tile_row;
    int tx_log2;            // lanes across a span = 1 << tx_log2
    int span_tiles;         // upper bound of tiles under a span
    int iz16;               // I_z base pointer is 16-byte aligned
    int64_t pitch16;        // mask pitch in 16-byte pieces
    int64_t items;          // spans * tile_rows * bands_per_tile_row
};

// Geometry of one item.
struct Item {
    int ti, row_lo, nrows, q_lo, nq, tj_first, ntiles;
};
__device__ __forceinline__ Item make_item(const Geom &g, const DecodePlan &p, int64_t id)
{
    Item it;
    const int span = (int)(id % p.spans);
    const int64_t band = id / p.spans;
    it.ti = (int)(band / p.bands_per_tile_row);
    it.row_lo = (int)(band - (int64_t)it.ti * p.bands_per_tile_row) * p.rows_per_band;
    const int row_hi = (it.row_lo + p.rows_per_band < g.r) ? it.row_lo + p.rows_per_band : g.r;
    it.nrows = row_hi - it.row_lo;
    it.q_lo = span * p.span_chunks;
    it.nq = (it.q_lo + p.span_chunks <= p.chunks) ? p.span_chunks : p.chunks - it.q_lo;
    it.tj_first = (int)(((int64_t)it.q_lo * 128) / g.c);
    const int64_t last_col = ((int64_t)(it.q_lo + it.nq) * 128 < g.n ? (int64_t)(it.q_lo + it.nq) * 128 : g.n) - 1;
    it.ntiles = (int)(last_col / g.c) - it.tj_first + 1;
    return it;
}

// 16-byte piece (l, q) of the item's Z table, straight from the packed I_z.
// ALIGNED (c % 128 == 0): the piece lies inside one tile.
template <bool ALIGNED>
__device__ __forceinline__ uint4 z_piece(const Geom &g, const DecodePlan &p, const Item &it,
                                         const uint32_t *__restrict__ Iz, int l, int q)
{
    const int Q = it.q_lo + q;
    if (ALIGNED) {
        const int pieces_per_tile = g.c >> 7;
        const int tj = Q / pieces_per_tile;
        const uint32_t *src =
            Iz + (((int64_t)it.ti * g.tile_cols + tj) * g.k + l) * (int64_t)g.izw + 4 * (Q - tj * pieces_per_tile);
        if (p.iz16) return *reinterpret_cast<const uint4 *>(src);
        return make_uint4(src[0], src[1], src[2], src[3]);
    }
    uint4 v;
    v.x = ztable_word(g, Iz, it.ti, l, 4 * Q + 0);
    v.y = ztable_word(g, Iz, it.ti, l, 4 * Q + 1);
    v.z = ztable_word(g, Iz, it.ti, l, 4 * Q + 2);
    v.w = ztable_word(g, Iz, it.ti, l, 4 * Q + 3);
    return v;
}

// Decode and store the rows of one item from its LDS tables.
//   Z   [k + 1][span_chunks] (last row zero)
//   IpL [tiles under the span][rows_per_band + 1][ipw]  (the + 1 keeps tiles on different banks)
// Lane layout: TX = 1 << tx_log2 lanes across the span's pieces, TY = nthreads / TX rows at a time.
template <bool ALIGNED>
__device__ __forceinline__ void decode_item_rows(const Geom &g, const DecodePlan &p, const Item &it,
                                                 const uint4 *__restrict__ Z, const uint32_t *__restrict__ IpL,
                                                 uint4 *__restrict__ mask, int nthreads)
{
    const int TX = 1 << p.tx_log2;
    const int tx = threadIdx.x & (TX - 1);
    const int ty = threadIdx.x >> p.tx_log2;
    const int TY = nthreads >> p.tx_log2;
    const int zero_row = g.k;
    const int ip_rows = p.rows_per_band + 1;
    for (int q = tx; q < it.nq; q += TX) {
        const int Q = it.q_lo + q;           // absolute 16-byte piece of the mask row
        const int64_t cb = (int64_t)Q * 128; // first column of the piece
        const uint4 *Zq = Z + q;
        uint4 *out = mask + ((int64_t)it.ti * g.r + it.row_lo + ty) * p.pitch16 + Q;
        const int64_t out_step = (int64_t)TY * p.pitch16;
        if (ALIGNED) {
            const int tl = (int)(cb / g.c) - it.tj_first;
            const uint32_t *ipr = IpL + (tl * ip_rows + ty) * g.ipw;
            const int ip_step = TY * g.ipw;
            for (int i = ty; i < it.nrows; i += TY, ipr += ip_step, out += out_step) {
                uint4 acc = make_uint4(0u, 0u, 0u, 0u);
                for (int iw = 0; iw < g.ipw; ++iw) acc = or_selected(acc, ipr[iw], 32 * iw, Zq, p.zshift, zero_row);
                *out = acc;
            }
        } else {
            const int64_t ce = (cb + 128 < g.n) ? cb + 128 : g.n;
            const int tj_lo = (int)(cb / g.c);
            for (int i = ty; i < it.nrows; i += TY, out += out_step) {
                uint4 acc = make_uint4(0u, 0u, 0u, 0u);
                int tj = tj_lo;
                for (int64_t tbeg = (int64_t)tj * g.c; tbeg < ce; tbeg += g.c, ++tj) {
                    const uint32_t *ipr = IpL + ((tj - it.tj_first) * ip_rows + i) * g.ipw;
                    // bits of this piece that belong to tile tj
                    const int lo = (int)((tbeg > cb ? tbeg : cb) - cb);
                    const int hi = (int)((tbeg + g.c < ce ? tbeg + g.c : ce) - cb);
                    uint4 tm;
                    tm.x = bit_range(lo < 0 ? 0 : lo, hi > 32 ? 32 : hi);
                    tm.y = bit_range(lo - 32 < 0 ? 0 : lo - 32, hi - 32 > 32 ? 32 : hi - 32);
                    tm.z = bit_range(lo - 64 < 0 ? 0 : lo - 64, hi - 64 > 32 ? 32 : hi - 64);
                    tm.w = bit_range(lo - 96 < 0 ? 0 : lo - 96, hi - 96 > 32 ? 32 : hi - 96);
                    uint4 v = make_uint4(0u, 0u, 0u, 0u);
                    for (int iw = 0; iw < g.ipw; ++iw) v = or_selected(v, ipr[iw], 32 * iw, Zq, p.zshift, zero_row);
                    acc.x |= v.x & tm.x;
                    acc.y |= v.y & tm.y;
                    acc.z |= v.z & tm.z;
                    acc.w |= v.w & tm.w;
                }
                *out = acc;
            }
        }
    }
}

// One-shot kernel: one item per workgroup of 256 lanes.
template <bool ALIGNED>
__global__ __launch_bounds__(kDecodeThreads) void decode_ztable_kernel(Geom g, DecodePlan p,
                                                                       const uint32_t *__restrict__ Ip,
                                                                       const uint32_t *__restrict__ Iz,
                                                                       uint4 *__restrict__ mask)
{
    extern __shared__ uint4 lrbi_dyn_smem[];
    uint4 *Z = lrbi_dyn_smem; // [k + 1][span_chunks]
    uint32_t *IpL = (uint32_t *)(Z + (size_t)(g.k + 1) * p.span_chunks);
    const Item it = make_item(g, p, blockIdx.x);
    const int TX = 1 << p.tx_log2;
    const int tx = threadIdx.x & (TX - 1);
    const int ty = threadIdx.x >> p.tx_log2;
    const int TY = kDecodeThreads >> p.tx_log2;
    const int ip_rows = p.rows_per_band + 1;

    // Loads go out in batches before any is consumed (a few memory round trips per workgroup).
    constexpr int kBatch = 8;
    for (int w = threadIdx.x; w < 4 * p.span_chunks; w += kDecodeThreads) ((uint32_t *)Z)[g.k * (4 * p.span_chunks) + w] = 0u;
    for (int q = tx; q < it.nq; q += TX) {
        for (int l0 = ty; l0 < g.k; l0 += TY * kBatch) {
            uint4 tmp[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int l = l0 + TY * j;
                tmp[j] = make_uint4(0u, 0u, 0u, 0u);
                if (l < g.k) tmp[j] = z_piece<ALIGNED>(g, p, it, Iz, l, q);
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int l = l0 + TY * j;
                if (l < g.k) Z[l * p.span_chunks + q] = tmp[j];
            }
        }
    }
    // I_p words of the band: per tile a contiguous run of nrows * ipw words; the flat index walks
    // (tile, word) without divisions
    const int per_tile = it.nrows * g.ipw;
    int tl = 0, e = threadIdx.x;
    while (e >= per_tile && tl < it.ntiles) { e -= per_tile; ++tl; }
    while (tl < it.ntiles) {
        uint32_t tmp[kBatch];
        int dst[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            tmp[j] = 0u;
            dst[j] = -1;
            if (tl < it.ntiles) {
                const int64_t t = (int64_t)it.ti * g.tile_cols + it.tj_first + tl;
                tmp[j] = Ip[(t * g.r + it.row_lo) * g.ipw + e];
                dst[j] = (tl * ip_rows) * g.ipw + e;
                e += kDecodeThreads;
                while (e >= per_tile && tl < it.ntiles) { e -= per_tile; ++tl; }
            }
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j)
            if (dst[j] >= 0) IpL[dst[j]] = tmp[j];
    }
    __syncthreads();
    decode_item_rows<ALIGNED>(g, p, it, Z, IpL, mask, kDecodeThreads);
}

// Streaming kernel: persistent workgroups of 1024 lanes, items id = blockIdx.x, + gridDim.x, ...
// LDS holds two copies of (Z, IpL).  While item j is decoded and stored from one copy, the loads
// of item j + 1 are in flight into registers; they are written to the other copy afterwards.
template <bool ALIGNED>
__global__ __launch_bounds__(kStreamThreads) void decode_stream_kernel(Geom g, DecodePlan p,
                                                                       const uint32_t *__restrict__ Ip,
                                                                       const uint32_t *__restrict__ Iz,
                                                                       uint4 *__restrict__ mask)
{
    extern __shared__ uint4 lrbi_dyn_smem[];
    const int z_pieces = (g.k + 1) * p.span_chunks;
    const int ip_rows = p.rows_per_band + 1;
    const int ip_words = p.span_tiles * ip_rows * g.ipw;
    const int buf_pieces = z_pieces + (ip_words + 3) / 4;
    // buffer b: Z at lrbi_dyn_smem + b * buf_pieces, IpL right behind it (kept as offsets from the
    // LDS symbol so that the compiler emits LDS instructions, not generic ones)
#define LRBI_ZB(b) (lrbi_dyn_smem + (b) * buf_pieces)
#define LRBI_IPB(b) ((uint32_t *)(lrbi_dyn_smem + (b) * buf_pieces + z_pieces))

    uint4 zreg[kMaxZPerLane];
    uint32_t ipreg[kMaxIpPerLane];
    int ipdst[kMaxIpPerLane];

    // the zero rows never change
    for (int w = threadIdx.x; w < 2 * p.span_chunks; w += kStreamThreads) {
        const int b = w / p.span_chunks, q = w - b * p.span_chunks;
        LRBI_ZB(b)[g.k * p.span_chunks + q] = make_uint4(0u, 0u, 0u, 0u);
    }

    auto load_item = [&](const Item &it) {
        const int total = g.k * it.nq;
#pragma unroll
        for (int j = 0; j < kMaxZPerLane; ++j) {
            const int idx = threadIdx.x + kStreamThreads * j;
            zreg[j] = make_uint4(0u, 0u, 0u, 0u);
            if (idx < total) {
                const int l = idx / it.nq, q = idx - l * it.nq;
                zreg[j] = z_piece<ALIGNED>(g, p, it, Iz, l, q);
            }
        }
        const int per_tile = it.nrows * g.ipw;
        const int ip_total = it.ntiles * per_tile;
#pragma unroll
        for (int j = 0; j < kMaxIpPerLane; ++j) {
            const int idx = threadIdx.x + kStreamThreads * j;
            ipreg[j] = 0u;
            ipdst[j] = -1;
            if (idx < ip_total) {
                const int tl = idx / per_tile, e = idx - tl * per_tile;
                const int64_t t = (int64_t)it.ti * g.tile_cols + it.tj_first + tl;
                ipreg[j] = Ip[(t * g.r + it.row_lo) * g.ipw + e];
                ipdst[j] = (tl * ip_rows) * g.ipw + e;
            }
        }
    };
    auto store_item = [&](const Item &it, int b) {
        const int total = g.k * it.nq;
#pragma unroll
        for (int j = 0; j < kMaxZPerLane; ++j) {
            const int idx = threadIdx.x + kStreamThreads * j;
            if (idx < total) {
                const int l = idx / it.nq, q = idx - l * it.nq;
                LRBI_ZB(b)[l * p.span_chunks + q] = zreg[j];
            }
        }
#pragma unroll
        for (int j = 0; j < kMaxIpPerLane; ++j)
            if (ipdst[j] >= 0) LRBI_IPB(b)[ipdst[j]] = ipreg[j];
    };

    int64_t id = blockIdx.x;
    if (id >= p.items) return;
    Item cur = make_item(g, p, id);
    load_item(cur);
    store_item(cur, 0);
    __syncthreads();
    int b = 0;
    for (;;) {
        const int64_t next_id = id + gridDim.x;
        const bool has_next = next_id < p.items;
        Item nxt = cur;
        if (has_next) {
            nxt = make_item(g, p, next_id);
            load_item(nxt); // in flight while the current item is decoded
        }
        decode_item_rows<ALIGNED>(g, p, cur, LRBI_ZB(b), LRBI_IPB(b), mask, kStreamThreads);
        if (!has_next) break;
        store_item(nxt, b ^ 1); // the other copy was last read before the previous barrier
        __syncthreads();
        b ^= 1;
        cur = nxt;
        id = next_id;
    }
#undef LRBI_ZB
#undef LRBI_IPB
}

// ---------------------------------------------------------------------------
// Nibble-table kernel (tile widths that are multiples of 128 columns).
//
// Walking the set bits of an I_p word costs a data-dependent loop per lane, and a wavefront
// runs as long as its busiest lane.  Here the OR over the selected I_z rows is tabulated
// instead: the k rank indices are cut into G = ceil(k / 4) groups of 4, and for every tile
// under the span and every group the 16 possible ORs of that group's I_z rows are built
// once per item in LDS ("four Russians").  A mask row piece is then the OR of exactly G table
// entries picked by the nibbles of the I_p word: no loop, no divergence, G independent LDS
// reads in flight.  Persistent workgroups of 1024 lanes; the factor loads of the next item
// are in flight while the current item's rows are decoded and stored.
//   T   [tiles][G][16][cpt] 16-byte pieces (cpt = c / 128 pieces per tile row), double buffered
//   IpL [tiles][rows + 1][ipw] words, double buffered
//   Zs  [tiles][k][cpt] pieces: the raw I_z rows of the item being built
// ---------------------------------------------------------------------------
struct NibblePlan {
    int chunks;        // 16-byte pieces per mask row
    int cpt;           // pieces per tile row (c / 128)
    int G;             // nibble groups per I_p row
    int span_tiles;    // tiles per span
    int spans;         // spans per mask row
    int rows_per_band;
    int bands_per_tile_row;
    int tx_log2;       // lanes across a span (power of two >= span_tiles * cpt)
    int iz16;
    int64_t pitch16;
    int64_t items;
    int t_pieces;      // pieces in one T buffer
    int ip_words;      // words in one IpL buffer (multiple of 4)
    int zs_pieces;     // pieces in Zs
    int wgs_per_cu;    // resident workgroups per compute unit the launch aims at
    // one grid stride of the item index, split the way an item index splits into (tile row, band, span)
    int step_span, step_band, step_ti;
    int ip_sh;         // a band's I_p words per tile fit 1 << ip_sh
    int ip_pitch;      // words between the I_p runs of neighbouring tiles in LDS
    int rot_div;       // bands per rotation of the span order
};
static constexpr int kNibTableBytes = 32 * 1024; // per workgroup
static constexpr int kNibTileSkew = 4; // unused 16-byte pieces after every tile's table
static constexpr int kNibMaxIpPerLane = 2; // I_p words a lane fetches per item (one band of every tile under the span)

struct NibItem {
    int ti, row_lo, nrows, tj_first, ntiles;
};
// Item index = (tile row * bands_per_tile_row + band) * spans + span.  A workgroup splits its first index once and
// then advances the three digits by the grid stride (split on the host), so no division runs per item.
struct NibCursor {
    int span, band, ti;
};
__device__ __forceinline__ NibCursor nib_cursor_at(const NibblePlan &p, uint32_t id)
{
    NibCursor cu;
    const uint32_t row = id / (uint32_t)p.spans;
    cu.span = (int)(id - row * (uint32_t)p.spans);
    cu.ti = (int)(row / (uint32_t)p.bands_per_tile_row);
    cu.band = (int)(row - (uint32_t)cu.ti * (uint32_t)p.bands_per_tile_row);
    return cu;
}
__device__ __forceinline__ void nib_cursor_step(const NibblePlan &p, NibCursor &cu)
{
    cu.span += p.step_span;
    cu.band += p.step_band;
    cu.ti += p.step_ti;
    if (cu.span >= p.spans) {
        cu.span -= p.spans;
        ++cu.band;
    }
    if (cu.band >= p.bands_per_tile_row) {
        cu.band -= p.bands_per_tile_row;
        ++cu.ti;
    }
}
__device__ __forceinline__ NibItem make_nib_item(const Geom &g, const NibblePlan &p, const NibCursor &cu)
{
    NibItem it;
    it.ti = cu.ti;
    it.row_lo = cu.band * p.rows_per_band;
    const int row_hi = (it.row_lo + p.rows_per_band < g.r) ? it.row_lo + p.rows_per_band : g.r;
    it.nrows = row_hi - it.row_lo;
    // Workgroups whose grid stride is a whole number of bands would stay on one span for good, and with them every
    // XCD (workgroup index modulo 8) on the same few 256-byte lanes of its L2: the span is rotated by one for every
    // rot_div bands, which is a bijection within a band
    const uint32_t rot = (uint32_t)(cu.ti * p.bands_per_tile_row + cu.band) / (uint32_t)p.rot_div;
    const int span = (int)(((uint32_t)cu.span + rot) % (uint32_t)p.spans);
    it.tj_first = span * p.span_tiles;
    it.ntiles = (it.tj_first + p.span_tiles <= g.tile_cols) ? p.span_tiles : g.tile_cols - it.tj_first;
    return it;
}

__device__ __forceinline__ uint4 or3x4(uint4 a, uint4 b, uint4 c)
{
    return make_uint4(a.x | b.x | c.x, a.y | b.y | c.y, a.z | b.z | c.z, a.w | b.w | c.w);
}

template <int GT /* compile-time G, 0 = run-time */, int CPT /* compile-time pieces per tile row, 0 = run-time */>
__global__ __launch_bounds__(kStreamThreads) LRBI_WAVES_PER_SIMD((GT >= 4 && CPT == 0) ? 4 : 8) void decode_nibble_kernel(Geom g, NibblePlan p,
                                                                       const uint32_t *__restrict__ Ip,
                                                                       const uint32_t *__restrict__ Iz,
                                                                       uint4 *__restrict__ mask)
{
    extern __shared__ uint4 lrbi_dyn_smem[];
    const int G = GT ? GT : p.G;
    const int cpt = CPT ? CPT : p.cpt;
    // a tile's table is followed by four unused pieces, so that the tables of neighbouring tiles start 64 bytes
    // apart modulo the bank width: the entries of the zero nibble (most nibbles) of four tiles then sit in
    // different banks
    const int tile_pieces = G * 16 * cpt + kNibTileSkew;
    // one table (it is rebuilt between two barriers, when nobody reads it), two I_p buffers (the next item's words
    // are stored while the current item is still being decoded), one buffer of raw I_z rows
#define LRBI_TB(b) (lrbi_dyn_smem)
#define LRBI_IPB(b) ((uint32_t *)(lrbi_dyn_smem + p.t_pieces + (b) * (p.ip_words / 4)))
    uint4 *Zs = lrbi_dyn_smem + p.t_pieces + 2 * (p.ip_words / 4);

    // The factor words of an item go from global memory straight into LDS (no registers, no second pass): every
    // wavefront copies runs of 64 consecutive words.  I_z: the k rows of a tile are contiguous (izw = 4 * cpt words
    // per row) and so are the tiles of a span, so the lane index is the piece index from the span's first tile on.
    // I_p: linear index = lane + 1024 * slot, split by a shift into (tile of the span, word within the tile's band);
    // the plan keeps a band within 1 << ip_sh words, and a wavefront's 64 words within one tile's run in LDS.
    const int z_per_tile = g.k * cpt;
    const int z_tl = (int)((uint32_t)threadIdx.x / (uint32_t)z_per_tile); // tile of the span this lane's I_z piece is in
    const uint32_t wave_first = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x & ~63u)); // uniform in a wavefront
    auto load_item = [&](const NibItem &it, int b) {
        const uint32_t *zsrc = Iz + ((int64_t)it.ti * g.tile_cols + it.tj_first) * g.k * (int64_t)g.izw;
        if (p.iz16) {
            if (z_tl < it.ntiles) load_to_lds16(lds_address(Zs + wave_first), zsrc, 16u * threadIdx.x);
        } else {
            const uint32_t z_words = (uint32_t)(it.ntiles * z_per_tile) * 4u;
#pragma unroll
            for (int q = 0; q < 4; ++q) { // words 256 * wave + 64 * q + lane of the run
                const uint32_t w = 4u * wave_first + 64u * q + (threadIdx.x & 63u);
                if (w < z_words) load_to_lds4(lds_address(Zs + wave_first) + 256u * q, zsrc, 4u * w);
            }
        }
        const uint32_t *isrc = Ip + (((int64_t)it.ti * g.tile_cols + it.tj_first) * g.r + it.row_lo) * g.ipw;
        const int ip_live = it.nrows * g.ipw; // words of a tile's band that exist (the last band may be short)
        const int tile_words = g.r * g.ipw;
#pragma unroll
        for (int j = 0; j < kNibMaxIpPerLane; ++j) {
            const int idx = threadIdx.x + kStreamThreads * j;
            const int tl = idx >> p.ip_sh, e = idx & ((1 << p.ip_sh) - 1);
            const int idx0 = (int)wave_first + kStreamThreads * j; // the wavefront's first word
            const int dst0 = (idx0 >> p.ip_sh) * p.ip_pitch + (idx0 & ((1 << p.ip_sh) - 1));
            if (tl < it.ntiles && e < ip_live)
                load_to_lds4(lds_address(LRBI_IPB(b) + dst0), isrc, 4u * (uint32_t)(tl * tile_words + e));
        }
    };
    auto build_table = [&](const NibItem &it, int b) {
        const int total = it.ntiles * G * 16 * cpt;
        for (int idx = threadIdx.x; idx < total; idx += kStreamThreads) {
            const int cq = idx % cpt;
            const int rest = idx / cpt;
            const int nib = rest & 15;
            const int tg = rest >> 4; // tile * G + g
            const int tl = tg / G, gg = tg - tl * G;
            uint4 acc = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int bit = 0; bit < 4; ++bit) {
                const int l = 4 * gg + bit;
                if (((nib >> bit) & 1) && l < g.k) acc = or4(acc, Zs[(tl * g.k + l) * cpt + cq]);
            }
            LRBI_TB(b)[tl * tile_pieces + (gg * 16 + nib) * cpt + cq] = acc;
        }
    };
    // Row loop of an item.  Lane (tx, ty): tx picks the 16-byte piece of the span, ty the row; a lane past the end of a
    // short last span repeats the last piece (the same bytes to the same address), so every wavefront issues the same
    // number of stores and the loop has no per-lane exit.
    const int TX = 1 << p.tx_log2;
    const int TY = kStreamThreads >> p.tx_log2;
    const int ty = threadIdx.x >> p.tx_log2;
    const int nbytes = 16 * cpt, gbytes = 256 * cpt;
    const int ip_step = TY * g.ipw;
    const uint32_t ostep = (uint32_t)((int64_t)TY * p.pitch16 * 16);
    const unsigned char *Tq; // byte address of this lane's column of table entries: entry (g, nib) at g * gbytes + nib * nbytes
    const uint32_t *ipr;
    unsigned char *obase;    // uniform base of the item's first row; a 32-bit byte offset per lane and row is added
    uint32_t ooff;
    uint32_t w_ahead;        // the I_p word is read one row ahead (rows past the band are never used)
    int row;
    auto begin_rows = [&](const NibItem &it, int b) {
        int tx = threadIdx.x & (TX - 1);
        if (tx >= it.ntiles * cpt) tx = it.ntiles * cpt - 1;
        const int tl = tx / cpt, cq = tx - tl * cpt;
        Tq = (const unsigned char *)(LRBI_TB(b) + tl * tile_pieces + cq);
        ipr = LRBI_IPB(b) + tl * p.ip_pitch + ty * g.ipw;
        obase = (unsigned char *)(mask + ((int64_t)it.ti * g.r + it.row_lo) * p.pitch16 + (int64_t)it.tj_first * cpt);
        ooff = (uint32_t)(((int64_t)ty * p.pitch16 + tl * cpt + cq) * 16);
        row = ty;
        w_ahead = ((GT == 1 || GT == 2 || GT == 4 || GT == 8) && ty < it.nrows) ? ipr[0] : 0u;
    };
    auto one_row = [&](const NibItem &it) {
        uint4 acc = make_uint4(0u, 0u, 0u, 0u);
        if (GT == 1 || GT == 2 || GT == 4 || GT == 8) {
            // one I_p word holds all nibbles; GT independent table reads (extract the nibble, scale, add),
            // OR tree of 3-input ORs
            const uint32_t w = w_ahead;
            w_ahead = (row + TY < it.nrows) ? ipr[ip_step] : 0u;
            constexpr int H = (GT > 4) ? 4 : (GT ? GT : 1); // reads in flight together (registers: 4 per read)
#pragma unroll
            for (int h0 = 0; h0 < (GT ? GT : 1); h0 += H) {
                uint4 e[H];
#pragma unroll
                for (int q = 0; q < H; ++q) {
                    const uint32_t nib = (w >> (4 * (h0 + q))) & 15u;
                    e[q] = *reinterpret_cast<const uint4 *>(Tq + (h0 + q) * gbytes + nib * nbytes);
                }
                if (H == 1) acc = or4(acc, e[0]);
                if (H == 2) acc = or3x4(acc, e[0], e[1]);
                if (H == 4) acc = or3x4(or3x4(acc, e[0], e[1]), e[2], e[3]);
#if defined(__HIP_DEVICE_COMPILE__)
                if (GT > 4) __builtin_amdgcn_sched_barrier(0); // the second half's reads start after the first half's ORs
#endif
            }
        } else {
            for (int gg = 0; gg < G; ++gg) {
                const uint32_t w = ipr[gg >> 3];
                const uint32_t nib = (w >> (4 * (gg & 7))) & 15u;
                acc = or4(acc, *reinterpret_cast<const uint4 *>(Tq + gg * gbytes + nib * nbytes));
            }
        }
        *reinterpret_cast<uint4 *>(obase + ooff) = acc;
        row += TY;
        ipr += ip_step;
        ooff += ostep;
    };

    int64_t id = blockIdx.x;
    if (id >= p.items) return;
    NibCursor cu = nib_cursor_at(p, blockIdx.x);
    NibItem cur = make_nib_item(g, p, cu);
    load_item(cur, 0);
    wait_loads<0>();
    __syncthreads();
    build_table(cur, 0);
    __syncthreads();
    int b = 0;
    for (;;) {
        const int64_t next_id = id + gridDim.x;
        const bool has_next = next_id < p.items;
        NibItem nxt = cur;
        if (has_next) {
            nib_cursor_step(p, cu);
            nxt = make_nib_item(g, p, cu);
            load_item(nxt, b ^ 1); // lands in Zs and buffer b^1 (last read before the previous barrier) during the row loop
        }
        begin_rows(cur, b);
        int issued = 0;
        while (row < cur.nrows) {
            one_row(cur);
            ++issued;
        }
        if (!has_next) break;
        // Loads and stores share one in-order completion counter per wavefront.  Waiting until nothing is outstanding
        // would wait for every store of the row loop and run the store pipeline dry once per item; waiting until no
        // more accesses are outstanding than stores were issued after the loads waits for the loads alone.  Lane 0 of
        // a wavefront has its lowest row, hence the most rows: its count is the wavefront's number of stores.
        const int stores = __builtin_amdgcn_readfirstlane(issued);
        if (stores >= 8) wait_loads<8>();
        else if (stores >= 4) wait_loads<4>();
        else if (stores >= 2) wait_loads<2>();
        else if (stores >= 1) wait_loads<1>();
        else wait_loads<0>();
        __syncthreads();
        build_table(nxt, b ^ 1);
        __syncthreads();
        b ^= 1;
        cur = nxt;
        id = next_id;
    }
#undef LRBI_TB
#undef LRBI_IPB
}

// Fills the plan and returns true when the nibble-table kernel can serve the geometry.
static bool plan_nibble(const Geom &g, NibblePlan &p, int64_t pitch_bytes, const void *dIz, int cus)
{
    if (g.c % 128 != 0) return false;
    p.cpt = g.c / 128;
    if (p.cpt > 64) return false;
    p.G = (g.k + 3) / 4;
    const int per_tile_pieces = p.G * 16 * p.cpt;
    // Up to four nibble groups (and eight, with the tile width known at compile time) the kernel fits in
    // 64 registers per lane, so two 1024-lane workgroups can share a compute unit (and its LDS): while one
    // waits at its item boundary (loads of the next item, table build, two barriers) the other keeps the
    // store path busy.
    p.wgs_per_cu = (p.G <= 2 || (p.G == 4 && p.cpt == 2) || (p.G == 8 && p.cpt == 4)) ? 2 : 1; // the variants that fit 64 registers per lane
    p.span_tiles = (kNibTableBytes / (p.G <= 4 ? 2 : 1) / 16) / per_tile_pieces; // the skew pieces come on top of the budget
    if (p.span_tiles > 64 / p.cpt) p.span_tiles = 64 / p.cpt;
    if (p.span_tiles > g.tile_cols) p.span_tiles = g.tile_cols;
    if (p.span_tiles < 1) return false;
    if (p.span_tiles * g.k * p.cpt > kStreamThreads) return false; // one I_z piece per lane
    p.chunks = (int)((g.n + 127) / 128);
    p.spans = (g.tile_cols + p.span_tiles - 1) / p.span_tiles;
    p.tx_log2 = 0;
    while ((1 << p.tx_log2) < p.span_tiles * p.cpt) ++p.tx_log2;
    p.rows_per_band = g.r;
    const int cap_rows = kNibMaxIpPerLane * kStreamThreads / (g.ipw * p.span_tiles);
    if (p.rows_per_band > cap_rows) p.rows_per_band = cap_rows;
    if (p.rows_per_band < 1) return false;
    // small masks: shorter bands until every compute unit has an item
    while (p.rows_per_band > 32 &&
           (int64_t)p.spans * g.tile_rows * ((g.r + p.rows_per_band - 1) / p.rows_per_band) < (int64_t)cus)
        p.rows_per_band = (p.rows_per_band + 1) / 2;
    // a lane finds its I_p words by shifting a linear index: bands padded to a power of two must fit the lanes' slots
    p.ip_sh = 0;
    while ((1 << p.ip_sh) < p.rows_per_band * g.ipw) ++p.ip_sh;
    while (((int64_t)p.span_tiles << p.ip_sh) > (int64_t)kNibMaxIpPerLane * kStreamThreads) {
        --p.ip_sh;
        p.rows_per_band = (1 << p.ip_sh) / g.ipw;
    }
    if (p.rows_per_band < 16 && p.rows_per_band < g.r) return false;
    p.bands_per_tile_row = (g.r + p.rows_per_band - 1) / p.rows_per_band;
    p.items = (int64_t)p.spans * g.tile_rows * p.bands_per_tile_row;
    if (p.items < (int64_t)cus || p.items > 0x7FFFFFFF) return false;
    p.iz16 = (((uintptr_t)dIz & 15) == 0) ? 1 : 0;
    p.pitch16 = pitch_bytes / 16;
    p.t_pieces = p.span_tiles * (per_tile_pieces + kNibTileSkew);
    // one spare row per tile keeps the rows that the tiles of a span read together in different banks; runs shorter
    // than a wavefront's 64 words are packed at their power-of-two pitch, so that the copy into LDS is linear
    p.ip_pitch = (p.ip_sh >= 6) ? (p.rows_per_band + 1) * g.ipw : (1 << p.ip_sh);
    p.ip_words = (p.span_tiles * p.ip_pitch + 3) / 4 * 4;
    p.zs_pieces = p.span_tiles * g.k * p.cpt;
    return true;
}

int launch_decode(const Geom &g, uint32_t flags, const uint32_t *dIp, const uint32_t *dIz, void *dMask,
                  int64_t pitch_bytes, hipStream_t stream)
{
    const int64_t chunks64 = (g.n + 127) / 128;
    DecodePlan p;
    p.chunks = (int)chunks64;
    p.pitch16 = pitch_bytes / 16;

    auto launch_generic = [&]() -> int {
        const int64_t items = g.m * chunks64;
        const int64_t blocks = (items + kDecodeThreads - 1) / kDecodeThreads;
        if (blocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
        LRBI_LAUNCH(decode_generic_kernel, dim3((unsigned)blocks), dim3(kDecodeThreads), 0, stream, g, dIp,
                           dIz, (uint4 *)dMask, p.pitch16, p.chunks);
        return LRBI_OK;
    };
    // cut-off edge tiles: only the generic kernel bounds its rows and columns by the matrix
    if ((flags & LRBI_FLAG_DECODE_GENERIC) || g.ragged) return launch_generic();

    const int cus = compute_units_of(stream);
    {
        NibblePlan np;
        if (plan_nibble(g, np, pitch_bytes, dIz, cus)) {
            const size_t lds = ((size_t)np.t_pieces + 2 * (np.ip_words / 4) + np.zs_pieces) * 16;
            auto kern = decode_nibble_kernel<0, 0>;
            if (np.G == 8 && np.cpt == 4) kern = decode_nibble_kernel<8, 4>;      // 512-column tiles, rank 32
            else if (np.G == 4 && np.cpt == 2) kern = decode_nibble_kernel<4, 2>; // 256-column tiles, rank 16
            else if (np.G == 2 && np.cpt == 1) kern = decode_nibble_kernel<2, 1>; // 128-column tiles, rank 8
            else if (np.G == 8) kern = decode_nibble_kernel<8, 0>;
            else if (np.G == 4) kern = decode_nibble_kernel<4, 0>;
            else if (np.G == 2) kern = decode_nibble_kernel<2, 0>;
            else if (np.G == 1) kern = decode_nibble_kernel<1, 0>;
            LRBI_SET_MAX_LDS(kern, lds);
            const int64_t want = (int64_t)np.wgs_per_cu * cus;
            const int64_t grid = (np.items < want) ? np.items : want;
            np.step_span = (int)(grid % np.spans);
            np.step_band = (int)((grid / np.spans) % np.bands_per_tile_row);
            np.step_ti = (int)((grid / np.spans) / np.bands_per_tile_row);
            np.rot_div = (grid / np.spans) > 0 ? (int)(grid / np.spans) : 1;
            LRBI_LAUNCH(kern, dim3((unsigned)grid), dim3(kStreamThreads), lds, stream, g, np, dIp, dIz,
                               (uint4 *)dMask);
            return LRBI_OK;
        }
    }

    // Column span per item: as wide as the Z table budget allows, at most 64 pieces (one
    // wavefront across).  Rows per band: as many as the I_p budget allows (one table build per
    // band), cut down only when that leaves compute units without work; when the shortest band still gives
    // too few items (small masks), the span is halved as well, down to 64-byte row segments.
    p.span_chunks = kZTableBudgetBytes / (16 * (g.k + 1));
    if (p.span_chunks < 1) p.span_chunks = 1;
    if (p.span_chunks > 64) p.span_chunks = 64;
    p.zshift = 0;
    while ((2 << p.zshift) <= p.span_chunks) ++p.zshift;
    while (p.zshift > 0 && (1 << (p.zshift - 1)) >= p.chunks) --p.zshift; // no wider than the row needs
    bool widest = true, streaming = false;
    for (;; --p.zshift, widest = false) {
        p.span_chunks = 1 << p.zshift;
        p.spans = (p.chunks + p.span_chunks - 1) / p.span_chunks;
        p.tx_log2 = p.zshift;
        p.span_tiles = (int)(((int64_t)p.span_chunks * 128 + g.c - 1) / g.c) + 1;
        p.rows_per_band = g.r;
        const int cap_rows = kIpBudgetBytes / (4 * g.ipw * p.span_tiles) - 1;
        if (p.rows_per_band > cap_rows) p.rows_per_band = cap_rows;
        if (p.rows_per_band < 1) {
            if (p.zshift > kSmallMaskMinShift) continue;
            return launch_generic(); // not even one row of I_p words fits next to the table
        }
        const int min_rows = (2 * g.k > 32) ? 2 * g.k : 32;
        while (p.rows_per_band > min_rows &&
               (int64_t)p.spans * g.tile_rows * ((g.r + p.rows_per_band - 1) / p.rows_per_band) < 2048)
            p.rows_per_band = (p.rows_per_band + 1) / 2;
        const int64_t items = (int64_t)p.spans * g.tile_rows * ((g.r + p.rows_per_band - 1) / p.rows_per_band);
        if (widest && items >= 4 * (int64_t)cus) streaming = true; // streaming pays off once every compute unit gets several items
        if (streaming || p.zshift <= kSmallMaskMinShift || items >= kSmallMaskItems) break;
    }
    p.bands_per_tile_row = (g.r + p.rows_per_band - 1) / p.rows_per_band;
    p.items = (int64_t)p.spans * g.tile_rows * p.bands_per_tile_row;
    if (p.items > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    p.iz16 = (((uintptr_t)dIz & 15) == 0) ? 1 : 0;
    const size_t z_bytes = (size_t)(g.k + 1) * p.span_chunks * 16;
    const size_t ip_bytes = ((size_t)p.span_tiles * (p.rows_per_band + 1) * g.ipw * 4 + 15) / 16 * 16;
    const bool aligned = (g.c % 128) == 0;

    if (streaming) {
        const size_t lds = 2 * (z_bytes + ip_bytes);
        auto kern = aligned ? decode_stream_kernel<true> : decode_stream_kernel<false>;
        LRBI_SET_MAX_LDS(kern, lds);
        LRBI_LAUNCH(kern, dim3((unsigned)cus), dim3(kStreamThreads), lds, stream, g, p, dIp, dIz, (uint4 *)dMask);
    } else {
        const size_t lds = z_bytes + ip_bytes;
        auto kern = aligned ? decode_ztable_kernel<true> : decode_ztable_kernel<false>;
        LRBI_LAUNCH(kern, dim3((unsigned)p.items), dim3(kDecodeThreads), lds, stream, g, p, dIp, dIz,
                           (uint4 *)dMask);
    }
    return LRBI_OK;
}

} // namespace lrbi
