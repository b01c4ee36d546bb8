// Mask decode to HBM: I_a,t = I_p,t (x) I_z,t for every tile (Eq. 3, Sec. 3.1),
// written as the one-bit-per-weight binary index form (Fig. 1).
//
// The kernel is bound by HBM stores when the integer work per 32-bit mask word
// stays small, so the design spends almost nothing per word:
//   * a workgroup owns a band of rows of one tile row and a span of columns;
//   * it first copies the I_z rows of every tile under that span into LDS,
//     shifted to their absolute bit position in the mask row ("Z table":
//     Z[l] is the concatenation over tiles of row l of each tile's I_z), so
//     tile boundaries that fall inside a word are resolved once per band and
//     not once per mask row;
//   * a lane then produces 128 mask bits at a time: it walks the SET bits of the
//     I_p row (about k*p of them) and ORs the matching 16-byte pieces of Z;
//   * consecutive lanes hold consecutive 16-byte pieces of one mask row, so the
//     stores are full-width and coalesced.
#include "lrbi_internal.hpp"

namespace lrbi {

static constexpr int kDecodeThreads = 256;
static constexpr int kZTableBudgetBytes = 32 * 1024;

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

// One 32-bit word of Z[l] at absolute word index w of the mask row (tile row ti).
template <bool ALIGNED>
__device__ __forceinline__ uint32_t ztable_word(const Geom &g, const uint32_t *__restrict__ Iz, int ti, int l, int w)
{
    const int64_t j0 = (int64_t)w * 32;
    if (j0 >= g.n) return 0u;
    if (ALIGNED) { // c is a multiple of 32: the word lies inside one tile
        const int wpt = g.c >> 5;
        const int tj = w / wpt;
        const int64_t t = (int64_t)ti * g.tile_cols + tj;
        return Iz[(t * g.k + l) * g.izw + (w - tj * wpt)];
    }
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

// ALIGNED: c % 128 == 0, every 128-bit piece lies inside one tile.
// Grid: blockIdx.x enumerates (row band, column span) with the span fastest.
template <bool ALIGNED>
__global__ __launch_bounds__(kDecodeThreads) void decode_ztable_kernel(
    Geom g, const uint32_t *__restrict__ Ip, const uint32_t *__restrict__ Iz, uint4 *__restrict__ mask,
    int64_t pitch16, int chunks /* 16-byte pieces per mask row */, int span_chunks, int spans,
    int rows_per_band, int bands_per_tile_row, int tx_log2)
{
    extern __shared__ uint4 lrbi_dyn_smem[];
    uint4 *Z = lrbi_dyn_smem; // [k][span_chunks]
    const int64_t bid = blockIdx.x;
    const int span = (int)(bid % spans);
    const int64_t band = bid / spans;
    const int ti = (int)(band / bands_per_tile_row);
    const int row_lo = (int)(band - (int64_t)ti * bands_per_tile_row) * rows_per_band;
    const int row_hi = (row_lo + rows_per_band < g.r) ? row_lo + rows_per_band : g.r;
    const int q_lo = span * span_chunks;
    const int nq = (q_lo + span_chunks <= chunks) ? span_chunks : chunks - q_lo;

    // build the Z table for this span
    {
        uint32_t *Zw = (uint32_t *)Z;
        const int words = 4 * nq;
        for (int idx = threadIdx.x; idx < g.k * words; idx += kDecodeThreads) {
            const int l = idx / words;
            const int w = idx - l * words;
            Zw[l * (4 * span_chunks) + w] = ztable_word<ALIGNED>(g, Iz, ti, l, 4 * q_lo + w);
        }
    }
    __syncthreads();

    const int TX = 1 << tx_log2;
    const int tx = threadIdx.x & (TX - 1);
    const int ty = threadIdx.x >> tx_log2;
    const int TY = kDecodeThreads >> tx_log2;
    for (int q = tx; q < nq; q += TX) {
        const int Q = q_lo + q;        // absolute 16-byte piece of the mask row
        const int64_t cb = (int64_t)Q * 128; // first column of the piece
        if (ALIGNED) {
            const int tj = (int)(cb / g.c);
            const int64_t t = (int64_t)ti * g.tile_cols + tj;
            const uint32_t *ipt = Ip + t * g.r * g.ipw;
            for (int il = row_lo + ty; il < row_hi; il += TY) {
                uint4 acc = make_uint4(0u, 0u, 0u, 0u);
                for (int iw = 0; iw < g.ipw; ++iw) {
                    uint32_t sel = ipt[(int64_t)il * g.ipw + iw];
                    while (sel) {
                        const int l = __builtin_ctz(sel) + 32 * iw;
                        sel &= sel - 1u;
                        acc = or4(acc, Z[l * span_chunks + q]);
                    }
                }
                mask[((int64_t)ti * g.r + il) * pitch16 + Q] = acc;
            }
        } else {
            const int64_t ce = (cb + 128 < g.n) ? cb + 128 : g.n;
            const int tj_lo = (int)(cb / g.c);
            for (int il = row_lo + ty; il < row_hi; il += TY) {
                uint4 acc = make_uint4(0u, 0u, 0u, 0u);
                int tj = tj_lo;
                for (int64_t tbeg = (int64_t)tj * g.c; tbeg < ce; tbeg += g.c, ++tj) {
                    const int64_t t = (int64_t)ti * g.tile_cols + tj;
                    const uint32_t *ipr = Ip + (t * g.r + il) * g.ipw;
                    // bits of this piece that belong to tile tj
                    const int lo = (int)((tbeg > cb ? tbeg : cb) - cb);
                    const int hi = (int)((tbeg + g.c < ce ? tbeg + g.c : ce) - cb);
                    uint4 tm;
                    tm.x = bit_range(lo < 0 ? 0 : lo, hi > 32 ? 32 : hi);
                    tm.y = bit_range(lo - 32 < 0 ? 0 : lo - 32, hi - 32 > 32 ? 32 : hi - 32);
                    tm.z = bit_range(lo - 64 < 0 ? 0 : lo - 64, hi - 64 > 32 ? 32 : hi - 64);
                    tm.w = bit_range(lo - 96 < 0 ? 0 : lo - 96, hi - 96 > 32 ? 32 : hi - 96);
                    uint4 v = make_uint4(0u, 0u, 0u, 0u);
                    for (int iw = 0; iw < g.ipw; ++iw) {
                        uint32_t sel = ipr[iw];
                        while (sel) {
                            const int l = __builtin_ctz(sel) + 32 * iw;
                            sel &= sel - 1u;
                            v = or4(v, Z[l * span_chunks + q]);
                        }
                    }
                    acc.x |= v.x & tm.x;
                    acc.y |= v.y & tm.y;
                    acc.z |= v.z & tm.z;
                    acc.w |= v.w & tm.w;
                }
                mask[((int64_t)ti * g.r + il) * pitch16 + Q] = acc;
            }
        }
    }
}

int launch_decode(const Geom &g, uint32_t flags, const uint32_t *dIp, const uint32_t *dIz, void *dMask,
                  int64_t pitch_bytes, hipStream_t stream)
{
    const int64_t chunks64 = (g.n + 127) / 128;
    const int chunks = (int)chunks64;
    const int64_t pitch16 = pitch_bytes / 16;

    if (flags & LRBI_FLAG_DECODE_GENERIC) {
        const int64_t items = g.m * chunks64;
        const int64_t blocks = (items + kDecodeThreads - 1) / kDecodeThreads;
        if (blocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
        hipLaunchKernelGGL(decode_generic_kernel, dim3((unsigned)blocks), dim3(kDecodeThreads), 0, stream, g, dIp,
                           dIz, (uint4 *)dMask, pitch16, chunks);
        LRBI_CHECK_LAUNCH();
        return LRBI_OK;
    }

    // column span per workgroup: as wide as the Z table budget allows
    int span_chunks = kZTableBudgetBytes / (16 * g.k);
    if (span_chunks < 1) span_chunks = 1;
    if (span_chunks > chunks) span_chunks = chunks;
    const int spans = (chunks + span_chunks - 1) / span_chunks;
    // lanes along the row: a power of two covering the span, at most one wavefront
    int tx_log2 = 0;
    while ((1 << tx_log2) < span_chunks && tx_log2 < 6) ++tx_log2;
    // rows per band: whole tile height unless that leaves the chip idle; building
    // the Z table costs about k words per column word, so keep bands well above k rows
    int rows_per_band = g.r;
    const int min_rows = (4 * g.k > 32) ? 4 * g.k : 32;
    while (rows_per_band > min_rows &&
           (int64_t)spans * g.tile_rows * ((g.r + rows_per_band - 1) / rows_per_band) < 2048)
        rows_per_band = (rows_per_band + 1) / 2;
    const int bands_per_tile_row = (g.r + rows_per_band - 1) / rows_per_band;
    const int64_t blocks = (int64_t)spans * g.tile_rows * bands_per_tile_row;
    if (blocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    const size_t lds = (size_t)g.k * span_chunks * 16;
    const bool aligned = (g.c % 128) == 0;
    if (aligned)
        hipLaunchKernelGGL(decode_ztable_kernel<true>, dim3((unsigned)blocks), dim3(kDecodeThreads), lds, stream, g,
                           dIp, dIz, (uint4 *)dMask, pitch16, chunks, span_chunks, spans, rows_per_band,
                           bands_per_tile_row, tx_log2);
    else
        hipLaunchKernelGGL(decode_ztable_kernel<false>, dim3((unsigned)blocks), dim3(kDecodeThreads), lds, stream, g,
                           dIp, dIz, (uint4 *)dMask, pitch16, chunks, span_chunks, spans, rows_per_band,
                           bands_per_tile_row, tx_log2);
    LRBI_CHECK_LAUNCH();
    return LRBI_OK;
}

} // namespace lrbi
