// Fused masked product on the matrix cores (f16 / bf16, fp32 accumulate):
// Y = (W o I_a) X with the mask of Eq. 3 rebuilt per K-slab inside the kernel.
//
// A workgroup of 4 wavefronts owns a BM x BN tile of Y and walks the n range
// (the reduction dimension) in slabs of BK = 64 columns of W.  Per slab:
//   1. 16-byte global loads bring the W slab (BM x 64) and the X slab (64 x BN)
//      into registers, one slab ahead of the arithmetic;
//   2. every lane rebuilds one or two 32-bit words of the slab's mask from the
//      packed factors (OR of the I_z words selected by the set bits of the I_p
//      row) and publishes them in a small LDS array;
//   3. when the W registers go to LDS, each 16-byte piece is ANDed with the
//      16-bit-lane expansion of its 8 mask bits: pruned weights become +0 by
//      select, so nothing stored under a 0 bit (NaN, Inf) reaches the product,
//      and the masking cost is paid once per slab, not once per MFMA operand;
//   4. the wavefronts read their operands from LDS and issue 32x32x16 MFMAs.
//      X sits in LDS in its natural [k][n] order, and the operand needs 8
//      consecutive k per lane, so it is gathered column-wise.
// LDS is double buffered; there is one workgroup barrier per slab.
//
// The MFMA is issued as D = X^T-fragment * W^T-fragment, i.e. the accumulator
// holds a 32(n) x 32(m) block: each lane then owns 4 consecutive n of one output
// row, which makes the stores of Y 8 bytes wide per lane.
//
// When m * N yields too few tiles to fill 256 compute units, the n range is cut
// into `splitk` slices; slices write fp32 partial tiles to the caller's
// workspace and a second kernel adds them in slice order (deterministic).
#include <stdlib.h>
#include <type_traits>
#include <utility>

#include "lrbi_internal.hpp"
#include "lrbi_mfma_common.hpp"

namespace lrbi {

static constexpr int kThreads = 256;
static constexpr int WS_STRIDE = BK + 8; // halfs; 16-byte pad keeps 16-byte row alignment

template <int BM, int BN> struct Smem {
    static constexpr int XS_STRIDE = BN + 8;
    static constexpr int ws_halfs = BM * WS_STRIDE;
    static constexpr int xs_halfs = BK * XS_STRIDE;
    static constexpr int ms_words = BM * 2;
    static constexpr size_t bytes = 2 * (size_t)(ws_halfs + xs_halfs) * 2 + 2 * (size_t)ms_words * 4;
};

// Mask word for (row, 32-column half) of the slab starting at column k0.
// ALIGNED: c % 64 == 0, so the slab lies inside tile column tj = k0 / c.
template <bool ALIGNED>
__device__ __forceinline__ uint32_t slab_mask_word(const Geom &g, const uint32_t *__restrict__ Ip,
                                                   const uint32_t *__restrict__ Iz, int64_t row, int k0, int half,
                                                   int tj, int wt /* word of the slab inside its tile */)
{
    if (row >= g.m) return 0u;
    const int ti = (int)(row / g.r);
    const int il = (int)(row - (int64_t)ti * g.r);
    if (!ALIGNED) return decode_word(g, Ip, Iz, ti, il, (k0 >> 5) + half);
    const int64_t t = (int64_t)ti * g.tile_cols + tj;
    const uint32_t *ip = Ip + (t * g.r + il) * g.ipw;
    const uint32_t *iz = Iz + t * g.k * (int64_t)g.izw + wt + half;
    uint32_t acc = 0u;
    for (int iw = 0; iw < g.ipw; ++iw) {
        uint32_t sel = ip[iw];
        const uint32_t *zr = iz + (int64_t)(32 * iw) * g.izw;
        while (sel) { // four ranks per round, their loads in flight together (fewer left: the last one again)
            const int l0 = __builtin_ctz(sel);
            sel &= sel - 1u;
            const int l1 = sel ? __builtin_ctz(sel) : l0;
            sel &= sel - 1u;
            const int l2 = sel ? __builtin_ctz(sel) : l1;
            sel &= sel - 1u;
            const int l3 = sel ? __builtin_ctz(sel) : l2;
            sel &= sel - 1u;
            acc |= (zr[(int64_t)l0 * g.izw] | zr[(int64_t)l1 * g.izw]) | (zr[(int64_t)l2 * g.izw] | zr[(int64_t)l3 * g.izw]);
        }
    }
    return acc;
}

template <typename Tag, int BM, int BN, int WAVES_M, int WAVES_N, bool ALIGNED, bool XVEC, bool SPLIT>
__global__ __launch_bounds__(kThreads) void mfma_gemm_kernel(
    Geom g, const uint16_t *__restrict__ W, int64_t ldw, const uint32_t *__restrict__ Ip,
    const uint32_t *__restrict__ Iz, const uint16_t *__restrict__ X, int64_t ldx, int N,
    uint16_t *__restrict__ Y, int64_t ldy, float *__restrict__ P, int64_t ldp, int mblocks, int nblocks,
    int64_t kper, int xcd_remap, int y_vec_ok, uint32_t *__restrict__ mask_out, int64_t mask_pitch32)
{
    static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per workgroup");
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int FM = WM / 32, FN = WN / 32;
    static_assert(FM >= 1 && FN >= 1, "wave tile must hold a 32x32 block");
    using S = Smem<BM, BN>;
    constexpr int XS_STRIDE = S::XS_STRIDE;
    constexpr int W_CHUNKS = BM * (BK / 8) / kThreads;  // 16-byte pieces of W per lane per slab
    constexpr int X_CPR = BN / 8;                       // 16-byte pieces per X row
    constexpr int X_CHUNKS = (BK * X_CPR + kThreads - 1) / kThreads;
    constexpr int M_WORDS = (BM * 2 + kThreads - 1) / kThreads;
    static_assert(BM * (BK / 8) % kThreads == 0, "W slab must split evenly");

    extern __shared__ uint4 lrbi_dyn_smem[];
    uint16_t *Ws = (uint16_t *)lrbi_dyn_smem;            // [2][BM][WS_STRIDE]
    uint16_t *Xs = Ws + 2 * S::ws_halfs;                 // [2][BK][XS_STRIDE]
    uint32_t *Ms = (uint32_t *)(Xs + 2 * S::xs_halfs);   // [2][BM][2]

    // workgroup -> (slice, row block, column block); column block fastest so that
    // workgroups sharing a W row block are neighbours.  With xcd_remap the hardware's
    // round-robin of consecutive workgroup ids over the 8 XCDs is undone, so that
    // neighbours land on the same XCD and share its L2.
    int64_t bid = blockIdx.x;
    if (xcd_remap) {
        const int64_t per = gridDim.x / 8;
        bid = (bid % 8) * per + bid / 8;
    }
    const int ni = (int)(bid % nblocks);
    const int mi = (int)((bid / nblocks) % mblocks);
    const int slice = (int)(bid / ((int64_t)nblocks * mblocks));
    const int64_t m0 = (int64_t)mi * BM;
    const int n0 = ni * BN;
    const int kbeg = (int)(slice * kper);
    const int kend = (int)((kbeg + kper < g.n) ? kbeg + kper : g.n);
    const int nslabs = (kend - kbeg + BK - 1) / BK;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int l32 = lane & 31, lg = lane >> 5;

    uint4 wreg[W_CHUNKS];
    uint4 xreg[X_CHUNKS];

    auto load_slab = [&](int slab) {
        const int k0 = kbeg + slab * BK;
#pragma unroll
        for (int i = 0; i < W_CHUNKS; ++i) {
            const int id = tid + kThreads * i;
            const int row = id >> 3, kc = id & 7;
            const int64_t gr = m0 + row;
            const int kk = k0 + kc * 8;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (gr < g.m && kk < kend) v = *reinterpret_cast<const uint4 *>(W + gr * ldw + kk);
            wreg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < X_CHUNKS; ++i) {
            const int id = tid + kThreads * i;
            const int krow = id / X_CPR, nc = id % X_CPR;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (id < BK * X_CPR) {
                const int kk = k0 + krow;
                const int nn = n0 + nc * 8;
                if (kk < kend) {
                    if (XVEC) {
                        if (nn < N) v = *reinterpret_cast<const uint4 *>(X + (int64_t)kk * ldx + nn);
                    } else {
                        uint16_t tmp[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) tmp[e] = (nn + e < N) ? X[(int64_t)kk * ldx + nn + e] : (uint16_t)0;
                        v = *reinterpret_cast<uint4 *>(tmp);
                    }
                }
            }
            xreg[i] = v;
        }
    };

    const int64_t mask_cols = (g.n + 127) / 128 * 128; // columns of a mask row up to the end of its last 16-byte piece
    auto decode_slab = [&](int slab, int buf) {
        const int k0 = kbeg + slab * BK;
        int tj = 0, wt = 0;
        if (ALIGNED) {
            tj = k0 / g.c;
            wt = (k0 - tj * g.c) >> 5;
        }
#pragma unroll
        for (int i = 0; i < M_WORDS; ++i) {
            const int idx = tid + kThreads * i;
            if (idx < BM * 2) {
                const int row = idx >> 1, half = idx & 1;
                const uint32_t word = slab_mask_word<ALIGNED>(g, Ip, Iz, m0 + row, k0, half, tj, wt);
                Ms[buf * S::ms_words + idx] = word;
                // The mask as a by-product (the stand-alone decode's layout: one bit per weight, whole 16-byte pieces
                // per row, pad bits zero): every (row, word) is formed by exactly one workgroup of the first column
                // block; the last slab of a row also clears what is left of the row's last 16-byte piece.
                if (mask_out && ni == 0 && m0 + row < g.m) {
                    const int col0 = k0 + 32 * half;
                    uint32_t *mrow = mask_out + (m0 + row) * mask_pitch32;
                    if (col0 < g.n) {
                        const int64_t left = g.n - col0;
                        mrow[col0 >> 5] = (left < 32) ? (word & ((1u << left) - 1u)) : word;
                    } else if (col0 < mask_cols) {
                        mrow[col0 >> 5] = 0u;
                    }
                    if (slab == nslabs - 1 && kend == g.n && col0 + 64 < mask_cols) mrow[(col0 + 64) >> 5] = 0u;
                }
            }
        }
    };

    auto stage_slab = [&](int buf) {
        uint16_t *ws = Ws + buf * S::ws_halfs;
        uint16_t *xs = Xs + buf * S::xs_halfs;
        const unsigned char *mb = (const unsigned char *)(Ms + buf * S::ms_words);
#pragma unroll
        for (int i = 0; i < W_CHUNKS; ++i) {
            const int id = tid + kThreads * i;
            const int row = id >> 3, kc = id & 7;
            const uint32_t bits = mb[row * 8 + kc];
            *reinterpret_cast<uint4 *>(ws + row * WS_STRIDE + kc * 8) = apply_mask8(wreg[i], bits);
        }
#pragma unroll
        for (int i = 0; i < X_CHUNKS; ++i) {
            const int id = tid + kThreads * i;
            if (id < BK * X_CPR) {
                const int krow = id / X_CPR, nc = id % X_CPR;
                *reinterpret_cast<uint4 *>(xs + krow * XS_STRIDE + nc * 8) = xreg[i];
            }
        }
    };

    f32x16 acc[FN][FM];
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // prologue: slab 0 into buffer 0, slab 1 in flight
    if (nslabs > 0) {
        load_slab(0);
        decode_slab(0, 0);
        __syncthreads();
        stage_slab(0);
        if (nslabs > 1) { // the mask words first: their dependent loads are waited for at once, and a wavefront's
            decode_slab(1, 1); // loads complete in order, so operand loads issued ahead of them would be drained
            load_slab(1);
        }
        __syncthreads();
    }

    for (int s = 0; s < nslabs; ++s) {
        const int buf = s & 1;
        const uint16_t *ws = Ws + buf * S::ws_halfs;
        const uint16_t *xs = Xs + buf * S::xs_halfs;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int kof = kk * 16 + 8 * lg;
            uint4 wf[FM], xf[FN];
#pragma unroll
            for (int b = 0; b < FM; ++b)
                wf[b] = *reinterpret_cast<const uint4 *>(ws + (wm * WM + b * 32 + l32) * WS_STRIDE + kof);
#pragma unroll
            for (int a = 0; a < FN; ++a) {
                const uint16_t *col = xs + kof * XS_STRIDE + wn * WN + a * 32 + l32;
                uint16_t tmp[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) tmp[e] = col[e * XS_STRIDE];
                xf[a] = *reinterpret_cast<uint4 *>(tmp);
            }
#pragma unroll
            for (int a = 0; a < FN; ++a)
#pragma unroll
                for (int b = 0; b < FM; ++b) acc[a][b] = mfma_32x32x16(Tag{}, xf[a], wf[b], acc[a][b]);
        }
        if (s + 1 < nslabs) stage_slab(buf ^ 1);
        if (s + 2 < nslabs) {
            decode_slab(s + 2, buf);
            load_slab(s + 2);
        }
        __syncthreads();
    }

    // epilogue: lane holds, per 32x32 block, rows n = 8*(v/4) + 4*lg + (v%4) and column m = l32
#pragma unroll
    for (int a = 0; a < FN; ++a) {
#pragma unroll
        for (int b = 0; b < FM; ++b) {
            const int64_t row = m0 + wm * WM + b * 32 + l32;
            if (row >= g.m) continue;
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int col = n0 + wn * WN + a * 32 + 8 * v4 + 4 * lg;
                if (SPLIT) {
                    if (col < ldp) {
                        float4 o = make_float4(acc[a][b][4 * v4 + 0], acc[a][b][4 * v4 + 1], acc[a][b][4 * v4 + 2],
                                               acc[a][b][4 * v4 + 3]);
                        *reinterpret_cast<float4 *>(P + ((int64_t)slice * g.m + row) * ldp + col) = o;
                    }
                } else {
                    uint16_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = cvt_store(Tag{}, acc[a][b][4 * v4 + e]);
                    if (y_vec_ok && col + 3 < N) {
                        *reinterpret_cast<uint2 *>(Y + row * ldy + col) = *reinterpret_cast<uint2 *>(o);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < N) Y[row * ldy + col + e] = o[e];
                    }
                }
            }
        }
    }
}

// Sum the fp32 partial tiles of all slices in slice order and round to the storage dtype.
template <typename Tag>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ P, int64_t ldp, int64_t m, int N,
                                                            int splitk, uint16_t *__restrict__ Y, int64_t ldy,
                                                            int y_vec_ok)
{
    const int64_t groups_per_row = ldp / 4;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= m * groups_per_row) return;
    const int64_t row = e / groups_per_row;
    const int col = (int)(e - row * groups_per_row) * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    const float *src = P + row * ldp + col;
    const int64_t plane = m * ldp;
    int k = 0;
    // eight slices at a time: their loads are in flight together, the additions stay in slice order
    for (; k + 8 <= splitk; k += 8) {
        float4 p[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) p[q] = *reinterpret_cast<const float4 *>(src + (int64_t)(k + q) * plane);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            s.x += p[q].x;
            s.y += p[q].y;
            s.z += p[q].z;
            s.w += p[q].w;
        }
    }
    for (; k < splitk; ++k) {
        const float4 p = *reinterpret_cast<const float4 *>(src + (int64_t)k * plane);
        s.x += p.x;
        s.y += p.y;
        s.z += p.z;
        s.w += p.w;
    }
    uint16_t o[4] = {cvt_store(Tag{}, s.x), cvt_store(Tag{}, s.y), cvt_store(Tag{}, s.z), cvt_store(Tag{}, s.w)};
    if (y_vec_ok && col + 3 < N) {
        *reinterpret_cast<uint2 *>(Y + row * ldy + col) = *reinterpret_cast<uint2 *>(o);
    } else {
        for (int q = 0; q < 4; ++q)
            if (col + q < N) Y[row * ldy + col + q] = o[q];
    }
}

// ---------------------------------------------------------------------------
// Panel kernel: the fast path for tile shapes that line up with the kernel's
// blocking (c % 128 == 0, r % BM == 0, k <= 64; hence no row or reduction tails).
//
// Differences from the kernel above:
//   * The mask is rebuilt one PANEL (512 columns = 8 slabs) at a time and well
//     ahead of its first use, entirely from LDS: the panel's slice of the I_z
//     rows ("Fz", k x 512 bits) and the I_p words of the workgroup's rows
//     ("Fip") are fetched with plain loads while earlier slabs are multiplied,
//     so no dependent global load sits in front of an MFMA.
//   * X operands come out of LDS with the gfx950 transposing read
//     (ds_read_b64_tr_b16): X stays in its natural [k][n] order and each lane
//     still receives 8 consecutive k of one column.
//   * Global loads run RS slabs ahead of the LDS staging (register stages).
//   * With KGROUPS = 2 the workgroup has 8 wavefronts: two groups of four, each
//     group covering the whole BM x BN tile for half of every slab's 64 columns.
//     Two wavefronts then share each SIMD, so one's mask arithmetic and LDS traffic
//     overlap the other's MFMAs, while LDS operand traffic per flop stays that of a
//     64 x 64 wave tile.  The two groups' accumulators are added through LDS at the end
//     (fixed order: group 0 + group 1).
// ---------------------------------------------------------------------------

template <int BM, int BN> struct SmemPanel {
    static constexpr int XPAD = (BN >= 64) ? 32 : 8; // halfs; keeps the transposing reads off shared banks
    static constexpr int XS_STRIDE = BN + XPAD;
    static constexpr int ws_halfs = BM * WS_STRIDE;
    static constexpr int xs_halfs = BK * XS_STRIDE;
    static constexpr int ms_words = BM * PANEL_WORDS;
    static constexpr int fz_words = FAST_MAX_K * PANEL_WORDS;
    static constexpr int fip_words = BM * PANEL_UNITS * 2;
    static constexpr size_t loop_bytes =
        2 * (size_t)(ws_halfs + xs_halfs) * 2 + 2 * (size_t)(ms_words + fz_words + fip_words) * 4;
    static constexpr size_t reduce_bytes = (size_t)BM * BN * 4; // one group's fp32 accumulators
    static constexpr size_t bytes = loop_bytes > reduce_bytes ? loop_bytes : reduce_bytes;
};

template <typename Tag, int BM, int BN, int WAVES_M, int WAVES_N, int KGROUPS, int RS, bool XVEC, bool SPLIT>
__global__ __launch_bounds__(256 * KGROUPS) void mfma_gemm_panel_kernel(
    Geom g, const uint16_t *__restrict__ W, int64_t ldw, const uint32_t *__restrict__ Ip,
    const uint32_t *__restrict__ Iz, const uint16_t *__restrict__ X, int64_t ldx, int N,
    uint16_t *__restrict__ Y, int64_t ldy, float *__restrict__ P, int64_t ldp, int mblocks, int nblocks,
    int64_t kper, int xcd_remap, int y_vec_ok)
{
    static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per group");
    static_assert(KGROUPS == 1 || KGROUPS == 2, "one or two wave groups");
    constexpr int NT = 256 * KGROUPS;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int FM = WM / 32, FN = WN / 32;
    static_assert(FM >= 1 && FN >= 1, "wave tile must hold a 32x32 block");
    constexpr int KK_PER = (BK / 16) / KGROUPS; // 16-column MFMA steps per slab and group
    using S = SmemPanel<BM, BN>;
    constexpr int XS_STRIDE = S::XS_STRIDE;
    constexpr int W_CHUNKS = BM * (BK / 8) / NT;
    constexpr int X_CPR = BN / 8;
    constexpr int X_TOTAL = BK * X_CPR;
    constexpr int X_CHUNKS = (X_TOTAL + NT - 1) / NT;
    constexpr bool X_EVEN = (X_TOTAL % NT) == 0;
    constexpr int FZ_LOADS = FAST_MAX_K * PANEL_WORDS / NT;
    constexpr int FIP_TOTAL = BM * PANEL_UNITS * 2;
    constexpr int FIP_LOADS = (FIP_TOTAL + NT - 1) / NT;
    constexpr int UNITS_TOTAL = BM * PANEL_UNITS;
    constexpr int UNITS = (UNITS_TOTAL + NT - 1) / NT;
    static_assert(BM * (BK / 8) % NT == 0, "W slab must split evenly");
    static_assert(FAST_MAX_K * PANEL_WORDS % NT == 0, "Fz must split evenly");

    extern __shared__ uint4 lrbi_dyn_smem[];
    uint16_t *Ws = (uint16_t *)lrbi_dyn_smem;            // [2][BM][WS_STRIDE]
    uint16_t *Xs = Ws + 2 * S::ws_halfs;                 // [2][BK][XS_STRIDE]
    uint32_t *Ms = (uint32_t *)(Xs + 2 * S::xs_halfs);   // [2][BM][PANEL_WORDS]   mask panels
    uint32_t *Fz = Ms + 2 * S::ms_words;                 // [2][64][PANEL_WORDS]   I_z rows under the panel
    uint32_t *Fip = Fz + 2 * S::fz_words;                // [2][BM][PANEL_UNITS][2] I_p words per row and unit

    int64_t bid = blockIdx.x;
    if (xcd_remap) {
        const int64_t per = gridDim.x / 8;
        bid = (bid % 8) * per + bid / 8;
    }
    const int ni = (int)(bid % nblocks);
    const int mi = (int)((bid / nblocks) % mblocks);
    const int slice = (int)(bid / ((int64_t)nblocks * mblocks));
    const int64_t m0 = (int64_t)mi * BM;
    const int n0 = ni * BN;
    const int kbeg = (int)(slice * kper);
    const int kend = (int)((kbeg + kper < g.n) ? kbeg + kper : g.n);
    const int nslabs = (kend - kbeg) / BK; // n % 128 == 0 and kper % 128 == 0: whole slabs only
    const int npanels = (nslabs + PANEL_SLABS - 1) / PANEL_SLABS;
    // the workgroup's rows lie inside one tile row (r % BM == 0)
    const int ti = (int)(m0 / g.r);
    const int il0 = (int)(m0 - (int64_t)ti * g.r);
    const int64_t trow = (int64_t)ti * g.tile_cols;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int kg = wave >> 2;       // wave group (k half of every slab)
    const int w4 = wave & 3;
    const int wm = w4 / WAVES_N, wn = w4 % WAVES_N;
    const int l32 = lane & 31, lg = lane >> 5;

    u32x4 wreg[RS][W_CHUNKS];
    u32x4 xreg[RS][X_CHUNKS];
    uint32_t fzreg[FZ_LOADS];
    uint32_t fipreg[FIP_LOADS];
    uint32_t mbits[W_CHUNKS]; // mask bytes of the slab that is staged next

    // W loads need no guards (no tails).  Addresses are a uniform base that advances per slab
    // plus a per-lane 32-bit offset that never changes.
    const uint16_t *wbase = W + m0 * ldw + kbeg;
    const uint16_t *xbase_g = X + (int64_t)kbeg * ldx + n0;
    uint32_t woff[W_CHUNKS], wlds[W_CHUNKS], moff[W_CHUNKS];
#pragma unroll
    for (int i = 0; i < W_CHUNKS; ++i) {
        const int id = tid + NT * i;
        const int row = id >> 3, kc = id & 7;
        woff[i] = (uint32_t)(row * ldw + kc * 8);
        wlds[i] = (uint32_t)(row * WS_STRIDE + kc * 8);
        moff[i] = (uint32_t)(row * (PANEL_WORDS * 4) + kc);
    }
    uint32_t xoff[X_CHUNKS], xlds[X_CHUNKS];
#pragma unroll
    for (int i = 0; i < X_CHUNKS; ++i) {
        const int id = (tid + NT * i) % X_TOTAL; // lanes beyond the slab repeat a valid piece (never stored)
        const int krow = id / X_CPR, nc = id % X_CPR;
        int nn = nc * 8;
        if (XVEC && n0 + nn + 8 > N) nn = N - 8 - n0; // piece beyond N: read a valid piece instead, its columns are dropped
        xoff[i] = (uint32_t)(krow * ldx + nn);
        xlds[i] = (uint32_t)(krow * XS_STRIDE + nc * 8);
    }

    auto load_slab = [&](int slab, auto stage_c) {
        constexpr int st = decltype(stage_c)::value;
        const uint16_t *wb = wbase + slab * BK;
        const uint16_t *xb = xbase_g + (int64_t)slab * BK * ldx;
#pragma unroll
        for (int i = 0; i < W_CHUNKS; ++i) wreg[st][i] = *reinterpret_cast<const u32x4 *>(wb + woff[i]);
#pragma unroll
        for (int i = 0; i < X_CHUNKS; ++i) {
            if constexpr (XVEC) {
                xreg[st][i] = *reinterpret_cast<const u32x4 *>(xb + xoff[i]);
            } else {
                const int nn = n0 + (((tid + NT * i) % X_TOTAL) % X_CPR) * 8;
                u32x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t lo = (nn + 2 * e < N) ? xb[xoff[i] + 2 * e] : 0u;
                    const uint32_t hi = (nn + 2 * e + 1 < N) ? xb[xoff[i] + 2 * e + 1] : 0u;
                    v[e] = lo | (hi << 16);
                }
                xreg[st][i] = v;
            }
        }
    };

    // mask bytes of `slab` (its panel is decoded and visible by now)
    auto fetch_mask_bytes = [&](int slab) {
        const unsigned char *mb = (const unsigned char *)(Ms + ((slab / PANEL_SLABS) & 1) * S::ms_words) +
                                  (slab % PANEL_SLABS) * (BK / 8);
#pragma unroll
        for (int i = 0; i < W_CHUNKS; ++i) mbits[i] = mb[moff[i]];
    };

    auto stage_slab = [&](int slab, auto stage_c) {
        constexpr int st = decltype(stage_c)::value;
        const int buf = slab & 1;
        uint16_t *ws = Ws + buf * S::ws_halfs;
        uint16_t *xs = Xs + buf * S::xs_halfs;
#pragma unroll
        for (int i = 0; i < W_CHUNKS; ++i)
            *reinterpret_cast<u32x4 *>(ws + wlds[i]) = apply_mask8(wreg[st][i], mbits[i]);
#pragma unroll
        for (int i = 0; i < X_CHUNKS; ++i)
            if (X_EVEN || tid + NT * i < X_TOTAL) *reinterpret_cast<u32x4 *>(xs + xlds[i]) = xreg[st][i];
    };

    // factor slices of one panel: global -> registers
    auto load_factors = [&](int panel) {
        const int kp = kbeg + panel * PW;
#pragma unroll
        for (int i = 0; i < FZ_LOADS; ++i) {
            const int idx = tid + NT * i;
            const int l = idx / PANEL_WORDS, w = idx % PANEL_WORDS;
            const int col = kp + 32 * w;
            uint32_t v = 0u;
            if (l < g.k && col < kend) {
                const int tj = col / g.c;
                v = Iz[((trow + tj) * g.k + l) * g.izw + ((col - tj * g.c) >> 5)];
            }
            fzreg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < FIP_LOADS; ++i) {
            const int idx = tid + NT * i;
            const int row = idx / (PANEL_UNITS * 2), u = (idx / 2) % PANEL_UNITS, iw = idx & 1;
            const int col = kp + 128 * u;
            uint32_t v = 0u;
            if (idx < FIP_TOTAL && iw < g.ipw && col < kend) {
                const int tj = col / g.c;
                v = Ip[((trow + tj) * g.r + il0 + row) * g.ipw + iw];
            }
            fipreg[i] = v;
        }
    };
    // registers -> LDS
    auto store_factors = [&](int panel) {
        uint32_t *fz = Fz + (panel & 1) * S::fz_words;
        uint32_t *fip = Fip + (panel & 1) * S::fip_words;
#pragma unroll
        for (int i = 0; i < FZ_LOADS; ++i) fz[tid + NT * i] = fzreg[i];
#pragma unroll
        for (int i = 0; i < FIP_LOADS; ++i) {
            const int idx = tid + NT * i;
            if (idx < FIP_TOTAL) fip[idx] = fipreg[i];
        }
    };
    // Eq. 3 for the panel: mask row piece = OR of the Fz pieces selected by the set bits of the I_p words
    auto decode_panel = [&](int panel) {
        const uint32_t *fz = Fz + (panel & 1) * S::fz_words;
        const uint32_t *fip = Fip + (panel & 1) * S::fip_words;
        uint32_t *ms = Ms + (panel & 1) * S::ms_words;
#pragma unroll
        for (int i = 0; i < UNITS; ++i) {
            const int uid = tid + NT * i;
            if (uid < UNITS_TOTAL) {
                const int row = uid / PANEL_UNITS, u = uid % PANEL_UNITS;
                uint4 acc = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
                for (int iw = 0; iw < 2; ++iw) {
                    uint32_t sel = fip[(row * PANEL_UNITS + u) * 2 + iw];
                    while (sel) {
                        const int l = __builtin_ctz(sel) + 32 * iw;
                        sel &= sel - 1u;
                        const uint4 z = *reinterpret_cast<const uint4 *>(fz + l * PANEL_WORDS + 4 * u);
                        acc.x |= z.x;
                        acc.y |= z.y;
                        acc.z |= z.z;
                        acc.w |= z.w;
                    }
                }
                *reinterpret_cast<uint4 *>(ms + row * PANEL_WORDS + 4 * u) = acc;
            }
        }
    };

    f32x16 acc[FN][FM];
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // transposing read: 16-lane group G = lane / 16 serves columns 16 * (G % 2) .. + 15 of a
    // 32-column block and k group G / 2; lane d of the group addresses row d / 4, columns 4 * (d % 4)
    const int d16 = lane & 15, G16 = lane >> 4;
    const uint32_t xfrag_off = (uint32_t)((kg * KK_PER * 16 + 8 * (G16 >> 1) + (d16 >> 2)) * XS_STRIDE + wn * WN +
                                          16 * (G16 & 1) + 4 * (d16 & 3));
    const uint32_t wfrag_off = (uint32_t)((wm * WM + l32) * WS_STRIDE + kg * KK_PER * 16 + 8 * lg);

    auto compute_slab = [&](int slab) {
        const int buf = slab & 1;
        const uint16_t *ws = Ws + buf * S::ws_halfs + wfrag_off;
        const uint16_t *xs = Xs + buf * S::xs_halfs + xfrag_off;
#pragma unroll
        for (int kk = 0; kk < KK_PER; ++kk) {
            uint4 wf[FM], xf[FN];
#pragma unroll
            for (int b = 0; b < FM; ++b)
                wf[b] = *reinterpret_cast<const uint4 *>(ws + b * 32 * WS_STRIDE + kk * 16);
#pragma unroll
            for (int a = 0; a < FN; ++a) {
                const uint16_t *p = xs + (kk * 16) * XS_STRIDE + a * 32;
                const uint2 lo = lds_read_tr16(p);
                const uint2 hi = lds_read_tr16(p + 4 * XS_STRIDE);
                xf[a] = make_uint4(lo.x, lo.y, hi.x, hi.y);
            }
#pragma unroll
            for (int a = 0; a < FN; ++a)
#pragma unroll
                for (int b = 0; b < FM; ++b) acc[a][b] = mfma_32x32x16(Tag{}, xf[a], wf[b], acc[a][b]);
        }
    };

    // ---- prologue: factors and mask of panel 0, slabs 0 .. RS-1 in flight, slab 0 staged
    const int last = nslabs - 1;
    load_factors(0);
    static_for<RS>([&](auto sc) {
        constexpr int st = decltype(sc)::value;
        load_slab(st < last ? st : last, sc);
    });
    store_factors(0);
    __syncthreads();
    decode_panel(0);
    __syncthreads();
    fetch_mask_bytes(0);
    stage_slab(0, std::integral_constant<int, 0>{});
    load_slab(RS < last ? RS : last, std::integral_constant<int, 0>{});
    __syncthreads();

    // ---- main loop, unrolled by RS so that register stages are compile-time.
    // The body has no data-dependent guards: past the end it stages and reloads the last slab
    // again (into the LDS buffer nobody reads).
    for (int s0 = 0; s0 < nslabs; s0 += RS) {
        static_for<RS>([&](auto sc) {
            constexpr int j = decltype(sc)::value;
            const int s = s0 + j;
            if (RS == 1 || s < nslabs) {
                using NextStage = std::integral_constant<int, (j + 1) % RS>;
                fetch_mask_bytes(s + 1 < last ? s + 1 : last);
                // the two wave groups run the two halves of the iteration in opposite order, so that on
                // every SIMD one wavefront issues MFMAs while the other does the mask arithmetic
                if (KGROUPS == 2 && kg == 1) {
                    stage_slab(s + 1, NextStage{});
                    compute_slab(s);
                } else {
                    compute_slab(s);
                    stage_slab(s + 1, NextStage{});
                }
                load_slab(s + 1 + RS < last ? s + 1 + RS : last, NextStage{});
                // next panel's factors and mask, spread over three slabs
                const int ps = s % PANEL_SLABS;
                const int next_panel = s / PANEL_SLABS + 1;
                if (next_panel < npanels) {
                    if (ps == 0) load_factors(next_panel);
                    if (ps == 1) store_factors(next_panel);
                    if (ps == 2) decode_panel(next_panel);
                }
                __syncthreads();
            }
        });
    }

    // ---- two wave groups: group 1 hands its accumulators to group 0 through LDS
    if (KGROUPS == 2) {
        float *red = (float *)lrbi_dyn_smem; // [4 waves][FN][FM][16][64 lanes]; the loop buffers are dead now
        float *mine = red + (size_t)w4 * (FN * FM * 16 * 64) + lane;
        if (kg == 1) {
#pragma unroll
            for (int a = 0; a < FN; ++a)
#pragma unroll
                for (int b = 0; b < FM; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mine[((a * FM + b) * 16 + v) * 64] = acc[a][b][v];
        }
        __syncthreads();
        if (kg == 1) return;
#pragma unroll
        for (int a = 0; a < FN; ++a)
#pragma unroll
            for (int b = 0; b < FM; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[a][b][v] += mine[((a * FM + b) * 16 + v) * 64];
    }

    // epilogue: lane holds, per 32x32 block, rows n = 8*(v/4) + 4*lg + (v%4) and column m = l32
#pragma unroll
    for (int a = 0; a < FN; ++a) {
#pragma unroll
        for (int b = 0; b < FM; ++b) {
            const int64_t row = m0 + wm * WM + b * 32 + l32;
            if (row >= g.m) continue;
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int col = n0 + wn * WN + a * 32 + 8 * v4 + 4 * lg;
                if (SPLIT) {
                    if (col < ldp) {
                        float4 o = make_float4(acc[a][b][4 * v4 + 0], acc[a][b][4 * v4 + 1], acc[a][b][4 * v4 + 2],
                                               acc[a][b][4 * v4 + 3]);
                        *reinterpret_cast<float4 *>(P + ((int64_t)slice * g.m + row) * ldp + col) = o;
                    }
                } else {
                    uint16_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = cvt_store(Tag{}, acc[a][b][4 * v4 + e]);
                    if (y_vec_ok && col + 3 < N) {
                        *reinterpret_cast<uint2 *>(Y + row * ldy + col) = *reinterpret_cast<uint2 *>(o);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < N) Y[row * ldy + col + e] = o[e];
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

struct TileDef {
    int bm, bn;
    bool panel; // panel kernel (needs c % 128 == 0, r % bm == 0, k <= 64)
};
// tile ids (desc.flags bits 16..19); 0 = automatic.  1-3: generic kernel, 4-8: panel kernel with 4
// wavefronts, 9-11: panel kernel with 8 wavefronts (two wave groups).
static const TileDef kTiles[] = {{0, 0, false},    {128, 128, false}, {128, 64, false}, {128, 32, false},
                                 {128, 128, true}, {128, 128, true},  {128, 64, true},  {128, 32, true},
                                 {128, 128, true}, {128, 128, true},  {128, 64, true},  {128, 32, true},
                                 {128, 128, true}, {128, 128, true},  {128, 128, true}};
static constexpr int kNumTiles = 14;
static constexpr int kFirstPipeTile = 12; // 12 .. 14: the software-pipelined kernel (lrbi_gemm_pipe.hip), variants 0 .. 2

static bool panel_ok(const Geom &g, int bm)
{
    return (g.c % 128 == 0) && (g.r % bm == 0) && (g.k <= FAST_MAX_K) && !g.ragged;
}

MfmaPlan plan_mfma(const Geom &g, uint32_t flags, int64_t N)
{
    MfmaPlan p;
    int tile = (int)((flags & LRBI_FLAG_TILE_MASK) >> LRBI_FLAG_TILE_SHIFT);
    if (tile >= 1 && tile <= kNumTiles && kTiles[tile].panel && !panel_ok(g, kTiles[tile].bm) &&
        !(tile >= kFirstPipeTile && pipe_shape_ok(g)))
        tile = 0;
    if (tile < 1 || tile > kNumTiles) {
        tile = (N > 64) ? 1 : (N > 32 ? 2 : 3);
        // 14 (the pipelined kernel, also at 33 to 64 columns: HBM-cold 4096 x 9216 at N = 64 25.0 against 26.9 us on
        // the 128 x 64 panel kernel) falls back to 9 / 10 when X is not 16-byte readable
        if (panel_ok(g, 128)) tile = (N > 32) ? 14 : 11;
        // tile widths of 64 (2 j + 1): no panel kernel, so the pipelined kernel also takes 33 to 64 columns (half of its
        // column block idle, but W is streamed at the same rate: 4096 x 9216 in 512 x 576 tiles, N = 64, 25 us against
        // 40 us on the generic kernel); falls back to the generic kernel when X is not 16-byte readable
        else if (N > 32 && pipe_shape_ok(g)) tile = 14;
        else if (tile == 1) {
            // few rows, many columns (a small convolution layer as a product): narrower column blocks that fill the
            // chip by themselves instead of a split with its round trip of partial planes (64 x 576, N = 16384:
            // 19.4 us against 18.7 + 4.2 us)
            const int64_t mb = (g.m + 127) / 128;
            if (mb * ((N + 127) / 128) < 192) {
                if (mb * ((N + 63) / 64) >= 192) tile = 2;
                else if (mb * ((N + 31) / 32) >= 192) tile = 3;
            }
        }
    }
    p.tile = tile;
    p.bm = kTiles[tile].bm;
    p.bn = kTiles[tile].bn;
    const int64_t mblocks = (g.m + p.bm - 1) / p.bm;
    const int64_t nblocks = (N + p.bn - 1) / p.bn;
    const int64_t tiles = mblocks * nblocks;
    const int64_t npairs = (g.n + 2 * BK - 1) / (2 * BK); // slices are cut at multiples of 128 columns
    int split = (int)((flags & LRBI_FLAG_SPLITK_MASK) >> LRBI_FLAG_SPLITK_SHIFT);
    if (split == 0) {
        split = 1;
        if (tiles < 192) {
            // The 512-lane panel kernels run one workgroup per compute unit (measured best: one slice per
            // unit, at least 8 slabs per slice), the 256-lane panel kernels two.  The general kernel pays a
            // round of dependent factor loads per slab, so short slices and more workgroups in flight pay off
            // (C4: 12 slices of 4 slabs, 23 us against 32 us with 6 slices).
            const bool general = tile < 4;
            const int64_t target = (tile >= 9) ? 256 : (general ? 1024 : 512);
            int64_t want = (target + tiles - 1) / tiles;
            const int64_t min_pairs = general ? 2 : 4;
            const int64_t cap = npairs / min_pairs > 1 ? npairs / min_pairs : 1;
            if (want > cap) want = cap;
            if (want > 64) want = 64;
            split = (int)(want < 1 ? 1 : want);
        }
    }
    if (split > npairs) split = (int)npairs;
    int64_t pairs_per = (npairs + split - 1) / split;
    split = (int)((npairs + pairs_per - 1) / pairs_per); // no empty slice
    p.splitk = split;
    p.kper = pairs_per * 2 * BK;
    const int64_t ldp = (N + 3) / 4 * 4;
    p.workspace_bytes = (split > 1) ? (uint64_t)split * (uint64_t)g.m * (uint64_t)ldp * 4u : 0u;
    return p;
}

// adds the split-K partial planes in slice order and rounds to the storage dtype
template <typename Tag>
static int launch_reduce(const Geom &g, const MfmaPlan &plan, int64_t N, void *dY, int64_t ldy, void *dWorkspace,
                         hipStream_t stream)
{
    const int64_t ldp = (N + 3) / 4 * 4;
    const int y_vec_ok = (((uintptr_t)dY & 7) == 0) && (ldy % 4 == 0);
    const int64_t items = g.m * (ldp / 4);
    const int64_t rblocks = (items + 255) / 256;
    if (rblocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    LRBI_LAUNCH(splitk_reduce_kernel<Tag>, dim3((unsigned)rblocks), dim3(256), 0, stream,
                       (const float *)dWorkspace, ldp, g.m, (int)N, plan.splitk, (uint16_t *)dY, ldy, y_vec_ok);
    return LRBI_OK;
}

template <typename Tag, int BM, int BN, int WAVES_M, int WAVES_N, int RS /* 0: generic kernel */, int KGROUPS = 1>
static int launch_tile(const Geom &g, const MfmaPlan &plan, const void *dW, int64_t ldw, const uint32_t *dIp,
                       const uint32_t *dIz, const void *dX, int64_t ldx, int64_t N, void *dY, int64_t ldy,
                       void *dWorkspace, hipStream_t stream, MaskOut mo)
{
    if (RS > 0 && mo.ptr) return LRBI_ERR_SHAPE; // only the generic kernel leaves the mask
    const int64_t mblocks = (g.m + BM - 1) / BM;
    const int64_t nblocks = (N + BN - 1) / BN;
    const int64_t blocks = mblocks * nblocks * plan.splitk;
    if (blocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    const bool aligned = (g.c % BK) == 0;
    const bool xvec = (((uintptr_t)dX & 15) == 0) && (ldx % 8 == 0) && (N % 8 == 0);
    const bool split = plan.splitk > 1 || plan.planes_only;
    const int y_vec_ok = (((uintptr_t)dY & 7) == 0) && (ldy % 4 == 0);
    const int xcd_remap = (blocks % 8 == 0) ? 1 : 0;
    const int64_t ldp = (N + 3) / 4 * 4;
    const dim3 grid((unsigned)blocks), block(RS > 0 ? 256 * KGROUPS : kThreads);

#define LRBI_LAUNCH_TILE(KERN, SMEM)                                                                                   \
    do {                                                                                                          \
        auto kern = KERN;                                                                                         \
        LRBI_SET_MAX_LDS(kern, (SMEM));                                                                           \
        LRBI_LAUNCH(kern, grid, block, (SMEM), stream, g, (const uint16_t *)dW, ldw, dIp, dIz,             \
                           (const uint16_t *)dX, ldx, (int)N, (uint16_t *)dY, ldy, (float *)dWorkspace, ldp,      \
                           (int)mblocks, (int)nblocks, plan.kper, xcd_remap, y_vec_ok);                           \
    } while (0)
#define LRBI_LAUNCH_GEN(KERN, SMEM)                                                                                    \
    do {                                                                                                          \
        auto kern = KERN;                                                                                         \
        LRBI_SET_MAX_LDS(kern, (SMEM));                                                                           \
        LRBI_LAUNCH(kern, grid, block, (SMEM), stream, g, (const uint16_t *)dW, ldw, dIp, dIz,             \
                           (const uint16_t *)dX, ldx, (int)N, (uint16_t *)dY, ldy, (float *)dWorkspace, ldp,      \
                           (int)mblocks, (int)nblocks, plan.kper, xcd_remap, y_vec_ok, (uint32_t *)mo.ptr,        \
                           mo.pitch16 * 4);                                                                       \
    } while (0)

    if constexpr (RS > 0) {
        const size_t smem = SmemPanel<BM, BN>::bytes;
        if (xvec) {
            if (split) LRBI_LAUNCH_TILE((mfma_gemm_panel_kernel<Tag, BM, BN, WAVES_M, WAVES_N, KGROUPS, RS, true, true>), smem);
            else LRBI_LAUNCH_TILE((mfma_gemm_panel_kernel<Tag, BM, BN, WAVES_M, WAVES_N, KGROUPS, RS, true, false>), smem);
        } else {
            if (split) LRBI_LAUNCH_TILE((mfma_gemm_panel_kernel<Tag, BM, BN, WAVES_M, WAVES_N, KGROUPS, RS, false, true>), smem);
            else LRBI_LAUNCH_TILE((mfma_gemm_panel_kernel<Tag, BM, BN, WAVES_M, WAVES_N, KGROUPS, RS, false, false>), smem);
        }
    } else {
        const size_t smem = Smem<BM, BN>::bytes;
        if (aligned) {
            if (xvec) {
                if (split) LRBI_LAUNCH_GEN((mfma_gemm_kernel<Tag, BM, BN, WAVES_M, WAVES_N, true, true, true>), smem);
                else LRBI_LAUNCH_GEN((mfma_gemm_kernel<Tag, BM, BN, WAVES_M, WAVES_N, true, true, false>), smem);
            } else {
                if (split) LRBI_LAUNCH_GEN((mfma_gemm_kernel<Tag, BM, BN, WAVES_M, WAVES_N, true, false, true>), smem);
                else LRBI_LAUNCH_GEN((mfma_gemm_kernel<Tag, BM, BN, WAVES_M, WAVES_N, true, false, false>), smem);
            }
        } else {
            if (xvec) {
                if (split) LRBI_LAUNCH_GEN((mfma_gemm_kernel<Tag, BM, BN, WAVES_M, WAVES_N, false, true, true>), smem);
                else LRBI_LAUNCH_GEN((mfma_gemm_kernel<Tag, BM, BN, WAVES_M, WAVES_N, false, true, false>), smem);
            } else {
                if (split) LRBI_LAUNCH_GEN((mfma_gemm_kernel<Tag, BM, BN, WAVES_M, WAVES_N, false, false, true>), smem);
                else LRBI_LAUNCH_GEN((mfma_gemm_kernel<Tag, BM, BN, WAVES_M, WAVES_N, false, false, false>), smem);
            }
        }
    }
#undef LRBI_LAUNCH_TILE
#undef LRBI_LAUNCH_GEN

    if (split && !plan.planes_only) return launch_reduce<Tag>(g, plan, N, dY, ldy, dWorkspace, stream);
    return LRBI_OK;
}

#define LRBI_TILE_ARGS g, plan, dW, ldw, dIp, dIz, dX, ldx, N, dY, ldy, dWorkspace, stream, mo
template <typename Tag>
static int launch_dtype(const Geom &g, const MfmaPlan &plan, const void *dW, int64_t ldw, const uint32_t *dIp,
                        const uint32_t *dIz, const void *dX, int64_t ldx, int64_t N, void *dY, int64_t ldy,
                        void *dWorkspace, hipStream_t stream, MaskOut mo)
{
    int tile = plan.tile;
    // the panel kernel keeps per-lane element offsets in 32 bits
    if (kTiles[tile].panel && (ldw > (1 << 24) || ldx > (1 << 24))) tile = (kTiles[tile].bn == 128) ? 1 : (kTiles[tile].bn == 64 ? 2 : 3);
    switch (tile) {
    case 1: return launch_tile<Tag, 128, 128, 2, 2, 0>(LRBI_TILE_ARGS);
    case 2: return launch_tile<Tag, 128, 64, 2, 2, 0>(LRBI_TILE_ARGS);
    case 3: return launch_tile<Tag, 128, 32, 4, 1, 0>(LRBI_TILE_ARGS);
    case 4: return launch_tile<Tag, 128, 128, 2, 2, 2>(LRBI_TILE_ARGS);
    case 5: return launch_tile<Tag, 128, 128, 2, 2, 3>(LRBI_TILE_ARGS);
    case 6: return launch_tile<Tag, 128, 64, 2, 2, 2>(LRBI_TILE_ARGS);
    case 7: return launch_tile<Tag, 128, 32, 4, 1, 3>(LRBI_TILE_ARGS);
    case 8: return launch_tile<Tag, 128, 128, 2, 2, 1>(LRBI_TILE_ARGS);
    case 9: return launch_tile<Tag, 128, 128, 2, 2, 2, 2>(LRBI_TILE_ARGS);
    case 10: return launch_tile<Tag, 128, 64, 2, 2, 2, 2>(LRBI_TILE_ARGS);
    case 11: return launch_tile<Tag, 128, 32, 4, 1, 2, 2>(LRBI_TILE_ARGS);
    default: return LRBI_ERR_FLAGS;
    }
}
#undef LRBI_TILE_ARGS

// The convolution form: plan as for N = batch * H * Wd columns on the pipelined kernel, which gathers its X operand
// from the padded activation; partial planes of a split reduction are added as for the matrix form.
int launch_mfma_conv(const Geom &g, const MfmaPlan &plan, lrbi_dtype dt, const ConvGeom &cg, const void *dW, int64_t ldw,
                     const uint32_t *dIp, const uint32_t *dIz, const void *dAct, int64_t N, void *dY, int64_t ldy,
                     void *dWorkspace, hipStream_t stream)
{
    if (((uintptr_t)dW & 15) != 0 || ldw % 8 != 0) return LRBI_ERR_ALIGN;
    if (plan.tile < kFirstPipeTile) return LRBI_ERR_SHAPE;
    const int rc = launch_pipe_conv(g, plan, dt, cg, dW, ldw, dIp, dIz, dAct, N, dY, ldy, dWorkspace, stream);
    if (rc != LRBI_OK) return rc;
    if (plan.splitk > 1 && !plan.planes_only) {
        if (dt == LRBI_F16) return launch_reduce<F16Tag>(g, plan, N, dY, ldy, dWorkspace, stream);
        return launch_reduce<BF16Tag>(g, plan, N, dY, ldy, dWorkspace, stream);
    }
    return LRBI_OK;
}

bool mfma_gemm_emits_mask(const Geom &g, const MfmaPlan &plan, const void *dW, int64_t ldw, const void *dIz,
                          const void *dX, int64_t ldx, int64_t N)
{
    if (((uintptr_t)dW & 15) != 0 || ldw % 8 != 0 || g.n % 8 != 0) return false;
    if (plan.tile >= 1 && plan.tile <= 3) return true; // the generic kernel: any shape
    return plan.tile >= kFirstPipeTile && pipe_ok(g, dIz, dX, ldw, ldx, N);
}

int launch_mfma_gemm(const Geom &g, const MfmaPlan &plan_in, lrbi_dtype dt, const void *dW, int64_t ldw,
                     const uint32_t *dIp, const uint32_t *dIz, const void *dX, int64_t ldx, int64_t N, void *dY,
                     int64_t ldy, void *dWorkspace, hipStream_t stream, MaskOut mo)
{
    // the W loads are 16 bytes wide
    if (((uintptr_t)dW & 15) != 0 || ldw % 8 != 0 || g.n % 8 != 0) return LRBI_ERR_ALIGN;
    MfmaPlan plan = plan_in;
    if (plan.tile >= kFirstPipeTile) {
        if (pipe_ok(g, dIz, dX, ldw, ldx, N)) {
            const int pf = plan.tile - kFirstPipeTile;
            const int rc = launch_pipe_gemm(g, plan, dt, pf, dW, ldw, dIp, dIz, dX, ldx, N, dY, ldy, dWorkspace, stream, mo);
            if (rc != LRBI_OK) return rc;
            if (plan.splitk > 1 && !plan.planes_only) {
                if (dt == LRBI_F16) return launch_reduce<F16Tag>(g, plan, N, dY, ldy, dWorkspace, stream);
                return launch_reduce<BF16Tag>(g, plan, N, dY, ldy, dWorkspace, stream);
            }
            return LRBI_OK;
        }
        plan.tile = panel_ok(g, 128) ? (N > 64 ? 9 : 10) : 1; // the staged panel kernels, or the generic one
    }
    if (mo.ptr && !(plan.tile >= 1 && plan.tile <= 3)) return LRBI_ERR_SHAPE; // the caller asks mfma_gemm_emits_mask() first
    if (dt == LRBI_F16)
        return launch_dtype<F16Tag>(g, plan, dW, ldw, dIp, dIz, dX, ldx, N, dY, ldy, dWorkspace, stream, mo);
    if (dt == LRBI_BF16)
        return launch_dtype<BF16Tag>(g, plan, dW, ldw, dIp, dIz, dX, ldx, N, dY, ldy, dWorkspace, stream, mo);
    return LRBI_ERR_DTYPE;
}

} // namespace lrbi
