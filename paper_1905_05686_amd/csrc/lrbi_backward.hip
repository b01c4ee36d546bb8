// Backward pass through the masking layer (Sec. 2: the decoded index acts as a binary masking
// layer on W, so retraining sends gradients through the kept weights only).  With
// Y = (W o I_a) X and dY the gradient with respect to Y:
//   transposed product   dX = (W o I_a)^T dY        (n x N)
//   weight gradient      dW = (dY X^T) o I_a        (m x n, pruned weights get exactly 0)
// As in the forward product the mask never goes through HBM: its words are rebuilt from the
// factors (Eq. 3) inside the kernels.
//
// Matrix-core kernels (f16 / bf16, 16-byte aligned operands), 256 lanes = 4 wavefronts:
//   * mfma_gemm_t_kernel: output tile 128 columns of W (rows of dX) x BQ batch columns, reduction
//     over the rows of W in slabs of 64, optionally split into slices over m (partial planes
//     added in slice order by bwd_reduce_kernel).  A slab of W (64 rows x 128 columns) is loaded
//     row-major (coalesced), masked in registers and staged in LDS as [row][column]; dY's slab
//     likewise as [row][batch column].  Both MFMA operands therefore need 8 consecutive
//     reduction steps of one column: the gfx950 transposing LDS read delivers exactly that.
//   * mfma_grad_kernel: output tile 128 x 128 of dW, reduction over the batch in slabs of 64.
//     dY rows and X rows are both contiguous along the batch, so both operands are staged as
//     [row][batch] and read with plain 16-byte LDS reads.  The fp32 tile is rounded, parked in
//     LDS and written as whole 256-byte row pieces, each 16-byte piece masked on its way out.
// Vector-ALU kernels (fp32, or operands without the alignment): plain, slow, any shape.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "lrbi_internal.hpp"
#include "lrbi_mfma_common.hpp"

namespace lrbi {

static constexpr int kBwdThreads = 256;
static constexpr int BJ = 128; // columns of W per workgroup (both kernels)

// ---------------------------------------------------------------------------
// dX = (W o I_a)^T dY on the matrix cores
// ---------------------------------------------------------------------------
template <int BQ> struct SmemT {
    // halfs; rows stay 16-byte aligned, and the four rows a 16-lane group of the transposing read touches fall
    // into different banks (measured: 6 % faster than a pad of 8)
    static constexpr int WS_STRIDE = BJ + 16;
    static constexpr int XS_STRIDE = BQ + 16;
    static constexpr int ws_halfs = BK * WS_STRIDE;
    static constexpr int xs_halfs = BK * XS_STRIDE;
    static constexpr int ms_words = BK * (BJ / 32);
    static constexpr int fz_words = FAST_MAX_K * (BJ / 32); // one tile's I_z rows over the workgroup's 128 columns
    static constexpr size_t bytes =
        2 * (size_t)(ws_halfs + xs_halfs) * 2 + 2 * (size_t)ms_words * 4 + 2 * (size_t)fz_words * 4;
};

// FAST: c % 128 == 0 (the workgroup's 128 columns lie in one tile column), r % 64 == 0 and r >= 128 (a slab lies in
// one tile row, three consecutive slabs in at most two), k <= 64, no cut-off tiles.  Then the I_z rows of the current
// tile row (k x 4 words) are kept in LDS, fetched three slabs ahead, and the I_p words of a slab's rows are requested
// one iteration before they are used: no dependent global load sits in the loop.
template <typename Tag, int BQ, int WAVES_J, int WAVES_Q, bool XVEC, bool SPLIT, bool FAST>
__global__ __launch_bounds__(kBwdThreads) void mfma_gemm_t_kernel(
    Geom g, const uint16_t *__restrict__ W, int64_t ldw, const uint32_t *__restrict__ Ip,
    const uint32_t *__restrict__ Iz, const uint16_t *__restrict__ DY, int64_t lddy, int N,
    uint16_t *__restrict__ DX, int64_t lddx, float *__restrict__ P, int64_t ldp, int jblocks, int qblocks,
    int64_t iper, int xcd_remap, int y_vec_ok)
{
    static_assert(WAVES_J * WAVES_Q == 4, "four wavefronts per workgroup");
    constexpr int WJ = BJ / WAVES_J, WQ = BQ / WAVES_Q;
    constexpr int FJ = WJ / 32, FQ = WQ / 32;
    static_assert(FJ >= 1 && FQ >= 1, "wave tile must hold a 32x32 block");
    using S = SmemT<BQ>;
    constexpr int WS_STRIDE = S::WS_STRIDE, XS_STRIDE = S::XS_STRIDE;
    constexpr int W_CPR = BJ / 8;                              // 16-byte pieces per slab row of W
    constexpr int W_CHUNKS = BK * W_CPR / kBwdThreads;          // pieces per lane per slab
    constexpr int X_CPR = BQ / 8;
    constexpr int X_CHUNKS = (BK * X_CPR + kBwdThreads - 1) / kBwdThreads;
    static_assert(BK * W_CPR % kBwdThreads == 0, "W slab must split evenly");
    static_assert(BK * (BJ / 32) == kBwdThreads, "one mask word per lane and slab");

    extern __shared__ uint4 lrbi_dyn_smem[];
    uint16_t *Ws = (uint16_t *)lrbi_dyn_smem;            // [2][BK][WS_STRIDE]
    uint16_t *Xs = Ws + 2 * S::ws_halfs;                 // [2][BK][XS_STRIDE]
    uint32_t *Ms = (uint32_t *)(Xs + 2 * S::xs_halfs);   // [2][BK][BJ / 32]
    uint32_t *Fz = Ms + 2 * S::ms_words;                 // [2][k][BJ / 32], by parity of the tile row

    // workgroup -> (slice, column block of W, batch block), batch block fastest: the workgroups that share a strip
    // of W are neighbours.  With xcd_remap the hardware's round-robin of consecutive workgroup ids over the 8 XCDs
    // is undone, so that those neighbours land on one XCD and the strip goes through one L2, not eight.
    int64_t bid = blockIdx.x;
    if (xcd_remap) {
        const int64_t per = gridDim.x / 8;
        bid = (bid % 8) * per + bid / 8;
    }
    const int qi = (int)(bid % qblocks);
    const int ji = (int)((bid / qblocks) % jblocks);
    const int slice = (int)(bid / ((int64_t)qblocks * jblocks));
    const int j0 = ji * BJ;
    const int q0 = qi * BQ;
    const int64_t ibeg = (int64_t)slice * iper;
    const int64_t iend = (ibeg + iper < g.m) ? ibeg + iper : g.m;
    const int nslabs = (int)((iend - ibeg + BK - 1) / BK);
    const int n = (int)g.n;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wj = wave / WAVES_Q, wq = wave % WAVES_Q;
    const int l32 = lane & 31, lg = lane >> 5;

    uint4 wreg[W_CHUNKS];
    uint4 xreg[X_CHUNKS];

    // Addresses: a base that is uniform over the workgroup (advanced per slab with scalar arithmetic) plus a
    // per-lane byte offset that never changes, so that no 64-bit multiply sits in the loop.  Offsets stay below
    // 2^31 (64 rows of at most 2^24 elements).  Every load is unconditional: a lane whose piece lies outside the
    // slice or the matrix reads the piece at the top of the slab / the left of the row instead (always valid) and
    // what it read is discarded (W: its mask word is zero; dY: zeroed when staged).  A load under a branch would
    // need its destination cleared first, and that write had the compiler wait for every load in flight.
    uint32_t woff[W_CHUNKS], woff_top[W_CHUNKS], xoff[X_CHUNKS], xoff_top[X_CHUNKS];
    int wrow[W_CHUNKS], xrow[X_CHUNKS];
    bool xcol_ok[X_CHUNKS];
#pragma unroll
    for (int c = 0; c < W_CHUNKS; ++c) {
        const int id = tid + kBwdThreads * c;
        wrow[c] = id / W_CPR;
        int pc = id % W_CPR;
        if (j0 + pc * 8 >= n) pc = 0; // n % 8 == 0: a piece is inside or outside as a whole; outside -> mask bits are 0
        woff[c] = (uint32_t)(((int64_t)wrow[c] * ldw + pc * 8) * 2);
        woff_top[c] = (uint32_t)(pc * 8 * 2);
    }
#pragma unroll
    for (int c = 0; c < X_CHUNKS; ++c) {
        const int id = (tid + kBwdThreads * c) % (BK * X_CPR); // lanes beyond the slab repeat earlier pieces
        xrow[c] = id / X_CPR;
        int nc = id % X_CPR;
        xcol_ok[c] = q0 + nc * 8 < N;
        if (!xcol_ok[c]) nc = 0;
        xoff[c] = (uint32_t)(((int64_t)xrow[c] * lddy + nc * 8) * 2);
        xoff_top[c] = (uint32_t)(nc * 8 * 2);
    }
    const char *wbase0 = (const char *)(W + ibeg * ldw + j0);
    const char *xbase0 = (const char *)(DY + ibeg * lddy + q0);
    int x_rows_left = 0; // rows of the slab whose dY pieces sit in xreg (for the zeroing at stage time)

    auto load_slab = [&](int slab) {
        const int rows_left = (int)(iend - ibeg) - slab * BK; // rows of this slab and beyond (>= 1)
        const char *wbase = wbase0 + (int64_t)slab * BK * ldw * 2;
        const char *xbase = xbase0 + (int64_t)slab * BK * lddy * 2;
#pragma unroll
        for (int c = 0; c < W_CHUNKS; ++c)
            wreg[c] = *reinterpret_cast<const uint4 *>(wbase + (wrow[c] < rows_left ? woff[c] : woff_top[c]));
#pragma unroll
        for (int c = 0; c < X_CHUNKS; ++c) {
            const char *src = xbase + (xrow[c] < rows_left ? xoff[c] : xoff_top[c]);
            if (XVEC) {
                xreg[c] = *reinterpret_cast<const uint4 *>(src); // N % 8 == 0
            } else {
                const uint16_t *h = reinterpret_cast<const uint16_t *>(src);
                const int room = N - q0 - ((tid + kBwdThreads * c) % X_CPR) * 8; // valid elements from this piece on
                uint16_t tmp[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) tmp[e] = h[(xcol_ok[c] && e < room) ? e : 0];
                xreg[c] = *reinterpret_cast<uint4 *>(tmp);
            }
        }
        x_rows_left = rows_left;
    };

    // FAST: tile column of the workgroup and the word offset of its 128 columns inside that tile's I_z rows
    const int tj = FAST ? j0 / g.c : 0;
    const int zw0 = FAST ? (j0 - tj * g.c) >> 5 : 0;
    // FAST: position of a slab's first row as (tile row, row inside the tile), advanced slab by slab without a
    // division (r % 64 == 0: a slab never straddles two tile rows)
    struct Cursor {
        int ti, o;
    };
    auto advance = [&](Cursor &c) {
        c.o += BK;
        if (c.o >= g.r) {
            c.o -= g.r;
            c.ti += 1;
        }
    };
    const uint32_t fz_off = (uint32_t)((((tid >> 2) * g.izw) + (tid & 3)) * 4); // lane's word of the I_z slice
    const uint32_t ip_off = (uint32_t)((tid >> 2) * g.ipw * 4);                 // lane's row of the slab's I_p rows
    // I_z rows of the tile row that slab `slab` (at cursor c) starts, when it starts one (or unconditionally):
    // global -> LDS
    auto fetch_fz = [&](int slab, const Cursor &c, bool always) {
        if (slab >= nslabs || !(always || c.o == 0)) return; // uniform over the workgroup
        const int64_t t = (int64_t)c.ti * g.tile_cols + tj;
        const char *base = (const char *)(Iz + t * g.k * (int64_t)g.izw + zw0);
        uint32_t *fz = Fz + (c.ti & 1) * S::fz_words;
        if (tid < g.k * 4) fz[tid] = *reinterpret_cast<const uint32_t *>(base + fz_off);
    };
    // I_p words (k <= 64: at most two) of this lane's row of slab `slab` (at cursor c).  Unconditional loads: a row
    // beyond the slice reads the slab's first row (its mask word is forced to zero in decode_slab); with one word
    // per row the second register repeats the first and is not looked at.
    auto load_ip = [&](int slab, const Cursor &c, uint32_t (&ipw)[2]) {
        if (slab >= nslabs) return; // uniform; the registers are not used for such a slab
        const int rows_left = (int)(iend - ibeg) - slab * BK;
        const int64_t t = (int64_t)c.ti * g.tile_cols + tj;
        const char *base = (const char *)(Ip + (t * g.r + c.o) * g.ipw);
        const uint32_t *ip = reinterpret_cast<const uint32_t *>(base + ((tid >> 2) < rows_left ? ip_off : 0u));
        ipw[0] = ip[0];
        ipw[1] = ip[g.ipw > 1 ? 1 : 0];
    };
    // one mask word per lane: (row of the slab, 32-column group of the workgroup's 128 columns)
    auto decode_slab = [&](int slab, int buf, int ti_fast, const uint32_t (&ipw)[2]) {
        uint32_t word = 0u;
        if (FAST) {
            const uint32_t *fz = Fz + (ti_fast & 1) * S::fz_words + (tid & 3);
            const int rows_left = (int)(iend - ibeg) - slab * BK;
            const bool live = (tid >> 2) < rows_left; // a row beyond the slice: its W piece is a stand-in, mask it out
#pragma unroll
            for (int iw = 0; iw < 2; ++iw) {
                uint32_t sel = (live && iw < g.ipw) ? ipw[iw] : 0u;
                while (sel) {
                    const int l = __builtin_ctz(sel) + 32 * iw;
                    sel &= sel - 1u;
                    word |= fz[l * 4];
                }
            }
        } else {
            const int64_t gi = ibeg + (int64_t)slab * BK + (tid >> 2);
            if (gi < iend) {
                const int ti = (int)(gi / g.r);
                const int il = (int)(gi - (int64_t)ti * g.r);
                word = decode_word(g, Ip, Iz, ti, il, (j0 >> 5) + (tid & 3));
            }
        }
        Ms[buf * S::ms_words + tid] = word;
    };

    auto stage_slab = [&](int buf) {
        uint16_t *ws = Ws + buf * S::ws_halfs;
        uint16_t *xs = Xs + buf * S::xs_halfs;
        const unsigned char *mb = (const unsigned char *)(Ms + buf * S::ms_words);
#pragma unroll
        for (int c = 0; c < W_CHUNKS; ++c) {
            const int id = tid + kBwdThreads * c;
            const int row = id / W_CPR, pc = id % W_CPR;
            const uint32_t bits = mb[row * (BJ / 8) + pc];
            *reinterpret_cast<uint4 *>(ws + row * WS_STRIDE + pc * 8) = apply_mask8(wreg[c], bits);
        }
#pragma unroll
        for (int c = 0; c < X_CHUNKS; ++c) {
            const int id = tid + kBwdThreads * c;
            if (id < BK * X_CPR) {
                const int row = id / X_CPR, nc = id % X_CPR;
                uint4 v = xreg[c];
                if (!(row < x_rows_left && xcol_ok[c])) v = make_uint4(0u, 0u, 0u, 0u);
                if (!XVEC) { // a piece that straddles N: zero its tail
                    const int room = N - q0 - nc * 8;
                    uint16_t *h = reinterpret_cast<uint16_t *>(&v);
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (e >= room) h[e] = 0;
                }
                *reinterpret_cast<uint4 *>(xs + row * XS_STRIDE + nc * 8) = v;
            }
        }
    };

    f32x16 acc[FQ][FJ];
#pragma unroll
    for (int a = 0; a < FQ; ++a)
#pragma unroll
        for (int b = 0; b < FJ; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // transposing read: 16-lane group G = lane / 16 serves columns 16 * (G % 2) .. + 15 of a 32-column
    // block and reduction group G / 2; lane d of the group addresses row d / 4, columns 4 * (d % 4)
    const int d16 = lane & 15, G16 = lane >> 4;
    const int frag_row = 8 * (G16 >> 1) + (d16 >> 2);
    const int frag_col = 16 * (G16 & 1) + 4 * (d16 & 3);
    const uint32_t wfrag_off = (uint32_t)(frag_row * WS_STRIDE + wj * WJ + frag_col);
    const uint32_t xfrag_off = (uint32_t)(frag_row * XS_STRIDE + wq * WQ + frag_col);

    // FAST: I_p words of the slabs in flight.  The words of slab x live in ip_even / ip_odd by the parity of x; the loop
    // is unrolled by two so that no register copy (which would wait for a load just requested) is needed.
    uint32_t ip_even[2] = {0u, 0u}, ip_odd[2] = {0u, 0u};
    Cursor c2{0, 0}, c3{0, 0}, c4{0, 0}; // slabs s + 2, s + 3, s + 4 of loop iteration s
    if (nslabs > 0) {
        uint32_t ip0[2] = {0u, 0u};
        Cursor c0{0, 0}, c1{0, 0};
        if (FAST) {
            c0.ti = (int)(ibeg / g.r);
            c0.o = (int)(ibeg - (int64_t)c0.ti * g.r);
            c1 = c0;
            advance(c1);
            c2 = c1;
            advance(c2);
            c3 = c2;
            advance(c3);
            c4 = c3;
            advance(c4);
            fetch_fz(0, c0, true);
            fetch_fz(1, c1, false);
            fetch_fz(2, c2, false);
            load_ip(0, c0, ip0);
            load_slab(0);
            __syncthreads();
            decode_slab(0, 0, c0.ti, ip0);
            load_ip(1, c1, ip_odd);
            load_ip(2, c2, ip_even);
        } else {
            load_slab(0);
            decode_slab(0, 0, 0, ip0);
        }
        __syncthreads();
        stage_slab(0);
        if (nslabs > 1) {
            load_slab(1);
            decode_slab(1, 1, c1.ti, ip_odd);
        }
        if (FAST) fetch_fz(3, c3, false);
        __syncthreads();
    }

    // one slab: multiply slab s, stage slab s + 1, request slab s + 2 and decode its mask words
    // (`use` holds its I_p words), request the I_p words of slab s + 3 into `next`
    auto iteration = [&](int s, const uint32_t (&use)[2], uint32_t (&next)[2]) __attribute__((always_inline)) {
        const int buf = s & 1;
        const uint16_t *ws = Ws + buf * S::ws_halfs + wfrag_off;
        const uint16_t *xs = Xs + buf * S::xs_halfs + xfrag_off;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            uint4 wf[FJ], xf[FQ];
#pragma unroll
            for (int b = 0; b < FJ; ++b) {
                const uint16_t *p = ws + (kk * 16) * WS_STRIDE + b * 32;
                const uint2 lo = lds_read_tr16(p);
                const uint2 hi = lds_read_tr16(p + 4 * WS_STRIDE);
                wf[b] = make_uint4(lo.x, lo.y, hi.x, hi.y);
            }
#pragma unroll
            for (int a = 0; a < FQ; ++a) {
                const uint16_t *p = xs + (kk * 16) * XS_STRIDE + a * 32;
                const uint2 lo = lds_read_tr16(p);
                const uint2 hi = lds_read_tr16(p + 4 * XS_STRIDE);
                xf[a] = make_uint4(lo.x, lo.y, hi.x, hi.y);
            }
#pragma unroll
            for (int a = 0; a < FQ; ++a)
#pragma unroll
                for (int b = 0; b < FJ; ++b) acc[a][b] = mfma_32x32x16(Tag{}, xf[a], wf[b], acc[a][b]);
        }
        if (s + 1 < nslabs) stage_slab(buf ^ 1);
        if (FAST) load_ip(s + 3, c3, next); // requested before the slab's own loads, used one iteration later
        if (s + 2 < nslabs) {
            load_slab(s + 2);
            decode_slab(s + 2, buf, c2.ti, use);
        }
        if (FAST) {
            fetch_fz(s + 4, c4, false);
            advance(c2);
            advance(c3);
            advance(c4);
        }
        __syncthreads();
    };
    for (int s = 0; s < nslabs; s += 2) {
        iteration(s, ip_even, ip_odd);     // slab s + 2 is even, slab s + 3 odd
        if (s + 1 < nslabs) iteration(s + 1, ip_odd, ip_even);
    }

    // epilogue: per 32x32 block the lane holds row (of dX) l32 and columns 8 * (v / 4) + 4 * lg + (v % 4)
#pragma unroll
    for (int a = 0; a < FQ; ++a) {
#pragma unroll
        for (int b = 0; b < FJ; ++b) {
            const int64_t row = j0 + wj * WJ + b * 32 + l32;
            if (row >= n) continue;
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int col = q0 + wq * WQ + a * 32 + 8 * v4 + 4 * lg;
                if (SPLIT) {
                    if (col < ldp) {
                        float4 o = make_float4(acc[a][b][4 * v4 + 0], acc[a][b][4 * v4 + 1], acc[a][b][4 * v4 + 2],
                                               acc[a][b][4 * v4 + 3]);
                        *reinterpret_cast<float4 *>(P + ((int64_t)slice * n + row) * ldp + col) = o;
                    }
                } else {
                    uint16_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = cvt_store(Tag{}, acc[a][b][4 * v4 + e]);
                    if (y_vec_ok && col + 3 < N) {
                        *reinterpret_cast<uint2 *>(DX + row * lddx + col) = *reinterpret_cast<uint2 *>(o);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < N) DX[row * lddx + col + e] = o[e];
                    }
                }
            }
        }
    }
}

// adds the partial planes of all slices in slice order and rounds to the storage dtype
template <typename Tag>
__global__ __launch_bounds__(256) void bwd_reduce_kernel(const float *__restrict__ P, int64_t ldp, int64_t rows, int N,
                                                         int slices, uint16_t *__restrict__ Y, int64_t ldy, int y_vec_ok)
{
    const int64_t groups_per_row = ldp / 4;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= rows * groups_per_row) return;
    const int64_t row = e / groups_per_row;
    const int col = (int)(e - row * groups_per_row) * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    const float *src = P + row * ldp + col;
    const int64_t plane = rows * ldp;
    int k = 0;
    // four slices at a time: their loads are in flight together, the additions stay in slice order
    for (; k + 4 <= slices; k += 4) {
        float4 p[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) p[q] = *reinterpret_cast<const float4 *>(src + (int64_t)(k + q) * plane);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            s.x += p[q].x;
            s.y += p[q].y;
            s.z += p[q].z;
            s.w += p[q].w;
        }
    }
    for (; k < slices; ++k) {
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
// dW = (dY X^T) o I_a on the matrix cores
// ---------------------------------------------------------------------------
struct SmemG {
    static constexpr int BI = 128;
    static constexpr int OP_STRIDE = BK + 8;  // halfs, operands [row][batch]
    static constexpr int CS_STRIDE = BJ + 8;  // halfs, output tile [row][column]
    static constexpr int op_halfs = 128 * OP_STRIDE;
    static constexpr int ms_words = BI * (BJ / 32);
    // one stage of both operands (the output tile reuses their space after the last slab) + mask words: 39 KB,
    // so that four workgroups share a compute unit.  Measured against two stages (75 KB, two workgroups, one
    // barrier per slab less): 36 us against 48 us on a batch of 128, 56 us against 60 us on a batch of 1024.
    static constexpr size_t op_bytes = 2 * (size_t)op_halfs * 2;
    static constexpr size_t cs_bytes = (size_t)BI * CS_STRIDE * 2;
    static constexpr size_t bytes = (op_bytes > cs_bytes ? op_bytes : cs_bytes) + (size_t)ms_words * 4;
};

template <typename Tag, bool VEC>
__global__ __launch_bounds__(kBwdThreads) void mfma_grad_kernel(Geom g, const uint16_t *__restrict__ DY, int64_t lddy,
                                                                const uint16_t *__restrict__ X, int64_t ldx, int N,
                                                                const uint32_t *__restrict__ Ip,
                                                                const uint32_t *__restrict__ Iz,
                                                                uint16_t *__restrict__ DW, int64_t lddw, int jblocks,
                                                                int w_vec_ok)
{
    using S = SmemG;
    constexpr int BI = S::BI;
    constexpr int OP_STRIDE = S::OP_STRIDE, CS_STRIDE = S::CS_STRIDE;
    constexpr int CHUNKS = 128 * (BK / 8) / kBwdThreads; // 16-byte pieces per lane, slab and operand
    constexpr int WI = 64, WJ = 64, FI = 2, FJ = 2;      // 2 x 2 wavefronts, 64 x 64 each

    extern __shared__ uint4 lrbi_dyn_smem[];
    uint16_t *As = (uint16_t *)lrbi_dyn_smem;            // [128][OP_STRIDE]  rows of dY
    uint16_t *Bs = As + S::op_halfs;                     // [128][OP_STRIDE]  rows of X
    uint16_t *Cs = (uint16_t *)lrbi_dyn_smem;            // [128][CS_STRIDE], after the last slab
    uint32_t *Ms = (uint32_t *)((char *)lrbi_dyn_smem + (S::op_bytes > S::cs_bytes ? S::op_bytes : S::cs_bytes));

    const int64_t bid = blockIdx.x;
    const int ji = (int)(bid % jblocks);
    const int64_t ii = bid / jblocks;
    const int64_t i0 = ii * BI;
    const int j0 = ji * BJ;
    const int n = (int)g.n;
    const int nslabs = (N + BK - 1) / BK;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wi = wave >> 1, wj = wave & 1;
    const int l32 = lane & 31, lg = lane >> 5;

    uint4 areg[CHUNKS], breg[CHUNKS];

    auto load_piece = [&](const uint16_t *base, int64_t ld, int64_t row, int64_t rows, int qq) -> uint4 {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (row < rows) {
            if (VEC) {
                if (qq < N) v = *reinterpret_cast<const uint4 *>(base + row * ld + qq); // N % 8 == 0
            } else {
                uint16_t tmp[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) tmp[e] = (qq + e < N) ? base[row * ld + qq + e] : (uint16_t)0;
                v = *reinterpret_cast<uint4 *>(tmp);
            }
        }
        return v;
    };
    // VEC: uniform base per slab + per-lane byte offsets (below 2^31: 128 rows of at most 2^22 elements) that are
    // recomputed per load from the lane's first row (registers are what limits the workgroups per compute unit),
    // every load unconditional: a lane whose row or batch column lies outside reads a valid stand-in (its row clamped
    // to the last one, batch column 0 of the slab) and the piece is cleared when it is staged
    const int row0 = tid >> 3;             // chunk c of this lane: row row0 + 32 c, 16-byte piece tid % 8
    const uint32_t kc16 = (uint32_t)((tid & 7) * 16);
    const int a_last = (int)((g.m - 1 - i0 < BI - 1) ? g.m - 1 - i0 : BI - 1); // last row of the block inside the matrix
    const int b_last = (int)((g.n - 1 - j0 < BJ - 1) ? g.n - 1 - j0 : BJ - 1);
    const uint32_t lda2 = (uint32_t)(lddy * 2), ldb2 = (uint32_t)(ldx * 2);
    const char *abase0 = (const char *)(DY + i0 * lddy);
    const char *bbase0 = (const char *)(X + (int64_t)j0 * ldx);
    int cols_left = 0; // batch columns from the first one of the slab whose pieces sit in areg / breg
    auto load_slab = [&](int slab) {
        const int k0 = slab * BK;
        if (VEC) {
            const char *abase = abase0 + (int64_t)k0 * 2;
            const char *bbase = bbase0 + (int64_t)k0 * 2;
            const uint32_t off = ((tid & 7) * 8 < N - k0) ? kc16 : 0u; // N % 8 == 0
#pragma unroll
            for (int c = 0; c < CHUNKS; ++c) {
                const int row = row0 + 32 * c;
                const uint32_t ar = (uint32_t)(row < a_last ? row : a_last), br = (uint32_t)(row < b_last ? row : b_last);
                areg[c] = *reinterpret_cast<const uint4 *>(abase + (ar * lda2 + off));
                breg[c] = *reinterpret_cast<const uint4 *>(bbase + (br * ldb2 + off));
            }
        } else {
#pragma unroll
            for (int c = 0; c < CHUNKS; ++c) {
                const int id = tid + kBwdThreads * c;
                const int row = id >> 3, kc = id & 7;
                areg[c] = load_piece(DY, lddy, i0 + row, g.m, k0 + kc * 8);
                breg[c] = load_piece(X, ldx, (int64_t)j0 + row, g.n, k0 + kc * 8);
            }
        }
        cols_left = N - k0;
    };
    auto stage_slab = [&]() {
        uint16_t *as = As;
        uint16_t *bs = Bs;
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            const int id = tid + kBwdThreads * c;
            const int row = id >> 3, kc = id & 7;
            uint4 av = areg[c], bv = breg[c];
            if (VEC) {
                const bool col_ok = kc * 8 < cols_left;
                if (!(row <= a_last && col_ok)) av = make_uint4(0u, 0u, 0u, 0u);
                if (!(row <= b_last && col_ok)) bv = make_uint4(0u, 0u, 0u, 0u);
            }
            *reinterpret_cast<uint4 *>(as + row * OP_STRIDE + kc * 8) = av;
            *reinterpret_cast<uint4 *>(bs + row * OP_STRIDE + kc * 8) = bv;
        }
    };

    f32x16 acc[FJ][FI];
#pragma unroll
    for (int a = 0; a < FJ; ++a)
#pragma unroll
        for (int b = 0; b < FI; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    load_slab(0); // requested first: the factor loads below queue up behind it
    // Mask words of the tile: 128 rows x 4 words, two per lane; needed only in the epilogue.
    // Tile shapes that line up with the block (it lies inside one tile, ranks up to 64): the block's slices of the
    // factors -- k rows x 4 words of I_z, 128 rows x ipw words of I_p -- are fetched with one independent load per
    // lane and parked in the mask array's own space; after the barrier below every lane forms its two mask words from
    // there (Eq. 3) into registers, and stores them behind the slab loop's first barrier, when nobody reads the
    // parked factors any more.  Other shapes: word by word from global memory (a chain of dependent loads).
    static_assert(S::ms_words == 2 * kBwdThreads && FAST_MAX_K * 4 <= kBwdThreads && BI * 2 <= kBwdThreads,
                  "factor slices fit the mask array, one load per lane and factor");
    // Tile widths that are an odd multiple of 64 (the 576-column tiles of Table 2), ranks up to 32: the block's upper
    // 64 columns may lie in the next tile column; words 2 and 3 of the I_z rows and a second set of I_p words (behind
    // the first one: one word per row) then come from that tile.
    const bool half = (g.c % BJ) != 0 && (g.c % 64) == 0 && g.k <= 32;
    const bool lined_up = ((g.c % BJ) == 0 || half) && (g.r % BI) == 0 && g.k <= FAST_MAX_K && !g.ragged;
    if (lined_up) {
        const int ti = (int)(i0 / g.r), tj = j0 / g.c;
        const int il0 = (int)(i0 - (int64_t)ti * g.r), coff = j0 - tj * g.c;
        const int64_t t = (int64_t)ti * g.tile_cols + tj;
        const int jb = (j0 + 64 < n) ? j0 + 64 : j0; // (a block whose upper half is past the matrix: stand-in, never stored)
        const int tjb = jb / g.c, coffb = jb - tjb * g.c;
        const int64_t tb = (int64_t)ti * g.tile_cols + tjb;
        const int w = tid & 3;
        uint32_t fzv = 0u, fpv = 0u;
        if (tid < g.k * 4)
            fzv = (half && w >= 2) ? Iz[(tb * g.k + (tid >> 2)) * g.izw + (coffb >> 5) + (w - 2)]
                                   : Iz[(t * g.k + (tid >> 2)) * g.izw + (coff >> 5) + w];
        if (tid < BI * g.ipw) fpv = Ip[(t * g.r + il0) * g.ipw + tid];
        else if (half) fpv = Ip[(tb * g.r + il0) + (tid - BI)];
        Ms[tid] = fzv;               // [k][4]
        Ms[kBwdThreads + tid] = fpv; // [128][ipw]; half: [2][128]
    }
    // this lane's two mask words
    auto mask_word = [&](int c) -> uint32_t {
        const int idx = tid + kBwdThreads * c;
        uint32_t word = 0u;
        if (lined_up) {
            const int row = idx >> 2, w = idx & 3;
            const int pbase = kBwdThreads + ((half && w >= 2) ? BI : 0);
            for (int iw = 0; iw < g.ipw; ++iw) {
                uint32_t sel = Ms[pbase + row * g.ipw + iw];
                while (sel) {
                    const int l = __builtin_ctz(sel) + 32 * iw;
                    sel &= sel - 1u;
                    word |= Ms[l * 4 + w];
                }
            }
        } else {
            const int64_t gi = i0 + (idx >> 2);
            if (gi < g.m) {
                const int ti = (int)(gi / g.r);
                const int il = (int)(gi - (int64_t)ti * g.r);
                word = decode_word(g, Ip, Iz, ti, il, (j0 >> 5) + (idx & 3));
            }
        }
        return word;
    };
    uint32_t mw0 = 0u, mw1 = 0u;
    if (!lined_up) { // from global memory: asked for before the wait for the operands
        mw0 = mask_word(0);
        mw1 = mask_word(1);
    }

    stage_slab();
    if (nslabs > 1) load_slab(1);
    __syncthreads();
    if (lined_up) { // from the parked factors, visible now
        mw0 = mask_word(0);
        mw1 = mask_word(1);
    }

    for (int s = 0; s < nslabs; ++s) {
        const uint16_t *as = As + (wi * WI + l32) * OP_STRIDE + 8 * lg;
        const uint16_t *bs = Bs + (wj * WJ + l32) * OP_STRIDE + 8 * lg;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            uint4 af[FI], bf[FJ];
#pragma unroll
            for (int b = 0; b < FI; ++b) af[b] = *reinterpret_cast<const uint4 *>(as + b * 32 * OP_STRIDE + kk * 16);
#pragma unroll
            for (int a = 0; a < FJ; ++a) bf[a] = *reinterpret_cast<const uint4 *>(bs + a * 32 * OP_STRIDE + kk * 16);
#pragma unroll
            for (int a = 0; a < FJ; ++a)
#pragma unroll
                for (int b = 0; b < FI; ++b) acc[a][b] = mfma_32x32x16(Tag{}, bf[a], af[b], acc[a][b]);
        }
        __syncthreads(); // everyone has read the stage before it is overwritten
        if (s == 0) { // ... and the parked factors: the mask words take their place
            Ms[tid] = mw0;
            Ms[tid + kBwdThreads] = mw1;
        }
        if (s + 1 < nslabs) stage_slab();
        if (s + 2 < nslabs) load_slab(s + 2);
        __syncthreads();
    }

    // the fp32 tile, rounded, into LDS (the operand buffers are free after the barrier above):
    // per 32x32 block the lane holds row l32 (of dW) and columns 8 * (v / 4) + 4 * lg + (v % 4)
#pragma unroll
    for (int a = 0; a < FJ; ++a) {
#pragma unroll
        for (int b = 0; b < FI; ++b) {
            const int row = wi * WI + b * 32 + l32;
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int col = wj * WJ + a * 32 + 8 * v4 + 4 * lg;
                uint16_t o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = cvt_store(Tag{}, acc[a][b][4 * v4 + e]);
                *reinterpret_cast<uint2 *>(Cs + row * CS_STRIDE + col) = *reinterpret_cast<uint2 *>(o);
            }
        }
    }
    __syncthreads();
    // masked, coalesced write: 16 pieces of 16 bytes per row
    const unsigned char *mb = (const unsigned char *)Ms;
#pragma unroll
    for (int c = 0; c < BI * (BJ / 8) / kBwdThreads; ++c) {
        const int id = tid + kBwdThreads * c;
        const int row = id >> 4, pc = id & 15;
        const int64_t gi = i0 + row;
        const int jj = j0 + pc * 8;
        if (gi >= g.m || jj >= n) continue;
        const uint4 v = apply_mask8(*reinterpret_cast<const uint4 *>(Cs + row * CS_STRIDE + pc * 8),
                                    (uint32_t)mb[row * (BJ / 8) + pc]);
        if (w_vec_ok && jj + 8 <= n) {
            *reinterpret_cast<uint4 *>(DW + gi * lddw + jj) = v;
        } else {
            const uint16_t *h = reinterpret_cast<const uint16_t *>(&v);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (jj + e < n) DW[gi * lddw + jj + e] = h[e];
        }
    }
}

// ---------------------------------------------------------------------------
// Vector-ALU kernels: any dtype, shape and alignment; plain and slow
// ---------------------------------------------------------------------------
template <typename T> struct BwdElem;
template <> struct BwdElem<float> {
    __device__ static float to_f32(float v) { return v; }
    __device__ static float from_f32(float v) { return v; }
};
template <> struct BwdElem<__half> {
    __device__ static float to_f32(__half v) { return __half2float(v); }
    __device__ static __half from_f32(float v) { return __float2half_rn(v); }
};
template <> struct BwdElem<__hip_bfloat16> {
    __device__ static float to_f32(__hip_bfloat16 v) { return __bfloat162float(v); }
    __device__ static __hip_bfloat16 from_f32(float v) { return __float2bfloat16(v); }
};

// One wavefront per 64 columns of W and 4 batch columns: lane = column j, loop over the rows of W.
template <typename T>
__global__ __launch_bounds__(64) void valu_gemm_t_kernel(Geom g, const T *__restrict__ W, int64_t ldw,
                                                         const uint32_t *__restrict__ Ip,
                                                         const uint32_t *__restrict__ Iz, const T *__restrict__ DY,
                                                         int64_t lddy, int N, T *__restrict__ DX, int64_t lddx)
{
    constexpr int NB = 4;
    const int64_t j = (int64_t)blockIdx.x * 64 + threadIdx.x;
    const int q0 = blockIdx.y * NB;
    const int nb = (N - q0 < NB) ? N - q0 : NB;
    float acc[NB] = {0.f, 0.f, 0.f, 0.f};
    const bool live = j < g.n;
    const int64_t jc = live ? j : g.n - 1; // clamped: every lane walks the same rows
    for (int64_t i = 0; i < g.m; ++i) {
        const int ti = (int)(i / g.r);
        const int il = (int)(i - (int64_t)ti * g.r);
        const uint32_t word = decode_word(g, Ip, Iz, ti, il, (int)(jc >> 5));
        if (!live || !((word >> (jc & 31)) & 1u)) continue; // pruned: the stored value is never read
        const float w = BwdElem<T>::to_f32(W[i * ldw + j]);
#pragma unroll
        for (int b = 0; b < NB; ++b)
            if (b < nb) acc[b] = fmaf(w, BwdElem<T>::to_f32(DY[i * lddy + q0 + b]), acc[b]);
    }
    if (live)
        for (int b = 0; b < nb; ++b) DX[j * lddx + q0 + b] = BwdElem<T>::from_f32(acc[b]);
}

// One wavefront per row of W and 64 columns: lane = column j, loop over the batch.
template <typename T>
__global__ __launch_bounds__(64) void valu_grad_kernel(Geom g, const T *__restrict__ DY, int64_t lddy,
                                                       const T *__restrict__ X, int64_t ldx, int N,
                                                       const uint32_t *__restrict__ Ip,
                                                       const uint32_t *__restrict__ Iz, T *__restrict__ DW,
                                                       int64_t lddw)
{
    const int64_t j = (int64_t)blockIdx.x * 64 + threadIdx.x;
    if (j >= g.n) return;
    for (int64_t i = blockIdx.y; i < g.m; i += gridDim.y) {
        const int ti = (int)(i / g.r);
        const int il = (int)(i - (int64_t)ti * g.r);
        const uint32_t word = decode_word(g, Ip, Iz, ti, il, (int)(j >> 5));
        float s = 0.f;
        if ((word >> (j & 31)) & 1u)
            for (int q = 0; q < N; ++q)
                s = fmaf(BwdElem<T>::to_f32(DY[i * lddy + q]), BwdElem<T>::to_f32(X[j * ldx + q]), s);
        DW[i * lddw + j] = BwdElem<T>::from_f32(s); // pruned: exactly zero
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
BwdPlan plan_gemm_t(const Geom &g, lrbi_dtype dt, int64_t N, bool aligned)
{
    BwdPlan p;
    // (also the narrowest batches: the vector-ALU kernel walks the m rows one by one per lane, with a chain of dependent
    // factor loads per row: 3.9 ms on a 4096 x 9216 matrix at one column, where the tile kernel takes 26 us)
    p.mfma = (dt != LRBI_F32) && aligned && N >= 1;
    p.bq = (N > 32) ? 128 : 32;
    p.slices = 1;
    p.iper = g.m;
    p.workspace_bytes = 0;
    if (!p.mfma) return p;
    const int64_t jblocks = (g.n + BJ - 1) / BJ, qblocks = (N + p.bq - 1) / p.bq;
    const int64_t tiles = jblocks * qblocks;
    const int64_t islabs = (g.m + BK - 1) / BK;
    // two workgroups fit a compute unit: at most 512 run at once, and one more than that costs a second round
    int64_t want = 512 / tiles;
    const int64_t cap = islabs / 4 > 1 ? islabs / 4 : 1; // at least four slabs per slice
    if (want > cap) want = cap;
    if (want > 64) want = 64;
    if (want < 1) want = 1;
    const int64_t slabs_per = (islabs + want - 1) / want;
    p.slices = (int)((islabs + slabs_per - 1) / slabs_per);
    p.iper = slabs_per * BK;
    const int64_t ldp = (N + 3) / 4 * 4;
    p.workspace_bytes = (p.slices > 1) ? (uint64_t)p.slices * (uint64_t)g.n * (uint64_t)ldp * 4u : 0u;
    return p;
}

template <typename Tag, int BQ, int WAVES_J, int WAVES_Q>
static int launch_gemm_t_tile(const Geom &g, const BwdPlan &plan, const void *dW, int64_t ldw, const uint32_t *dIp,
                              const uint32_t *dIz, const void *dDY, int64_t lddy, int64_t N, void *dDX, int64_t lddx,
                              void *dWorkspace, hipStream_t stream)
{
    const int64_t jblocks = (g.n + BJ - 1) / BJ, qblocks = (N + BQ - 1) / BQ;
    const int64_t blocks = jblocks * qblocks * plan.slices;
    if (blocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    const bool xvec = (((uintptr_t)dDY & 15) == 0) && (lddy % 8 == 0) && (N % 8 == 0);
    const bool split = plan.slices > 1;
    const int y_vec_ok = (((uintptr_t)dDX & 7) == 0) && (lddx % 4 == 0);
    const int64_t ldp = (N + 3) / 4 * 4;
    const size_t smem = SmemT<BQ>::bytes;
    const int xcd_remap = (blocks % 8 == 0) ? 1 : 0;
    const bool fast = (g.c % 128 == 0) && (g.r % BK == 0) && (g.r >= 2 * BK) && (g.k <= FAST_MAX_K) && !g.ragged;
#define LRBI_LAUNCH_T(XV, SP)                                                                                      \
    do {                                                                                                           \
        auto kern = fast ? mfma_gemm_t_kernel<Tag, BQ, WAVES_J, WAVES_Q, XV, SP, true>                              \
                         : mfma_gemm_t_kernel<Tag, BQ, WAVES_J, WAVES_Q, XV, SP, false>;                            \
        LRBI_SET_MAX_LDS(kern, smem);                                                                              \
        LRBI_LAUNCH(kern, dim3((unsigned)blocks), dim3(kBwdThreads), smem, stream, g, (const uint16_t *)dW, \
                           ldw, dIp, dIz, (const uint16_t *)dDY, lddy, (int)N, (uint16_t *)dDX, lddx,              \
                           (float *)dWorkspace, ldp, (int)jblocks, (int)qblocks, plan.iper, xcd_remap, y_vec_ok);  \
    } while (0)
    if (xvec) {
        if (split) LRBI_LAUNCH_T(true, true);
        else LRBI_LAUNCH_T(true, false);
    } else {
        if (split) LRBI_LAUNCH_T(false, true);
        else LRBI_LAUNCH_T(false, false);
    }
#undef LRBI_LAUNCH_T
    if (split) {
        const int64_t items = g.n * (ldp / 4);
        const int64_t rblocks = (items + 255) / 256;
        if (rblocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
        LRBI_LAUNCH(bwd_reduce_kernel<Tag>, dim3((unsigned)rblocks), dim3(256), 0, stream,
                           (const float *)dWorkspace, ldp, g.n, (int)N, plan.slices, (uint16_t *)dDX, lddx, y_vec_ok);
    }
    return LRBI_OK;
}

template <typename T>
static int launch_valu_t(const Geom &g, const void *dW, int64_t ldw, const uint32_t *dIp, const uint32_t *dIz,
                         const void *dDY, int64_t lddy, int64_t N, void *dDX, int64_t lddx, hipStream_t stream)
{
    const int64_t bx = (g.n + 63) / 64, by = (N + 3) / 4;
    if (bx > 0x7FFFFFFF || by > 65535) return LRBI_ERR_SHAPE;
    LRBI_LAUNCH(valu_gemm_t_kernel<T>, dim3((unsigned)bx, (unsigned)by), dim3(64), 0, stream, g, (const T *)dW, ldw,
                       dIp, dIz, (const T *)dDY, lddy, (int)N, (T *)dDX, lddx);
    return LRBI_OK;
}

int launch_gemm_t(const Geom &g, const BwdPlan &plan, lrbi_dtype dt, const void *dW, int64_t ldw, const uint32_t *dIp,
                  const uint32_t *dIz, const void *dDY, int64_t lddy, int64_t N, void *dDX, int64_t lddx,
                  void *dWorkspace, hipStream_t stream)
{
    if (!plan.mfma) {
        switch (dt) {
        case LRBI_F32: return launch_valu_t<float>(g, dW, ldw, dIp, dIz, dDY, lddy, N, dDX, lddx, stream);
        case LRBI_F16: return launch_valu_t<__half>(g, dW, ldw, dIp, dIz, dDY, lddy, N, dDX, lddx, stream);
        case LRBI_BF16: return launch_valu_t<__hip_bfloat16>(g, dW, ldw, dIp, dIz, dDY, lddy, N, dDX, lddx, stream);
        default: return LRBI_ERR_DTYPE;
        }
    }
    // tile shapes that line up with its blocking: the pipelined kernel (both operands straight into LDS)
    if (plan.bq == 128 && pipe_t_ok(g, dW, ldw, dIz, dDY, lddy, N)) {
        int64_t iper = g.m;
        const int slices = pipe_t_slices(g, N, plan.slices, &iper);
        const int rc = launch_pipe_t_gemm(g, slices, iper, dt, dW, ldw, dIp, dIz, dDY, lddy, N, dDX, lddx, dWorkspace,
                                          stream);
        if (rc != LRBI_OK || slices == 1) return rc;
        const int64_t ldp = (N + 3) / 4 * 4;
        const int y_vec_ok = (((uintptr_t)dDX & 7) == 0) && (lddx % 4 == 0);
        const int64_t rblocks = (g.n * (ldp / 4) + 255) / 256;
        if (rblocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
        if (dt == LRBI_F16)
            LRBI_LAUNCH(bwd_reduce_kernel<F16Tag>, dim3((unsigned)rblocks), dim3(256), 0, stream,
                        (const float *)dWorkspace, ldp, g.n, (int)N, slices, (uint16_t *)dDX, lddx, y_vec_ok);
        else
            LRBI_LAUNCH(bwd_reduce_kernel<BF16Tag>, dim3((unsigned)rblocks), dim3(256), 0, stream,
                        (const float *)dWorkspace, ldp, g.n, (int)N, slices, (uint16_t *)dDX, lddx, y_vec_ok);
        return LRBI_OK;
    }
#define LRBI_T_ARGS g, plan, dW, ldw, dIp, dIz, dDY, lddy, N, dDX, lddx, dWorkspace, stream
    if (dt == LRBI_F16) {
        if (plan.bq == 128) return launch_gemm_t_tile<F16Tag, 128, 2, 2>(LRBI_T_ARGS);
        return launch_gemm_t_tile<F16Tag, 32, 4, 1>(LRBI_T_ARGS);
    }
    if (plan.bq == 128) return launch_gemm_t_tile<BF16Tag, 128, 2, 2>(LRBI_T_ARGS);
    return launch_gemm_t_tile<BF16Tag, 32, 4, 1>(LRBI_T_ARGS);
#undef LRBI_T_ARGS
}

template <typename T>
static int launch_valu_grad(const Geom &g, const void *dDY, int64_t lddy, const void *dX, int64_t ldx, int64_t N,
                            const uint32_t *dIp, const uint32_t *dIz, void *dDW, int64_t lddw, hipStream_t stream)
{
    const int64_t bx = (g.n + 63) / 64;
    if (bx > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    const unsigned by = (unsigned)(g.m < 65535 ? g.m : 65535);
    LRBI_LAUNCH(valu_grad_kernel<T>, dim3((unsigned)bx, by), dim3(64), 0, stream, g, (const T *)dDY, lddy,
                       (const T *)dX, ldx, (int)N, dIp, dIz, (T *)dDW, lddw);
    return LRBI_OK;
}

int launch_grad(const Geom &g, lrbi_dtype dt, bool mfma, const void *dDY, int64_t lddy, const void *dX, int64_t ldx,
                int64_t N, const uint32_t *dIp, const uint32_t *dIz, void *dDW, int64_t lddw, hipStream_t stream)
{
    if (!mfma) {
        switch (dt) {
        case LRBI_F32: return launch_valu_grad<float>(g, dDY, lddy, dX, ldx, N, dIp, dIz, dDW, lddw, stream);
        case LRBI_F16: return launch_valu_grad<__half>(g, dDY, lddy, dX, ldx, N, dIp, dIz, dDW, lddw, stream);
        case LRBI_BF16: return launch_valu_grad<__hip_bfloat16>(g, dDY, lddy, dX, ldx, N, dIp, dIz, dDW, lddw, stream);
        default: return LRBI_ERR_DTYPE;
        }
    }
    const int64_t iblocks = (g.m + 127) / 128, jblocks = (g.n + BJ - 1) / BJ;
    const int64_t blocks = iblocks * jblocks;
    if (blocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    const bool vec = (((uintptr_t)dDY & 15) == 0) && (lddy % 8 == 0) && (((uintptr_t)dX & 15) == 0) && (ldx % 8 == 0) &&
                     (N % 8 == 0) && lddy < ((int64_t)1 << 22) && ldx < ((int64_t)1 << 22);
    const int w_vec_ok = (((uintptr_t)dDW & 15) == 0) && (lddw % 8 == 0);
    const size_t smem = SmemG::bytes;
#define LRBI_LAUNCH_G(TAG, V)                                                                                      \
    do {                                                                                                           \
        auto kern = mfma_grad_kernel<TAG, V>;                                                                      \
        LRBI_SET_MAX_LDS(kern, smem);                                                                              \
        LRBI_LAUNCH(kern, dim3((unsigned)blocks), dim3(kBwdThreads), smem, stream, g, (const uint16_t *)dDY, \
                           lddy, (const uint16_t *)dX, ldx, (int)N, dIp, dIz, (uint16_t *)dDW, lddw, (int)jblocks,  \
                           w_vec_ok);                                                                              \
    } while (0)
    if (dt == LRBI_F16) {
        if (vec) LRBI_LAUNCH_G(F16Tag, true);
        else LRBI_LAUNCH_G(F16Tag, false);
    } else {
        if (vec) LRBI_LAUNCH_G(BF16Tag, true);
        else LRBI_LAUNCH_G(BF16Tag, false);
    }
#undef LRBI_LAUNCH_G
    return LRBI_OK;
}

} // namespace lrbi
