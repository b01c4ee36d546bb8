// Candidate evaluation of Algorithm 1 (Sec. 2.1): threshold the real-valued factors of every
// tile, form I_a = I_p (x) I_z (Eq. 3) on chip, and return per tile the number of ones of I_a
// and the cost (sum of the magnitudes that magnitude pruning keeps and I_a prunes).
//
// One workgroup per tile, or per band of rows of a tile when the tiles alone would not fill the chip
// (the bands' partial results then go through a caller-provided workspace).
//   1. The tile's M_z (k x c floats) and M_p (r x k floats) are compared with the tile's
//      thresholds; the resulting bits go to LDS in the packed layouts (I_z rows of
//      2 * ceil(c / 64) words, I_p rows of ceil(k / 32) words) and, when asked for, to global
//      memory as the packed factors.
//   2. The tile is walked as a row-major list of 16-byte pieces of W (8 columns of a 16-bit
//      type, 4 of fp32), four pieces per lane in flight.  For a piece the lane rebuilds the
//      32-bit mask word over it (OR of the I_z words selected by the set bits of the row's I_p
//      words, all from LDS), counts the ones, and adds |w| for every column with w kept by
//      magnitude and pruned by the mask.  Per-lane sums are kept in double; lanes, then
//      wavefronts, are added in a fixed order.  For the usual tile widths (a power of two of
//      whole 32-column words per row) a lane keeps its word column and walks down the rows
//      instead: one mask look-up per 32 columns, constant offsets; for the 16-bit types the
//      weights the mask keeps are cleared with a packed 16-bit multiply before the magnitude test.
// The roofline is the single sweep over W (HBM); measured, the kernel is bound by vector-ALU
// issue (about five instructions per weight plus the mask look-up per piece).
//
// The same file holds the threshold search of Algorithm 1 that drives this kernel (further down).
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <math.h>

#include "lrbi_internal.hpp"
#include "lrbi_mfma_common.hpp"

namespace lrbi {

static constexpr int kEvalThreads = 512;
static constexpr int kEvalWaves = kEvalThreads / 64;

template <typename T> struct Mag;
template <> struct Mag<float> {
    static constexpr int VEC = 4;
};
template <> struct Mag<__half> {
    static constexpr int VEC = 8;
};
template <> struct Mag<__hip_bfloat16> {
    static constexpr int VEC = 8;
};

// magnitude of element e of a 16-byte piece, exact in fp32
template <typename T> __device__ __forceinline__ float piece_abs(const uint32_t (&w)[4], int e);
template <> __device__ __forceinline__ float piece_abs<float>(const uint32_t (&w)[4], int e)
{
    return fabsf(__builtin_bit_cast(float, w[e]));
}
template <> __device__ __forceinline__ float piece_abs<__half>(const uint32_t (&w)[4], int e)
{
    const uint16_t h = (uint16_t)((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xFFFFu));
    return fabsf(__half2float(__builtin_bit_cast(__half, h)));
}
template <> __device__ __forceinline__ float piece_abs<__hip_bfloat16>(const uint32_t (&w)[4], int e)
{
    const uint32_t h = (e & 1) ? (w[e >> 1] & 0xFFFF0000u) : (w[e >> 1] << 16);
    return fabsf(__builtin_bit_cast(float, h));
}

// per-tile state of the threshold search
struct SearchState {
    double lo, hi, sz;     // bisection interval and current probe of S_z
    double rep_cost;       // representative of the current S_p: the probe closest to the target
    long long rep_diff;    // |ones - target| of the representative, -1 = none yet
    unsigned long long rep_kept;
    float rep_tz;
    float tp;              // threshold of I_p for the current S_p
    long long best_diff;   // winner so far, -1 = none
    int best_eligible;
    int pad;
};

// rows x columns of tile t's part inside the matrix
__device__ __forceinline__ void tile_extent(const Geom &g, int64_t t, int &rt, int &ct)
{
    const int64_t ti = t / g.tile_cols, tj = t - ti * g.tile_cols;
    rt = (int)((g.m - ti * g.r < g.r) ? g.m - ti * g.r : g.r);
    ct = (int)((g.n - tj * g.c < g.c) ? g.n - tj * g.c : g.c);
}

// entry of the sorted factor at index round(sparsity * count): entries below it become 0
__device__ __forceinline__ float threshold_at(const float *sorted, int count, double sparsity)
{
    // separate multiply and add (no fused operation): the index must be the same as in plain double arithmetic
    long long idx = (long long)floor(__dadd_rn(__dmul_rn(sparsity, (double)count), 0.5));
    if (idx < 0) idx = 0;
    return (idx >= count) ? __builtin_inff() : sorted[idx];
}

// What the threshold search (further down) does with a tile's result after every probe.  It runs in the evaluation
// itself: by the lane that has just written the tile's ones and cost (one workgroup per tile), or by the lane that
// adds the bands of the tile, so a probe costs no launch of its own for this.  st == nullptr: plain evaluation.
struct SearchStepArgs {
    SearchState *st;
    const float *sortedMz;
    int64_t stride_z;
    double keep_fraction;  // 1 - S
    long long tolerance;
    int last_step;
    float *Tz;             // the thresholds being probed: read, then replaced by the next probe's
    float *TpBest, *TzBest;
    unsigned long long *KeptBest;
    double *CostBest;
};

__device__ __forceinline__ void search_step_tile(const Geom &g, const SearchStepArgs &a, int64_t t, unsigned long long kept,
                                                 double cost)
{
    int rt, ct;
    tile_extent(g, t, rt, ct);
    // target number of ones of this tile, round((1 - S) rt ct), in plain double arithmetic
    const long long target =
        (long long)floor(__dadd_rn(__dmul_rn(__dmul_rn(a.keep_fraction, (double)rt), (double)ct), 0.5));
    SearchState s = a.st[t];
    const long long k = (long long)kept;
    const long long diff = (k > target) ? k - target : target - k;
    if (s.rep_diff < 0 || diff < s.rep_diff) {
        s.rep_diff = diff;
        s.rep_tz = a.Tz[t];
        s.rep_kept = kept;
        s.rep_cost = cost;
    }
    if (k > target) s.lo = s.sz; // too many ones: I_z must get sparser
    else s.hi = s.sz;
    s.sz = 0.5 * (s.lo + s.hi);
    a.Tz[t] = threshold_at(a.sortedMz + t * a.stride_z, g.k * ct, s.sz);
    if (a.last_step) {
        const int eligible = s.rep_diff <= a.tolerance;
        bool better;
        if (s.best_diff < 0) better = true;
        else if (eligible != s.best_eligible) better = eligible != 0;
        else if (eligible) better = s.rep_cost < a.CostBest[t];
        else better = s.rep_diff < s.best_diff;
        if (better) {
            s.best_diff = s.rep_diff;
            s.best_eligible = eligible;
            a.TpBest[t] = s.tp;
            a.TzBest[t] = s.rep_tz;
            a.KeptBest[t] = s.rep_kept;
            a.CostBest[t] = s.rep_cost;
        }
    }
    a.st[t] = s;
}

// one addend of the cost, in double (a magnitude and its square are exact there)
template <bool SQ> __device__ __forceinline__ void cost_add(double &acc, float a)
{
    const double d = (double)a;
    if (SQ) acc = __fma_rn(d, d, acc);
    else acc += d;
}

// SQ: the cost sums squared magnitudes (manipulation method 2); cost_scale multiplies a workgroup's sum (method 3:
// every counted weight is one that magnitude pruning keeps, i.e. an amplified one, so the factor is common)
template <typename T, bool SQ>
__global__ __launch_bounds__(kEvalThreads) void threshold_eval_kernel(Geom g, const T *__restrict__ W, int64_t ldw,
                                                                      float w_threshold, double cost_scale,
                                                                      const float *__restrict__ Mp,
                                                                      const float *__restrict__ Mz,
                                                                      const float *__restrict__ Tp,
                                                                      const float *Tz, // may be step.Tz
                                                                      uint32_t *__restrict__ IpOut,
                                                                      uint32_t *__restrict__ IzOut,
                                                                      unsigned long long *__restrict__ Kept,
                                                                      double *__restrict__ Cost, int w_vec_ok,
                                                                      int bands, int rows_per_band, SearchStepArgs step)
{
    constexpr int VEC = Mag<T>::VEC;
    extern __shared__ uint4 lrbi_dyn_smem[];
    uint32_t *iz = reinterpret_cast<uint32_t *>(lrbi_dyn_smem); // [k][izw]
    uint32_t *ip = iz + g.k * g.izw;                            // [r][ipw]
    static __shared__ double wave_cost[kEvalWaves];
    static __shared__ unsigned long long wave_kept[kEvalWaves];

    // workgroup = (tile, band of rows); with several bands per tile the results are partial sums
    // (one slot per workgroup) that a second kernel adds in band order
    const int64_t t = blockIdx.x / bands;
    const int band = (int)(blockIdx.x - t * bands);
    const int ti = (int)(t / g.tile_cols), tj = (int)(t - (int64_t)ti * g.tile_cols);
    // the part of the tile inside the matrix (an edge tile may be cut off): rt x ct
    const int rt = (int)((g.m - (int64_t)ti * g.r < g.r) ? g.m - (int64_t)ti * g.r : g.r);
    const int ct = (int)((g.n - (int64_t)tj * g.c < g.c) ? g.n - (int64_t)tj * g.c : g.c);
    const int row_lo = band * rows_per_band;
    const int band_hi = (row_lo + rows_per_band < g.r) ? row_lo + rows_per_band : g.r; // rows of the stored factor
    const int row_hi = (band_hi < rt) ? band_hi : rt;
    const int nrows = (row_hi > row_lo) ? row_hi - row_lo : 0;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float tp = Tp[t], tz = Tz[t];

    // ---- 1. binary factors of the tile
    // I_z: a wavefront compares 64 consecutive entries of one row of M_z per step (one coalesced
    // read) and the 64 outcomes, gathered across the lanes, are the two packed words of that step;
    // eight steps' reads are requested together
    const float *mz = Mz + t * (int64_t)g.k * g.c;
    const int steps_per_row = g.izw / 2;
    const int zsteps = g.k * steps_per_row;
    constexpr int ZB = 8;
    for (int st0 = wave; st0 < zsteps; st0 += ZB * kEvalWaves) {
        float v[ZB];
        bool ok[ZB];
#pragma unroll
        for (int q = 0; q < ZB; ++q) {
            const int st = st0 + q * kEvalWaves;
            const int l = st / steps_per_row, sq = st - l * steps_per_row;
            const int j = 64 * sq + lane;
            ok[q] = (st < zsteps) && (j < ct); // columns a cut-off tile leaves outside the matrix stay 0
            v[q] = ok[q] ? mz[(int64_t)l * g.c + j] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < ZB; ++q) {
            const int st = st0 + q * kEvalWaves;
            if (st < zsteps) { // uniform over the wavefront
                const int l = st / steps_per_row, sq = st - l * steps_per_row;
                const unsigned long long b = __ballot(ok[q] && v[q] >= tz);
                if (lane < 2) {
                    const uint32_t bits = (uint32_t)(lane ? (b >> 32) : b);
                    iz[l * g.izw + 2 * sq + lane] = bits;
                    if (IzOut && band == 0) IzOut[(t * g.k + l) * (int64_t)g.izw + 2 * sq + lane] = bits;
                }
            }
        }
    }
    // I_p: one lane per (row, 32-bit word); its up to 32 entries are read eight at a time
    const float *mp = Mp + (t * (int64_t)g.r + row_lo) * g.k;
    for (int idx = tid; idx < nrows * g.ipw; idx += kEvalThreads) {
        const int i = idx / g.ipw, wq = idx - i * g.ipw; // row of the band
        uint32_t bits = 0u;
        const int l0 = 32 * wq;
        const float *mrow = mp + (int64_t)i * g.k;
        for (int b0 = 0; b0 < 32 && l0 + b0 < g.k; b0 += 8) {
            float v[8];
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const int l = l0 + b0 + b;
                v[b] = mrow[l < g.k ? l : g.k - 1]; // clamped: always a valid address
            }
#pragma unroll
            for (int b = 0; b < 8; ++b)
                if (l0 + b0 + b < g.k && v[b] >= tp) bits |= 1u << (b0 + b);
        }
        ip[idx] = bits;
        if (IpOut) IpOut[(t * g.r + row_lo + i) * (int64_t)g.ipw + wq] = bits;
    }
    // stored rows of I_p that a cut-off tile leaves outside the matrix are written as zero
    if (IpOut)
        for (int idx = nrows * g.ipw + tid; idx < (band_hi - row_lo) * g.ipw; idx += kEvalThreads)
            IpOut[(t * g.r + row_lo) * (int64_t)g.ipw + idx] = 0u;
    __syncthreads();

    // ---- 2. the tile as a list of 16-byte pieces (row-major): ones of I_a, and magnitudes kept by
    // pruning but cleared by I_a.  Four pieces per lane are in flight: their W loads are issued
    // before the first is consumed (the loads do not depend on the mask).
    // four partial sums per lane (element e of a piece goes to sum e mod 4): the double-precision additions of a
    // piece then form four short dependency chains instead of one long one
    double cost4[4] = {0.0, 0.0, 0.0, 0.0};
    unsigned long long kept = 0ull;
    const int64_t col0 = (int64_t)tj * g.c;
    const int P = (ct + VEC - 1) / VEC;    // pieces per row of the tile's part inside the matrix
    const int items = nrows * P;
    const bool p_pow2 = (P & (P - 1)) == 0;
    const int p_shift = 31 - __builtin_clz(P);
    const T *wtile = W + ((int64_t)ti * g.r + row_lo) * ldw + col0;
    constexpr int U = 4;
    // Usual tile widths (whole 32-column words per row, rows 16-byte aligned): a lane keeps its word
    // column and walks down the rows.  Per row it requests the word's pieces of W (no test in front of a load: every
    // row it visits is inside the band), rebuilds the mask word ONCE for all of them, and its offsets, its word of
    // the I_z rows and its addresses' increment are constants: no index arithmetic in the loop.
    constexpr int PW = 32 / VEC; // 16-byte pieces per mask word
    const int words = ct >> 5;
    const bool walk = (ct % 32 == 0) && words > 0 && words <= kEvalThreads && w_vec_ok && (col0 % VEC == 0);
    if (walk) {
        // (one division per lane, outside the loop; when the words do not divide the workgroup, e.g. the 18 words of a
        // 576-column tile, the lanes past the last whole row sit out)
        const int wc = tid % words;
        const int rstep = kEvalThreads / words;
        const int r0 = (tid / words < rstep) ? tid / words : nrows;
        const uint32_t *izc = iz + wc;
        const T *wp = wtile + (int64_t)r0 * ldw + 32 * wc;
        const int64_t wstride = (int64_t)rstep * ldw;
        for (int i = r0; i < nrows; i += rstep) {
            uint4 v[PW];
#pragma unroll
            for (int q = 0; q < PW; ++q) v[q] = *reinterpret_cast<const uint4 *>(wp + q * VEC);
            const uint32_t *ipr = ip + i * g.ipw;
            uint32_t word = 0u;
            for (int q = 0; q < g.ipw; ++q) {
                uint32_t sel = ipr[q];
                while (sel) {
                    const int l = __builtin_ctz(sel) + 32 * q;
                    sel &= sel - 1u;
                    word |= izc[l * g.izw];
                }
            }
            kept += (unsigned long long)__builtin_popcount(word);
            const uint32_t lost_word = ~word;
#pragma unroll
            for (int q = 0; q < PW; ++q) {
                const uint32_t lost = (lost_word >> (q * VEC)) & ((1u << VEC) - 1u);
                if (sizeof(T) == 2) {
                    // 16-bit types: the weights I_a keeps are cleared four packed multiplies at a time (an exact
                    // select on the bit pattern); what is left only needs the magnitude test
                    const uint4 z = apply_mask8(v[q], lost);
                    const uint32_t zz[4] = {z.x, z.y, z.z, z.w};
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const float a = piece_abs<T>(zz, e);
                        cost_add<SQ>(cost4[e & 3], (a >= w_threshold) ? a : 0.f);
                    }
                } else {
                    const uint32_t ww[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const float a = piece_abs<T>(ww, e);
                        const float add = (((lost >> e) & 1u) && a >= w_threshold) ? a : 0.f;
                        cost_add<SQ>(cost4[e & 3], add);
                    }
                }
            }
            wp += wstride;
        }
    }
    for (int base = tid; !walk && base < items; base += U * kEvalThreads) {
        uint32_t w4[U][4];
        uint32_t bits_u[U], valid_u[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int id = base + u * kEvalThreads;
            bits_u[u] = 0u;
            valid_u[u] = 0u;
#pragma unroll
            for (int e = 0; e < 4; ++e) w4[u][e] = 0u;
            if (id < items) {
                const int i = p_pow2 ? (id >> p_shift) : id / P; // no emulated division for the usual tile widths
                const int j = (id - i * P) * VEC;
                const T *wrow = wtile + (int64_t)i * ldw;
                const int nvalid = (ct - j < VEC) ? ct - j : VEC;
                const int mis = (int)((col0 + j) % VEC);
                const bool vec = w_vec_ok && (nvalid == VEC) && mis == 0;
                if (vec) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(wrow + j);
                    w4[u][0] = v.x; w4[u][1] = v.y; w4[u][2] = v.z; w4[u][3] = v.w;
                } else if (w_vec_ok && (nvalid == VEC) && 2 * mis == VEC) {
                    // tiles that start half a piece off (300-column tiles: every other tile column): two 8-byte loads
                    const uint2 v0 = *reinterpret_cast<const uint2 *>(wrow + j);
                    const uint2 v1 = *reinterpret_cast<const uint2 *>(wrow + j + VEC / 2);
                    w4[u][0] = v0.x; w4[u][1] = v0.y; w4[u][2] = v1.x; w4[u][3] = v1.y;
                } else if (sizeof(T) == 4) {
                    const uint32_t *wr = reinterpret_cast<const uint32_t *>(wrow);
#pragma unroll
                    for (int e = 0; e < 4; ++e) w4[u][e] = (e < nvalid) ? wr[j + e] : 0u;
                } else {
                    const uint16_t *wr = reinterpret_cast<const uint16_t *>(wrow);
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (e < nvalid) w4[u][e >> 1] |= (uint32_t)wr[j + e] << (16 * (e & 1));
                }
                // mask bits of columns j .. j + VEC - 1 (inside one 32-bit word: VEC divides 32)
                const uint32_t *ipr = ip + i * g.ipw;
                uint32_t word = 0u;
                for (int q = 0; q < g.ipw; ++q) {
                    uint32_t sel = ipr[q];
                    while (sel) {
                        const int l = __builtin_ctz(sel) + 32 * q;
                        sel &= sel - 1u;
                        word |= iz[l * g.izw + (j >> 5)];
                    }
                }
                valid_u[u] = (1u << nvalid) - 1u;
                bits_u[u] = (word >> (j & 31)) & valid_u[u];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            kept += (unsigned long long)__builtin_popcount(bits_u[u]);
            const uint32_t lost = valid_u[u] & ~bits_u[u];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float a = piece_abs<T>(w4[u], e);
                // the addend is selected (0 when the weight is kept by I_a, pruned by magnitude, or NaN), the sum is not
                const float add = (((lost >> e) & 1u) && a >= w_threshold) ? a : 0.f;
                cost_add<SQ>(cost4[e & 3], add);
            }
        }
    }
    double cost = (cost4[0] + cost4[1]) + (cost4[2] + cost4[3]);
    // lanes in a fixed order, then wavefronts in a fixed order
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
        cost += __shfl_xor(cost, s, 64);
        kept += __shfl_xor(kept, s, 64);
    }
    if (lane == 0) {
        wave_cost[wave] = cost;
        wave_kept[wave] = kept;
    }
    __syncthreads();
    if (tid == 0) {
        double c = 0.0;
        unsigned long long kk = 0ull;
        for (int w = 0; w < kEvalWaves; ++w) {
            c += wave_cost[w];
            kk += wave_kept[w];
        }
        c *= cost_scale;
        Cost[blockIdx.x] = c;
        Kept[blockIdx.x] = kk;
        if (step.st && bands == 1) search_step_tile(g, step, t, kk, c);
    }
}

// adds the bands' partial results of every tile in band order
__global__ __launch_bounds__(256) void threshold_eval_reduce_kernel(const unsigned long long *__restrict__ pk,
                                                                    const double *__restrict__ pc, int64_t tiles,
                                                                    int bands, unsigned long long *__restrict__ Kept,
                                                                    double *__restrict__ Cost, Geom g, SearchStepArgs step)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= tiles) return;
    unsigned long long kk = 0ull;
    double c = 0.0;
    for (int b = 0; b < bands; ++b) {
        kk += pk[t * bands + b];
        c += pc[t * bands + b];
    }
    Kept[t] = kk;
    Cost[t] = c;
    if (step.st) search_step_tile(g, step, t, kk, c);
}

size_t threshold_eval_lds_bytes(const Geom &g)
{
    return ((size_t)g.k * g.izw + (size_t)g.r * g.ipw) * 4;
}

// Bands of rows per tile: enough workgroups to fill the chip when there are few tiles, at
// least 32 rows per band.  Depends on the geometry only, so that the workspace query and the
// launch agree.
EvalPlan plan_threshold_eval(const Geom &g)
{
    EvalPlan p;
    const int64_t tiles = (int64_t)g.tile_rows * g.tile_cols;
    int64_t bands = (512 + tiles - 1) / tiles;
    const int64_t max_bands = g.r / 32 > 1 ? g.r / 32 : 1;
    if (bands > max_bands) bands = max_bands;
    if (bands < 1) bands = 1;
    p.rows_per_band = (int)((g.r + bands - 1) / bands);
    p.bands = (int)((g.r + p.rows_per_band - 1) / p.rows_per_band);
    p.workspace_bytes = (p.bands > 1) ? (uint64_t)tiles * p.bands * 16u : 0u;
    return p;
}

template <typename T>
static int launch_eval_t(const Geom &g, const void *dW, int64_t ldw, float w_threshold, CostManip manip, const float *dMp,
                         const float *dMz, const float *dTp, const float *dTz, void *dIp, void *dIz, uint64_t *dKept,
                         double *dCost, void *dWorkspace, hipStream_t stream, const SearchStepArgs &step)
{
    const int64_t tiles = (int64_t)g.tile_rows * g.tile_cols;
    EvalPlan plan = plan_threshold_eval(g);
    if (!dWorkspace) { // no room for partial results: one workgroup per tile
        plan.bands = 1;
        plan.rows_per_band = g.r;
    }
    if (tiles * plan.bands > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    unsigned long long *pk = (unsigned long long *)dKept;
    double *pc = dCost;
    if (plan.bands > 1) {
        pk = (unsigned long long *)dWorkspace;
        pc = (double *)((char *)dWorkspace + (size_t)tiles * plan.bands * 8);
    }
    const size_t smem = (threshold_eval_lds_bytes(g) + 15) / 16 * 16;
    const int w_vec_ok = (((uintptr_t)dW & 15) == 0) && (ldw % Mag<T>::VEC == 0);
    auto kern = manip.squared ? threshold_eval_kernel<T, true> : threshold_eval_kernel<T, false>;
    LRBI_SET_MAX_LDS(kern, smem);
    LRBI_LAUNCH(kern, dim3((unsigned)(tiles * plan.bands)), dim3(kEvalThreads), smem, stream, g, (const T *)dW,
                       ldw, w_threshold, manip.scale, dMp, dMz, dTp, dTz, (uint32_t *)dIp, (uint32_t *)dIz, pk, pc, w_vec_ok,
                       plan.bands, plan.rows_per_band, step);
    if (plan.bands > 1) {
        LRBI_LAUNCH(threshold_eval_reduce_kernel, dim3((unsigned)((tiles + 255) / 256)), dim3(256), 0, stream, pk,
                           pc, tiles, plan.bands, (unsigned long long *)dKept, dCost, g, step);
    }
    return LRBI_OK;
}

static int launch_eval_step(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, float w_threshold, CostManip manip,
                            const float *dMp,
                            const float *dMz, const float *dTp, const float *dTz, void *dIp, void *dIz, uint64_t *dKept,
                            double *dCost, void *dWorkspace, hipStream_t stream, const SearchStepArgs &step)
{
    switch (dt) {
    case LRBI_F32:
        return launch_eval_t<float>(g, dW, ldw, w_threshold, manip, dMp, dMz, dTp, dTz, dIp, dIz, dKept, dCost, dWorkspace, stream,
                                    step);
    case LRBI_F16:
        return launch_eval_t<__half>(g, dW, ldw, w_threshold, manip, dMp, dMz, dTp, dTz, dIp, dIz, dKept, dCost, dWorkspace, stream,
                                     step);
    case LRBI_BF16:
        return launch_eval_t<__hip_bfloat16>(g, dW, ldw, w_threshold, manip, dMp, dMz, dTp, dTz, dIp, dIz, dKept, dCost, dWorkspace,
                                             stream, step);
    default: return LRBI_ERR_DTYPE;
    }
}

int launch_threshold_eval(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, float w_threshold, CostManip manip,
                          const float *dMp, const float *dMz, const float *dTp, const float *dTz, void *dIp, void *dIz,
                          uint64_t *dKept, double *dCost, void *dWorkspace, hipStream_t stream)
{
    SearchStepArgs none{};
    none.st = nullptr;
    return launch_eval_step(g, dt, dW, ldw, w_threshold, manip, dMp, dMz, dTp, dTz, dIp, dIz, dKept, dCost, dWorkspace, stream,
                            none);
}

// ---------------------------------------------------------------------------
// Threshold search of Algorithm 1 (Sec. 2.1), all tiles in lockstep: for every S_p of the
// caller's list, a bisection on S_z whose probes are evaluated by the kernel above (one launch
// per probe for all tiles); the per-tile search state lives in the caller's workspace and is
// advanced inside those launches (search_step_tile), so the host never waits for the device.
// ---------------------------------------------------------------------------

// Sorts the used entries of one tile's factor (ascending, bitonic network over `padded` = 2^j slots, the
// tail filled with +inf).  which = 0: M_p, the first rt rows of k entries; which = 1: M_z, the first ct
// entries of each of the k rows (rt x ct = the tile's part inside the matrix).  One workgroup per tile.  Up
// to 16384 slots the network runs in on-chip memory and the sorted values are written to out + tile *
// stride; beyond that it runs in place in out + tile * stride (stride >= padded), slower, the workgroup's
// own barriers ordering its global accesses.
__global__ __launch_bounds__(512) void tile_sort_kernel(Geom g, int which, const float *__restrict__ in, float *out,
                                                        int padded, int64_t stride, int on_chip)
{
    extern __shared__ uint4 lrbi_dyn_smem[];
    int rt, ct;
    tile_extent(g, blockIdx.x, rt, ct);
    const int cols = which ? ct : g.k;           // used entries per stored row
    const int pitch = which ? g.c : g.k;         // entries per stored row
    const int n = which ? g.k * ct : rt * g.k;
    float *dst = out + (int64_t)blockIdx.x * stride;
    float *v = on_chip ? reinterpret_cast<float *>(lrbi_dyn_smem) : dst;
    const float *src = in + (int64_t)blockIdx.x * (which ? (int64_t)g.k * g.c : (int64_t)g.r * g.k);
    for (int i = threadIdx.x; i < padded; i += 512) {
        float x = __builtin_inff();
        if (i < n) {
            const int row = i / cols;
            x = src[(int64_t)row * pitch + (i - row * cols)];
        }
        v[i] = x;
    }
    __syncthreads();
    for (int size = 2; size <= padded; size <<= 1) {
        for (int stride2 = size >> 1; stride2 > 0; stride2 >>= 1) {
            for (int i = threadIdx.x; i < padded / 2; i += 512) {
                const int lo = 2 * i - (i & (stride2 - 1)); // lower index of the pair at this distance
                const int hi = lo + stride2;
                const bool up = (lo & size) == 0;
                const float a = v[lo], b = v[hi];
                if ((a > b) == up) {
                    v[lo] = b;
                    v[hi] = a;
                }
            }
            __syncthreads();
        }
    }
    if (on_chip)
        for (int i = threadIdx.x; i < n; i += 512) dst[i] = v[i];
}

__global__ __launch_bounds__(256) void search_begin_kernel(Geom g, SearchState *__restrict__ st,
                                                           const float *__restrict__ sortedMp,
                                                           const float *__restrict__ sortedMz, int64_t stride_p,
                                                           int64_t stride_z, int64_t tiles, double sp, double sz0,
                                                           int first, float *__restrict__ Tp, float *__restrict__ Tz)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= tiles) return;
    int rt, ct;
    tile_extent(g, t, rt, ct);
    SearchState s = st[t];
    if (first) {
        s.best_diff = -1;
        s.best_eligible = 0;
    }
    s.tp = threshold_at(sortedMp + t * stride_p, rt * g.k, sp);
    s.lo = 0.0;
    s.hi = 1.0;
    s.sz = sz0;
    s.rep_diff = -1;
    st[t] = s;
    Tp[t] = s.tp;
    Tz[t] = threshold_at(sortedMz + t * stride_z, g.k * ct, sz0);
}

constexpr int kSortOnChip = 16384; // floats: 64 KiB of on-chip memory

static int64_t pow2_at_least(int64_t n)
{
    int64_t p = 1;
    while (p < n) p <<= 1;
    return p;
}

SearchPlan plan_search(const Geom &g)
{
    SearchPlan p;
    const uint64_t tiles = (uint64_t)g.tile_rows * g.tile_cols;
    auto up = [](uint64_t v) { return (v + 255) / 256 * 256; };
    p.np = g.r * g.k;
    p.nz = g.k * g.c;
    // a factor of more than kSortOnChip entries is sorted in place in the workspace, in 2^j slots
    p.stride_p = p.np <= kSortOnChip ? p.np : pow2_at_least(p.np);
    p.stride_z = p.nz <= kSortOnChip ? p.nz : pow2_at_least(p.nz);
    p.off_sorted_mp = 0;
    p.off_sorted_mz = up(p.off_sorted_mp + tiles * (uint64_t)p.stride_p * 4);
    p.off_state = up(p.off_sorted_mz + tiles * (uint64_t)p.stride_z * 4);
    p.off_tp = up(p.off_state + tiles * sizeof(SearchState));
    p.off_tz = up(p.off_tp + tiles * 4);
    p.off_kept = up(p.off_tz + tiles * 4);
    p.off_cost = up(p.off_kept + tiles * 8);
    p.off_eval = up(p.off_cost + tiles * 8);
    p.bytes = p.off_eval + plan_threshold_eval(g).workspace_bytes;
    return p;
}

int launch_search(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, float w_threshold, CostManip manip,
                  const float *dMp,
                  const float *dMz, double target_sparsity, int n_sp, const double *sp_values, int steps,
                  int64_t tolerance, float *dTpBest, float *dTzBest, uint64_t *dKeptBest, double *dCostBest, void *dIp,
                  void *dIz, void *dWorkspace, hipStream_t stream)
{
    const SearchPlan p = plan_search(g);
    const int64_t tiles = (int64_t)g.tile_rows * g.tile_cols;
    char *ws = (char *)dWorkspace;
    float *sortedMp = (float *)(ws + p.off_sorted_mp);
    float *sortedMz = (float *)(ws + p.off_sorted_mz);
    SearchState *state = (SearchState *)(ws + p.off_state);
    float *Tp = (float *)(ws + p.off_tp);
    float *Tz = (float *)(ws + p.off_tz);
    uint64_t *kept = (uint64_t *)(ws + p.off_kept);
    double *cost = (double *)(ws + p.off_cost);
    void *eval_ws = plan_threshold_eval(g).workspace_bytes ? (void *)(ws + p.off_eval) : nullptr;

    // 1. sorted factors of every tile (the quantile look-up of "convert with (S_p, S_z)")
    for (int which = 0; which < 2; ++which) {
        const int n = which ? p.nz : p.np;
        const int padded = (int)pow2_at_least(n);
        const int on_chip = n <= kSortOnChip;
        const size_t smem = on_chip ? (size_t)padded * 4 : 0;
        LRBI_SET_MAX_LDS(tile_sort_kernel, kSortOnChip * 4);
        LRBI_LAUNCH(tile_sort_kernel, dim3((unsigned)tiles), dim3(512), smem, stream, g, which, which ? dMz : dMp,
                           which ? sortedMz : sortedMp, padded, which ? p.stride_z : p.stride_p, on_chip);
    }
    // 2. sweep over S_p, bisection on S_z
    const unsigned sblocks = (unsigned)((tiles + 255) / 256);
    for (int a = 0; a < n_sp; ++a) {
        const double sp = sp_values[a];
        double sz0 = 0.0;
        if (sp < 1.0) {
            sz0 = (pow(target_sparsity, 1.0 / (double)g.k) - sp) / (1.0 - sp); // Eq. 7 solved for S_z
            if (sz0 < 0.0) sz0 = 0.0;
            if (sz0 > 1.0) sz0 = 1.0;
        }
        LRBI_LAUNCH(search_begin_kernel, dim3(sblocks), dim3(256), 0, stream, g, state, sortedMp, sortedMz,
                           p.stride_p, p.stride_z, tiles, sp, sz0, a == 0 ? 1 : 0, Tp, Tz);
        for (int step = 0; step < steps; ++step) {
            // one launch per probe (two with row bands): the tile's search state is advanced where its result is formed
            SearchStepArgs sa;
            sa.st = state;
            sa.sortedMz = sortedMz;
            sa.stride_z = p.stride_z;
            sa.keep_fraction = 1.0 - target_sparsity;
            sa.tolerance = (long long)tolerance;
            sa.last_step = step == steps - 1 ? 1 : 0;
            sa.Tz = Tz;
            sa.TpBest = dTpBest;
            sa.TzBest = dTzBest;
            sa.KeptBest = (unsigned long long *)dKeptBest;
            sa.CostBest = dCostBest;
            const int rc = launch_eval_step(g, dt, dW, ldw, w_threshold, manip, dMp, dMz, Tp, Tz, nullptr, nullptr, kept, cost,
                                            eval_ws, stream, sa);
            if (rc != LRBI_OK) return rc;
        }
    }
    // 3. the winning thresholds once more, now writing the packed binary factors
    if (dIp)
        return launch_threshold_eval(g, dt, dW, ldw, w_threshold, manip, dMp, dMz, dTpBest, dTzBest, dIp, dIz, dKeptBest,
                                     dCostBest, eval_ws, stream);
    return LRBI_OK;
}


} // namespace lrbi
