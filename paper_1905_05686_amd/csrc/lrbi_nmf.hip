// Non-negative factorisation of the magnitude matrix, tile by tile (Algorithm 1's first step, Sec. 2.1):
// M = |W| (optionally manipulated, Sec. 3.2) ~ M_p M_z with M_p (r x k), M_z (k x c) >= 0, minimising the
// Frobenius distance.  The paper uses an off-the-shelf library and names no algorithm; this is Lee and Seung's
// multiplicative update for that objective, from the caller's starting point, M_z first and then M_p:
//     M_z <- M_z * (M_p^T M) / (M_p^T M_p M_z + eps)
//     M_p <- M_p * (M M_z^T) / (M_p M_z M_z^T + eps)
// Per half update two kernels, all tiles per launch: the k x k Gram matrix of the factor that stays fixed
// (M_p^T M_p or M_z M_z^T, one lane per entry), then the update itself.
// M_z update: a workgroup of four wavefronts owns 64 columns of a tile; lane = column, and each wavefront takes a
// quarter of the tile's rows.  The rows of M_p, which every lane needs, are staged in LDS chunk by chunk and read as
// broadcasts while the lane streams its column of W (coalesced across the lanes); the four partial numerators of a
// column are added through LDS in wavefront order; the denominators come from the Gram rows (staged in LDS) and
// the lane's column of the old M_z.  Splitting tiles this finely is what fills the chip: 64 tiles of 512 columns
// give 512 workgroups.  The M_p update is the mirror image (lane = row, M_z staged transposed, a wavefront per
// quarter of the columns).  New factors go to a second buffer (the other half update still needs the old values),
// the two buffers swap every iteration.  fp32 throughout, every sum in a fixed order.  The ranks are processed KC
// (8, 16 or 32) at a time, so any k up to 256 (the paper's largest) is served; each pass streams W again.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "lrbi_internal.hpp"

namespace lrbi {

static constexpr int kNmfThreads = 256;
static constexpr int kNmfStageFloats = 8192; // 32 KiB of staged factor rows
static constexpr int kNmfMaxK = 256;
// A workgroup owns kNmfThreads / PARTS columns (rows) of a tile, one per lane, and PARTS groups of lanes share them, each
// taking a part of the rows (columns): PARTS = 4 when the tiles alone would not fill the chip, else 1.
static constexpr int ZB = 16; // rows of W requested together in the M_z update

template <typename T> struct NmfElem;
template <> struct NmfElem<float> {
    __device__ static float to_f32(float v) { return v; }
};
template <> struct NmfElem<__half> {
    __device__ static float to_f32(__half v) { return __half2float(v); }
};
template <> struct NmfElem<__hip_bfloat16> {
    __device__ static float to_f32(__hip_bfloat16 v) { return __bfloat162float(v); }
};

// magnitude with the manipulation of Sec. 3.2: 1 none, 2 squared, 3 amplified where magnitude pruning keeps the weight
template <typename T> __device__ __forceinline__ float nmf_mag(T w, int method, float w_threshold, float amplify)
{
    // selects, not branches: a branch per element kept the compiler from requesting a batch of loads together
    const float a = fabsf(NmfElem<T>::to_f32(w));
    const float squared = a * a;
    const float amplified = (a >= w_threshold) ? a * amplify : a;
    return (method == 2) ? squared : ((method == 3) ? amplified : a);
}

__device__ __forceinline__ void nmf_tile_extent(const Geom &g, int64_t t, int &ti, int &tj, int &rt, int &ct)
{
    ti = (int)(t / g.tile_cols);
    tj = (int)(t - (int64_t)ti * g.tile_cols);
    rt = (int)((g.m - (int64_t)ti * g.r < g.r) ? g.m - (int64_t)ti * g.r : g.r);
    ct = (int)((g.n - (int64_t)tj * g.c < g.c) ? g.n - (int64_t)tj * g.c : g.c);
}

// Gram matrix of a tile's fixed factor: G[a][b] = sum_i Mp[i][a] Mp[i][b] (ZSIDE = false, rows of the tile in
// ascending order) or sum_j Mz[a][j] Mz[b][j] (ZSIDE = true, columns in ascending order).  The factor is staged in LDS
// chunk by chunk as [row or column][k] (M_z transposed on the way in); a lane owns four neighbouring entries of G (one
// when k is not a multiple of 4) and reads one broadcast value and one 16-byte piece per staged row.
template <bool ZSIDE>
__global__ __launch_bounds__(kNmfThreads) void nmf_gram_kernel(Geom g, const float *__restrict__ F, float *__restrict__ G,
                                                              int eblocks)
{
    __align__(16) static __shared__ float stage[kNmfStageFloats];
    const int64_t t = blockIdx.x / eblocks;
    const int eb = (int)(blockIdx.x - t * eblocks);
    const int tid = threadIdx.x;
    const int k = g.k;
    const bool k4 = (k % 4) == 0;
    int ti, tj, rt, ct;
    nmf_tile_extent(g, t, ti, tj, rt, ct);
    const int count = ZSIDE ? ct : rt;                 // rows (columns) summed over
    const int per_chunk = kNmfStageFloats / k;
    const float *f = F + (ZSIDE ? t * (int64_t)k * g.c : t * (int64_t)g.r * k);
    const int unit = eb * kNmfThreads + tid;           // four entries (k4) or one
    const int units = k4 ? k * k / 4 : k * k;
    const bool live = unit < units;
    const int a = live ? (k4 ? unit / (k / 4) : unit / k) : 0;
    const int b = live ? (k4 ? (unit - a * (k / 4)) * 4 : unit - a * k) : 0;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i0 = 0; i0 < count; i0 += per_chunk) {
        const int n = (count - i0 < per_chunk) ? count - i0 : per_chunk;
        __syncthreads();
        if (ZSIDE) { // consecutive lanes read consecutive columns of one row of M_z
            for (int e = tid; e < n * k; e += kNmfThreads) {
                const int l = e / n, jj = e - l * n;
                stage[jj * k + l] = f[(int64_t)l * g.c + i0 + jj];
            }
        } else {
            for (int e = tid; e < n * k; e += kNmfThreads) stage[e] = f[(int64_t)i0 * k + e];
        }
        __syncthreads();
        if (!live) continue;
        if (k4) {
            for (int i = 0; i < n; ++i) {
                const float pa = stage[i * k + a];
                const float4 pb = *reinterpret_cast<const float4 *>(stage + i * k + b);
                s.x = fmaf(pa, pb.x, s.x);
                s.y = fmaf(pa, pb.y, s.y);
                s.z = fmaf(pa, pb.z, s.z);
                s.w = fmaf(pa, pb.w, s.w);
            }
        } else {
            for (int i = 0; i < n; ++i) s.x = fmaf(stage[i * k + a], stage[i * k + b], s.x);
        }
    }
    if (!live) return;
    float *gt = G + t * (int64_t)k * k + (int64_t)a * k + b;
    if (k4) *reinterpret_cast<float4 *>(gt) = s;
    else *gt = s.x;
}

// M_z update.  Workgroup = (tile, block of 256 / PARTS columns); lane = column, group of lanes = part of the rows.
template <typename T, int KC, int PARTS>
__global__ __launch_bounds__(kNmfThreads) void nmf_update_z_kernel(Geom g, const T *__restrict__ W, int64_t ldw, int method,
                                                                  float w_threshold, float amplify,
                                                                  const float *__restrict__ Mp,
                                                                  const float *__restrict__ MzCur,
                                                                  float *__restrict__ MzNew, const float *__restrict__ G,
                                                                  float eps, int cblocks)
{
    extern __shared__ uint4 lrbi_dyn_smem[];
    float *stage = (float *)lrbi_dyn_smem;   // [rows of the chunk][k]; then the partial sums [part][rank][lane]
    float *gramL = stage + kNmfStageFloats;  // the pass's rows of M_p^T M_p: [KC][k]
    constexpr int kNmfParts = PARTS, kNmfOwn = kNmfThreads / PARTS;
    static_assert(kNmfParts * KC * kNmfOwn <= kNmfStageFloats && KC * kNmfMaxK <= kNmfStageFloats, "LDS reuse");
    const int64_t t = blockIdx.x / cblocks;
    const int cb = (int)(blockIdx.x - t * cblocks);
    int ti, tj, rt, ct;
    nmf_tile_extent(g, t, ti, tj, rt, ct);
    const int tid = threadIdx.x;
    const int lane = tid & (kNmfOwn - 1), part = tid / kNmfOwn;
    const int j = cb * kNmfOwn + lane;
    const bool live = j < ct;
    const int k = g.k;
    const bool k4 = (k % 4) == 0;
    const int rows_per_chunk = kNmfStageFloats / k;
    const float *mp = Mp + t * (int64_t)g.r * k;
    const float *mzc = MzCur + t * (int64_t)k * g.c;
    float *mzn = MzNew + t * (int64_t)k * g.c;
    const float *gt = G + t * (int64_t)k * k;
    const T *wcol = W + (int64_t)ti * g.r * ldw + (int64_t)tj * g.c + (live ? j : 0);

    for (int l0 = 0; l0 < k; l0 += KC) {
        const bool full = l0 + KC <= k;             // every rank of this pass exists
        const int kt = full ? KC : k - l0;          // ranks of this pass
        float acc[KC];
#pragma unroll
        for (int l = 0; l < KC; ++l) acc[l] = 0.f;
        __syncthreads(); // the previous pass has read its Gram rows and partial sums
        for (int e = tid; e < kt * k; e += kNmfThreads) gramL[e] = gt[(int64_t)l0 * k + e];
        for (int i0 = 0; i0 < rt; i0 += rows_per_chunk) {
            const int rows = (rt - i0 < rows_per_chunk) ? rt - i0 : rows_per_chunk;
            __syncthreads(); // the previous chunk has been consumed
            for (int e = tid; e < rows * k; e += kNmfThreads) stage[e] = mp[(int64_t)i0 * k + e];
            __syncthreads();
            // this wavefront's rows of the chunk
            const int per = (rows + kNmfParts - 1) / kNmfParts;
            const int ibeg = part * per, iend = (ibeg + per < rows) ? ibeg + per : rows;
            if (live) {
                // sixteen rows at a time: their W loads are requested together; the rows of M_p come out of the staged
                // chunk as broadcast reads
                for (int i = ibeg; i < iend; i += ZB) {
                    T raw[ZB];
                    float mv[ZB];
#pragma unroll
                    for (int u = 0; u < ZB; ++u) {
                        const int iu = (i + u < iend) ? i + u : iend - 1; // clamped: always a valid row
                        raw[u] = wcol[(int64_t)(i0 + iu) * ldw];
                    }
#pragma unroll
                    for (int u = 0; u < ZB; ++u) {
                        const float m = nmf_mag<T>(raw[u], method, w_threshold, amplify);
                        mv[u] = (i + u < iend) ? m : 0.f;
                    }
#pragma unroll
                    for (int u = 0; u < ZB; ++u) {
                        const int iu = (i + u < iend) ? i + u : iend - 1;
                        const float *row = stage + iu * k + l0;
                        if (full && k4) { // rows of the staged chunk are 16-byte aligned: four ranks per LDS read
#pragma unroll
                            for (int l = 0; l < KC; l += 4) {
                                const float4 v = *reinterpret_cast<const float4 *>(row + l);
                                acc[l + 0] = fmaf(v.x, mv[u], acc[l + 0]);
                                acc[l + 1] = fmaf(v.y, mv[u], acc[l + 1]);
                                acc[l + 2] = fmaf(v.z, mv[u], acc[l + 2]);
                                acc[l + 3] = fmaf(v.w, mv[u], acc[l + 3]);
                            }
                        } else { // ranks beyond k repeat the last one; their sums are never stored
#pragma unroll
                            for (int l = 0; l < KC; ++l) acc[l] = fmaf(row[l < kt ? l : kt - 1], mv[u], acc[l]);
                        }
                    }
                }
            }
        }
        __syncthreads(); // the last chunk has been consumed: the staging area takes the partial sums
#pragma unroll
        for (int l = 0; l < KC; ++l) stage[(part * KC + l) * kNmfOwn + lane] = acc[l];
        __syncthreads();
        if (live) {
            // this lane finishes the ranks part, part + 4, ... of its column: numerator in wavefront order, denominator
            // from the Gram rows and the column of the old M_z
            float den[KC / kNmfParts];
#pragma unroll
            for (int q = 0; q < KC / kNmfParts; ++q) den[q] = 0.f;
            for (int b = 0; b < k; ++b) {
                const float z = mzc[(int64_t)b * g.c + j];
#pragma unroll
                for (int q = 0; q < KC / kNmfParts; ++q) {
                    const int l = part + kNmfParts * q;
                    if (l < kt) den[q] = fmaf(gramL[l * k + b], z, den[q]);
                }
            }
#pragma unroll
            for (int q = 0; q < KC / kNmfParts; ++q) {
                const int l = part + kNmfParts * q;
                if (l < kt) {
                    float num = 0.f;
#pragma unroll
                    for (int w = 0; w < kNmfParts; ++w) num += stage[(w * KC + l) * kNmfOwn + lane];
                    const int64_t at = (int64_t)(l0 + l) * g.c + j;
                    mzn[at] = mzc[at] * num / (den[q] + eps);
                }
            }
        }
    }
}

// M_p update.  Workgroup = (tile, block of 256 / PARTS rows); lane = row, group of lanes = part of the columns.
template <typename T, int KC, int PARTS>
__global__ __launch_bounds__(kNmfThreads) void nmf_update_p_kernel(Geom g, const T *__restrict__ W, int64_t ldw, int method,
                                                                  float w_threshold, float amplify,
                                                                  const float *__restrict__ MpCur,
                                                                  const float *__restrict__ Mz,
                                                                  float *__restrict__ MpNew, const float *__restrict__ G,
                                                                  float eps, int rblocks, int w_vec_ok)
{
    extern __shared__ uint4 lrbi_dyn_smem[];
    float *stage = (float *)lrbi_dyn_smem;   // [columns of the chunk][k]: M_z transposed; then the partial sums
    float *gramL = stage + kNmfStageFloats;  // the pass's rows of M_z M_z^T (symmetric): [KC][k]
    constexpr int kNmfParts = PARTS, kNmfOwn = kNmfThreads / PARTS;
    const int64_t t = blockIdx.x / rblocks;
    const int rb = (int)(blockIdx.x - t * rblocks);
    int ti, tj, rt, ct;
    nmf_tile_extent(g, t, ti, tj, rt, ct);
    const int tid = threadIdx.x;
    const int lane = tid & (kNmfOwn - 1), part = tid / kNmfOwn;
    const int i = rb * kNmfOwn + lane;
    const bool live = i < rt;
    const int k = g.k;
    const bool k4 = (k % 4) == 0;
    const int cols_per_chunk = (kNmfStageFloats / k) & ~31; // a multiple of 32: every part is a multiple of 8 columns
    const float *mz = Mz + t * (int64_t)k * g.c;
    const float *mpc = MpCur + (t * (int64_t)g.r + (live ? i : 0)) * k;
    float *mpn = MpNew + (t * (int64_t)g.r + (live ? i : 0)) * k;
    const float *gt = G + t * (int64_t)k * k;
    const T *wrow = W + ((int64_t)ti * g.r + (live ? i : 0)) * ldw + (int64_t)tj * g.c;

    for (int l0 = 0; l0 < k; l0 += KC) {
        const bool full = l0 + KC <= k;             // every rank of this pass exists
        const int kt = full ? KC : k - l0;          // ranks of this pass
        float acc[KC];
#pragma unroll
        for (int l = 0; l < KC; ++l) acc[l] = 0.f;
        __syncthreads();
        for (int e = tid; e < kt * k; e += kNmfThreads) gramL[e] = gt[(int64_t)l0 * k + e];
        for (int j0 = 0; j0 < ct; j0 += cols_per_chunk) {
            const int cols = (ct - j0 < cols_per_chunk) ? ct - j0 : cols_per_chunk;
            __syncthreads();
            // transpose while staging: consecutive lanes read consecutive columns of one row of M_z
            for (int e = tid; e < cols * k; e += kNmfThreads) {
                const int l = e / cols, jj = e - l * cols;
                stage[jj * k + l] = mz[(int64_t)l * g.c + j0 + jj];
            }
            __syncthreads();
            // this wavefront's columns of the chunk, a multiple of 8 so that the 16-byte loads of W stay aligned
            const int per = ((cols + kNmfParts - 1) / kNmfParts + 7) & ~7;
            const int jbeg = (part * per < cols) ? part * per : cols, jend = (jbeg + per < cols) ? jbeg + per : cols;
            if (live) {
                // eight columns at a time: one 16-byte load of the lane's row of W where the alignment allows it
                constexpr int VEC = 16 / (int)sizeof(T);
                const bool vec = w_vec_ok && (((int64_t)tj * g.c + j0) % VEC == 0);
                for (int jj = jbeg; jj < jend; jj += 8) {
                    float mv[8];
                    if (vec && jj + 8 <= jend) {
                        T tmp[8];
#pragma unroll
                        for (int q = 0; q < 8 / VEC; ++q)
                            *reinterpret_cast<uint4 *>(tmp + q * VEC) = *reinterpret_cast<const uint4 *>(wrow + j0 + jj + q * VEC);
#pragma unroll
                        for (int u = 0; u < 8; ++u) mv[u] = nmf_mag<T>(tmp[u], method, w_threshold, amplify);
                    } else {
                        T raw[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const int ju = (jj + u < jend) ? jj + u : jend - 1;
                            raw[u] = wrow[j0 + ju];
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const float m = nmf_mag<T>(raw[u], method, w_threshold, amplify);
                            mv[u] = (jj + u < jend) ? m : 0.f;
                        }
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int ju = (jj + u < jend) ? jj + u : jend - 1;
                        const float *col = stage + ju * k + l0;
                        if (full && k4) { // rows of the staged chunk are 16-byte aligned: four ranks per LDS read
#pragma unroll
                            for (int l = 0; l < KC; l += 4) {
                                const float4 v = *reinterpret_cast<const float4 *>(col + l);
                                acc[l + 0] = fmaf(v.x, mv[u], acc[l + 0]);
                                acc[l + 1] = fmaf(v.y, mv[u], acc[l + 1]);
                                acc[l + 2] = fmaf(v.z, mv[u], acc[l + 2]);
                                acc[l + 3] = fmaf(v.w, mv[u], acc[l + 3]);
                            }
                        } else { // ranks beyond k repeat the last one; their sums are never stored
#pragma unroll
                            for (int l = 0; l < KC; ++l) acc[l] = fmaf(col[l < kt ? l : kt - 1], mv[u], acc[l]);
                        }
                    }
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int l = 0; l < KC; ++l) stage[(part * KC + l) * kNmfOwn + lane] = acc[l];
        __syncthreads();
        if (live) {
            float den[KC / kNmfParts];
#pragma unroll
            for (int q = 0; q < KC / kNmfParts; ++q) den[q] = 0.f;
            for (int b = 0; b < k; ++b) {
                const float pv = mpc[b];
#pragma unroll
                for (int q = 0; q < KC / kNmfParts; ++q) {
                    const int l = part + kNmfParts * q;
                    if (l < kt) den[q] = fmaf(pv, gramL[l * k + b], den[q]);
                }
            }
#pragma unroll
            for (int q = 0; q < KC / kNmfParts; ++q) {
                const int l = part + kNmfParts * q;
                if (l < kt) {
                    float num = 0.f;
#pragma unroll
                    for (int w = 0; w < kNmfParts; ++w) num += stage[(w * KC + l) * kNmfOwn + lane];
                    mpn[l0 + l] = mpc[l0 + l] * num / (den[q] + eps);
                }
            }
        }
    }
}

__global__ __launch_bounds__(256) void nmf_copy_kernel(const float *__restrict__ src, float *__restrict__ dst, int64_t count)
{
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256) dst[e] = src[e];
}

static int nmf_copy(const float *src, float *dst, int64_t count, hipStream_t stream)
{
    int64_t blocks = (count + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    LRBI_LAUNCH(nmf_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, src, dst, count);
    return LRBI_OK;
}

template <typename T, int KC, int PARTS>
static int nmf_iterate(const Geom &g, const void *dW, int64_t ldw, int method, float w_threshold, float amplify, float *dMp,
                       float *dMz, int iters, float eps, float *wsMp, float *wsMz, float *wsG, hipStream_t stream)
{
    constexpr int kNmfOwn = kNmfThreads / PARTS;
    const int64_t tiles = (int64_t)g.tile_rows * g.tile_cols;
    const int cblocks = (g.c + kNmfOwn - 1) / kNmfOwn, rblocks = (g.r + kNmfOwn - 1) / kNmfOwn;
    const int eunits = (g.k % 4 == 0) ? g.k * g.k / 4 : g.k * g.k; // a lane owns four entries of the Gram matrix, or one
    const int eblocks = (eunits + kNmfThreads - 1) / kNmfThreads;
    if (tiles * cblocks > 0x7FFFFFFF || tiles * rblocks > 0x7FFFFFFF || tiles * eblocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    const size_t lds = ((size_t)kNmfStageFloats + (size_t)KC * g.k) * 4; // staging area + the pass's Gram rows
    LRBI_SET_MAX_LDS((nmf_update_z_kernel<T, KC, PARTS>), lds);
    LRBI_SET_MAX_LDS((nmf_update_p_kernel<T, KC, PARTS>), lds);
    float *mp_cur = dMp, *mp_new = wsMp, *mz_cur = dMz, *mz_new = wsMz;
    const int w_vec_ok = (((uintptr_t)dW & 15) == 0) && ((ldw * (int64_t)sizeof(T)) % 16 == 0);
    for (int it = 0; it < iters; ++it) {
        LRBI_LAUNCH((nmf_gram_kernel<false>), dim3((unsigned)(tiles * eblocks)), dim3(kNmfThreads), 0, stream, g, mp_cur, wsG,
                    eblocks);
        LRBI_LAUNCH((nmf_update_z_kernel<T, KC, PARTS>), dim3((unsigned)(tiles * cblocks)), dim3(kNmfThreads), lds, stream, g,
                           (const T *)dW, ldw, method, w_threshold, amplify, mp_cur, mz_cur, mz_new, wsG, eps, cblocks);
        LRBI_LAUNCH((nmf_gram_kernel<true>), dim3((unsigned)(tiles * eblocks)), dim3(kNmfThreads), 0, stream, g, mz_new, wsG,
                    eblocks);
        LRBI_LAUNCH((nmf_update_p_kernel<T, KC, PARTS>), dim3((unsigned)(tiles * rblocks)), dim3(kNmfThreads), lds, stream, g,
                           (const T *)dW, ldw, method, w_threshold, amplify, mp_cur, mz_new, mp_new, wsG, eps, rblocks, w_vec_ok);
        float *tmp = mp_cur;
        mp_cur = mp_new;
        mp_new = tmp;
        tmp = mz_cur;
        mz_cur = mz_new;
        mz_new = tmp;
    }
    if (mp_cur != dMp) { // an odd number of iterations ends in the workspace
        int rc = nmf_copy(mp_cur, dMp, tiles * g.r * g.k, stream);
        if (rc != LRBI_OK) return rc;
        rc = nmf_copy(mz_cur, dMz, tiles * (int64_t)g.k * g.c, stream);
        if (rc != LRBI_OK) return rc;
    }
    return LRBI_OK;
}

template <typename T>
static int nmf_dtype(const Geom &g, const void *dW, int64_t ldw, int method, float w_threshold, float amplify, float *dMp,
                     float *dMz, int iters, float eps, float *wsMp, float *wsMz, float *wsG, hipStream_t stream)
{
    // ranks held in registers per pass: the smallest of 8 / 16 / 32 that covers k (several passes above 32); tiles are
    // split four ways more finely when whole-tile column blocks would leave compute units idle
    const int64_t coarse = (int64_t)g.tile_rows * g.tile_cols * ((((g.c < g.r) ? g.c : g.r) + kNmfThreads - 1) / kNmfThreads);
    const bool fine = coarse < 2 * (int64_t)compute_units_of(stream);
#define LRBI_NMF_ARGS g, dW, ldw, method, w_threshold, amplify, dMp, dMz, iters, eps, wsMp, wsMz, wsG, stream
    if (g.k <= 8) return fine ? nmf_iterate<T, 8, 4>(LRBI_NMF_ARGS) : nmf_iterate<T, 8, 1>(LRBI_NMF_ARGS);
    if (g.k <= 16) return fine ? nmf_iterate<T, 16, 4>(LRBI_NMF_ARGS) : nmf_iterate<T, 16, 1>(LRBI_NMF_ARGS);
    return fine ? nmf_iterate<T, 32, 4>(LRBI_NMF_ARGS) : nmf_iterate<T, 32, 1>(LRBI_NMF_ARGS);
#undef LRBI_NMF_ARGS
}

uint64_t nmf_workspace_bytes(const Geom &g)
{
    const uint64_t tiles = (uint64_t)g.tile_rows * g.tile_cols;
    const uint64_t mp = (tiles * g.r * g.k * 4 + 255) / 256 * 256;
    const uint64_t mz = (tiles * g.k * g.c * 4 + 255) / 256 * 256;
    const uint64_t gram = (tiles * g.k * g.k * 4 + 255) / 256 * 256;
    return mp + mz + gram;
}

int launch_nmf(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, int method, float w_threshold, float amplify,
               float *dMp, float *dMz, int iters, float eps, void *dWorkspace, hipStream_t stream)
{
    if (g.k > kNmfMaxK) return LRBI_ERR_RANK;
    const uint64_t tiles = (uint64_t)g.tile_rows * g.tile_cols;
    float *wsMp = (float *)dWorkspace;
    float *wsMz = (float *)((char *)dWorkspace + (tiles * g.r * g.k * 4 + 255) / 256 * 256);
    float *wsG = (float *)((char *)wsMz + (tiles * g.k * g.c * 4 + 255) / 256 * 256);
    // the second buffers start as copies, so that what a cut-off tile does not use is the same in both
    int rc = nmf_copy(dMp, wsMp, (int64_t)(tiles * g.r * g.k), stream);
    if (rc != LRBI_OK) return rc;
    rc = nmf_copy(dMz, wsMz, (int64_t)(tiles * g.k * g.c), stream);
    if (rc != LRBI_OK) return rc;
    switch (dt) {
    case LRBI_F32: return nmf_dtype<float>(g, dW, ldw, method, w_threshold, amplify, dMp, dMz, iters, eps, wsMp, wsMz, wsG, stream);
    case LRBI_F16: return nmf_dtype<__half>(g, dW, ldw, method, w_threshold, amplify, dMp, dMz, iters, eps, wsMp, wsMz, wsG, stream);
    case LRBI_BF16:
        return nmf_dtype<__hip_bfloat16>(g, dW, ldw, method, w_threshold, amplify, dMp, dMz, iters, eps, wsMp, wsMz, wsG, stream);
    default: return LRBI_ERR_DTYPE;
    }
}

} // namespace lrbi
