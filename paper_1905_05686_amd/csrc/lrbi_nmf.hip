// Non-negative factorisation of the magnitude matrix, tile by tile (Algorithm 1's first step, Sec. 2.1):
// M = |W| (optionally manipulated, Sec. 3.2) ~ M_p M_z with M_p (r x k), M_z (k x c) >= 0, minimising the
// Frobenius distance.  The paper uses an off-the-shelf library and names no algorithm; this is Lee and Seung's
// multiplicative update for that objective, from the caller's starting point, M_z first and then M_p:
//     M_z <- M_z * (M_p^T M) / (M_p^T M_p M_z + eps)
//     M_p <- M_p * (M M_z^T) / (M_p M_z M_z^T + eps)
// One kernel per half update, all tiles per launch.  In the M_z update a lane owns one column j of a tile: it
// streams the column of W (coalesced across the lanes), while the rows of M_p, which every lane needs, are staged
// in LDS chunk by chunk and read as broadcasts; the k x k matrix M_p^T M_p is accumulated in LDS from the same
// chunks; the lane then forms its k numerators and denominators and writes its column of the new M_z.  The M_p
// update is the mirror image (a lane owns a row i, M_z is staged transposed, M_z M_z^T in LDS).  New factors go to a
// second buffer (the other half update still needs the old values), the two buffers swap every iteration.
// fp32 throughout, every sum in a fixed order.  Limits: k <= 64 (the k x k matrix and the chunks live in LDS).
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "lrbi_internal.hpp"

namespace lrbi {

static constexpr int kNmfThreads = 256;
static constexpr int kNmfStageFloats = 8192; // 32 KiB of staged factor rows
static constexpr int kNmfMaxK = 64;
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

// M_z update.  Workgroup = (tile, block of 256 columns); lane = column.
template <typename T, int KC>
__global__ __launch_bounds__(kNmfThreads) void nmf_update_z_kernel(Geom g, const T *__restrict__ W, int64_t ldw, int method,
                                                                  float w_threshold, float amplify,
                                                                  const float *__restrict__ Mp,
                                                                  const float *__restrict__ MzCur,
                                                                  float *__restrict__ MzNew, float eps, int cblocks)
{
    __align__(16) static __shared__ float stage[kNmfStageFloats];       // [rows of the chunk][k]
    __align__(16) static __shared__ float gram[kNmfMaxK * kNmfMaxK];    // M_p^T M_p
    const int64_t t = blockIdx.x / cblocks;
    const int cb = (int)(blockIdx.x - t * cblocks);
    int ti, tj, rt, ct;
    nmf_tile_extent(g, t, ti, tj, rt, ct);
    const int tid = threadIdx.x;
    const int j = cb * kNmfThreads + tid;
    const bool live = j < ct;
    const int k = g.k;
    const bool k4 = (k % 4) == 0;
    const int rows_per_chunk = kNmfStageFloats / k;
    const float *mp = Mp + t * (int64_t)g.r * k;
    const float *mzc = MzCur + t * (int64_t)k * g.c;
    float *mzn = MzNew + t * (int64_t)k * g.c;
    const T *wcol = W + (int64_t)ti * g.r * ldw + (int64_t)tj * g.c + (live ? j : 0);

    for (int e = tid; e < k * k; e += kNmfThreads) gram[e] = 0.f;

    for (int l0 = 0; l0 < k; l0 += KC) {
        const bool full = l0 + KC <= k;             // every rank of this pass exists
        const int kt = full ? KC : k - l0;          // ranks of this pass
        float acc[KC];
#pragma unroll
        for (int l = 0; l < KC; ++l) acc[l] = 0.f;
        for (int i0 = 0; i0 < rt; i0 += rows_per_chunk) {
            const int rows = (rt - i0 < rows_per_chunk) ? rt - i0 : rows_per_chunk;
            __syncthreads(); // the previous chunk has been consumed
            for (int e = tid; e < rows * k; e += kNmfThreads) stage[e] = mp[(int64_t)i0 * k + e];
            __syncthreads();
            if (l0 == 0) { // M_p^T M_p, every lane its own entries, rows in ascending order
                if (k4) { // four neighbouring entries per lane: one broadcast read and one 16-byte read per row
                    for (int e4 = tid; e4 < k * k / 4; e4 += kNmfThreads) {
                        const int a = e4 / (k / 4), b = (e4 - a * (k / 4)) * 4;
                        float4 s = *reinterpret_cast<const float4 *>(gram + a * k + b);
                        for (int i = 0; i < rows; ++i) {
                            const float pa = stage[i * k + a];
                            const float4 pb = *reinterpret_cast<const float4 *>(stage + i * k + b);
                            s.x = fmaf(pa, pb.x, s.x);
                            s.y = fmaf(pa, pb.y, s.y);
                            s.z = fmaf(pa, pb.z, s.z);
                            s.w = fmaf(pa, pb.w, s.w);
                        }
                        *reinterpret_cast<float4 *>(gram + a * k + b) = s;
                    }
                } else {
                    for (int e = tid; e < k * k; e += kNmfThreads) {
                        const int a = e / k, b = e - a * k;
                        float s = gram[e];
                        for (int i = 0; i < rows; ++i) s = fmaf(stage[i * k + a], stage[i * k + b], s);
                        gram[e] = s;
                    }
                }
            }
            if (live) {
                // sixteen rows at a time: their W loads are requested together; the rows of M_p come out of the staged
                // chunk as broadcast reads (reading them from global memory at lane-uniform addresses, i.e. as scalar
                // loads, was measured slower: 165 us against 100 us per launch on the 256 x 256, rank 16 layer)
                for (int i = 0; i < rows; i += ZB) {
                    T raw[ZB];
                    float mv[ZB];
#pragma unroll
                    for (int u = 0; u < ZB; ++u) {
                        const int iu = (i + u < rows) ? i + u : rows - 1; // clamped: always a valid row
                        raw[u] = wcol[(int64_t)(i0 + iu) * ldw];
                    }
#pragma unroll
                    for (int u = 0; u < ZB; ++u) {
                        const float m = nmf_mag<T>(raw[u], method, w_threshold, amplify);
                        mv[u] = (i + u < rows) ? m : 0.f;
                    }
#pragma unroll
                    for (int u = 0; u < ZB; ++u) {
                        const int iu = (i + u < rows) ? i + u : rows - 1;
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
        __syncthreads(); // gram complete
        if (live) {
            float den[KC];
#pragma unroll
            for (int l = 0; l < KC; ++l) den[l] = 0.f;
            for (int b = 0; b < k; ++b) {
                const float z = mzc[(int64_t)b * g.c + j];
#pragma unroll
                for (int l = 0; l < KC; ++l)
                    if (l0 + l < k) den[l] = fmaf(gram[(l0 + l) * k + b], z, den[l]);
            }
#pragma unroll
            for (int l = 0; l < KC; ++l)
                if (l0 + l < k) {
                    const int64_t at = (int64_t)(l0 + l) * g.c + j;
                    mzn[at] = mzc[at] * acc[l] / (den[l] + eps);
                }
        }
    }
}

// M_p update.  Workgroup = (tile, block of 256 rows); lane = row.
template <typename T, int KC>
__global__ __launch_bounds__(kNmfThreads) void nmf_update_p_kernel(Geom g, const T *__restrict__ W, int64_t ldw, int method,
                                                                  float w_threshold, float amplify,
                                                                  const float *__restrict__ MpCur,
                                                                  const float *__restrict__ Mz,
                                                                  float *__restrict__ MpNew, float eps, int rblocks,
                                                                  int w_vec_ok)
{
    __align__(16) static __shared__ float stage[kNmfStageFloats];       // [columns of the chunk][k]: M_z transposed
    __align__(16) static __shared__ float gram[kNmfMaxK * kNmfMaxK];    // M_z M_z^T
    const int64_t t = blockIdx.x / rblocks;
    const int rb = (int)(blockIdx.x - t * rblocks);
    int ti, tj, rt, ct;
    nmf_tile_extent(g, t, ti, tj, rt, ct);
    const int tid = threadIdx.x;
    const int i = rb * kNmfThreads + tid;
    const bool live = i < rt;
    const int k = g.k;
    const bool k4 = (k % 4) == 0;
    const int cols_per_chunk = (kNmfStageFloats / k) & ~7; // a multiple of 8 keeps later chunks aligned
    const float *mz = Mz + t * (int64_t)k * g.c;
    const float *mpc = MpCur + (t * (int64_t)g.r + (live ? i : 0)) * k;
    float *mpn = MpNew + (t * (int64_t)g.r + (live ? i : 0)) * k;
    const T *wrow = W + ((int64_t)ti * g.r + (live ? i : 0)) * ldw + (int64_t)tj * g.c;

    for (int e = tid; e < k * k; e += kNmfThreads) gram[e] = 0.f;

    for (int l0 = 0; l0 < k; l0 += KC) {
        const bool full = l0 + KC <= k;             // every rank of this pass exists
        const int kt = full ? KC : k - l0;          // ranks of this pass
        float acc[KC];
#pragma unroll
        for (int l = 0; l < KC; ++l) acc[l] = 0.f;
        for (int j0 = 0; j0 < ct; j0 += cols_per_chunk) {
            const int cols = (ct - j0 < cols_per_chunk) ? ct - j0 : cols_per_chunk;
            __syncthreads();
            // transpose while staging: consecutive lanes read consecutive columns of one row of M_z
            for (int e = tid; e < cols * k; e += kNmfThreads) {
                const int l = e / cols, jj = e - l * cols;
                stage[jj * k + l] = mz[(int64_t)l * g.c + j0 + jj];
            }
            __syncthreads();
            if (l0 == 0) {
                if (k4) {
                    for (int e4 = tid; e4 < k * k / 4; e4 += kNmfThreads) {
                        const int a = e4 / (k / 4), b = (e4 - a * (k / 4)) * 4;
                        float4 s = *reinterpret_cast<const float4 *>(gram + a * k + b);
                        for (int jj = 0; jj < cols; ++jj) {
                            const float za = stage[jj * k + a];
                            const float4 zb = *reinterpret_cast<const float4 *>(stage + jj * k + b);
                            s.x = fmaf(za, zb.x, s.x);
                            s.y = fmaf(za, zb.y, s.y);
                            s.z = fmaf(za, zb.z, s.z);
                            s.w = fmaf(za, zb.w, s.w);
                        }
                        *reinterpret_cast<float4 *>(gram + a * k + b) = s;
                    }
                } else {
                    for (int e = tid; e < k * k; e += kNmfThreads) {
                        const int a = e / k, b = e - a * k;
                        float s = gram[e];
                        for (int jj = 0; jj < cols; ++jj) s = fmaf(stage[jj * k + a], stage[jj * k + b], s);
                        gram[e] = s;
                    }
                }
            }
            if (live) {
                // eight columns at a time: one 16-byte load of the lane's row of W where the alignment allows it
                constexpr int VEC = 16 / (int)sizeof(T);
                const bool vec = w_vec_ok && (((int64_t)tj * g.c + j0) % VEC == 0);
                for (int jj = 0; jj < cols; jj += 8) {
                    float mv[8];
                    if (vec && jj + 8 <= cols) {
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
                            const int ju = (jj + u < cols) ? jj + u : cols - 1;
                            raw[u] = wrow[j0 + ju];
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const float m = nmf_mag<T>(raw[u], method, w_threshold, amplify);
                            mv[u] = (jj + u < cols) ? m : 0.f;
                        }
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int ju = (jj + u < cols) ? jj + u : cols - 1;
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
        if (live) {
            float den[KC];
#pragma unroll
            for (int l = 0; l < KC; ++l) den[l] = 0.f;
            for (int b = 0; b < k; ++b) {
                const float p = mpc[b];
#pragma unroll
                for (int l = 0; l < KC; ++l)
                    if (l0 + l < k) den[l] = fmaf(p, gram[b * k + l0 + l], den[l]);
            }
#pragma unroll
            for (int l = 0; l < KC; ++l)
                if (l0 + l < k) mpn[l0 + l] = mpc[l0 + l] * acc[l] / (den[l] + eps);
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

template <typename T, int KC>
static int nmf_iterate(const Geom &g, const void *dW, int64_t ldw, int method, float w_threshold, float amplify, float *dMp,
                       float *dMz, int iters, float eps, float *wsMp, float *wsMz, hipStream_t stream)
{
    const int64_t tiles = (int64_t)g.tile_rows * g.tile_cols;
    const int cblocks = (g.c + kNmfThreads - 1) / kNmfThreads, rblocks = (g.r + kNmfThreads - 1) / kNmfThreads;
    if (tiles * cblocks > 0x7FFFFFFF || tiles * rblocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    float *mp_cur = dMp, *mp_new = wsMp, *mz_cur = dMz, *mz_new = wsMz;
    const int w_vec_ok = (((uintptr_t)dW & 15) == 0) && ((ldw * (int64_t)sizeof(T)) % 16 == 0);
    for (int it = 0; it < iters; ++it) {
        LRBI_LAUNCH((nmf_update_z_kernel<T, KC>), dim3((unsigned)(tiles * cblocks)), dim3(kNmfThreads), 0, stream, g,
                           (const T *)dW, ldw, method, w_threshold, amplify, mp_cur, mz_cur, mz_new, eps, cblocks);
        LRBI_LAUNCH((nmf_update_p_kernel<T, KC>), dim3((unsigned)(tiles * rblocks)), dim3(kNmfThreads), 0, stream, g,
                           (const T *)dW, ldw, method, w_threshold, amplify, mp_cur, mz_new, mp_new, eps, rblocks, w_vec_ok);
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
                     float *dMz, int iters, float eps, float *wsMp, float *wsMz, hipStream_t stream)
{
    // ranks held in registers per pass: the smallest of 8 / 16 / 32 that covers k (two passes for 32 < k <= 64)
    if (g.k <= 8) return nmf_iterate<T, 8>(g, dW, ldw, method, w_threshold, amplify, dMp, dMz, iters, eps, wsMp, wsMz, stream);
    if (g.k <= 16) return nmf_iterate<T, 16>(g, dW, ldw, method, w_threshold, amplify, dMp, dMz, iters, eps, wsMp, wsMz, stream);
    return nmf_iterate<T, 32>(g, dW, ldw, method, w_threshold, amplify, dMp, dMz, iters, eps, wsMp, wsMz, stream);
}

uint64_t nmf_workspace_bytes(const Geom &g)
{
    const uint64_t tiles = (uint64_t)g.tile_rows * g.tile_cols;
    const uint64_t mp = (tiles * g.r * g.k * 4 + 255) / 256 * 256;
    const uint64_t mz = (tiles * g.k * g.c * 4 + 255) / 256 * 256;
    return mp + mz;
}

int launch_nmf(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, int method, float w_threshold, float amplify,
               float *dMp, float *dMz, int iters, float eps, void *dWorkspace, hipStream_t stream)
{
    if (g.k > kNmfMaxK) return LRBI_ERR_RANK;
    const uint64_t tiles = (uint64_t)g.tile_rows * g.tile_cols;
    float *wsMp = (float *)dWorkspace;
    float *wsMz = (float *)((char *)dWorkspace + (tiles * g.r * g.k * 4 + 255) / 256 * 256);
    // the second buffers start as copies, so that what a cut-off tile does not use is the same in both
    int rc = nmf_copy(dMp, wsMp, (int64_t)(tiles * g.r * g.k), stream);
    if (rc != LRBI_OK) return rc;
    rc = nmf_copy(dMz, wsMz, (int64_t)(tiles * g.k * g.c), stream);
    if (rc != LRBI_OK) return rc;
    switch (dt) {
    case LRBI_F32: return nmf_dtype<float>(g, dW, ldw, method, w_threshold, amplify, dMp, dMz, iters, eps, wsMp, wsMz, stream);
    case LRBI_F16: return nmf_dtype<__half>(g, dW, ldw, method, w_threshold, amplify, dMp, dMz, iters, eps, wsMp, wsMz, stream);
    case LRBI_BF16:
        return nmf_dtype<__hip_bfloat16>(g, dW, ldw, method, w_threshold, amplify, dMp, dMz, iters, eps, wsMp, wsMz, stream);
    default: return LRBI_ERR_DTYPE;
    }
}

} // namespace lrbi
