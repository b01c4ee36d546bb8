// Candidate evaluation of Algorithm 1 (Sec. 2.2): threshold the real-valued factors of every
// tile, form I_a = I_p (x) I_z (Eq. 3) on chip, and return per tile the number of ones of I_a
// and the cost (sum of the magnitudes that magnitude pruning keeps and I_a prunes).
//
// One workgroup per tile.
//   1. The tile's M_z (k x c floats) and M_p (r x k floats) are compared with the tile's
//      thresholds; the resulting bits go to LDS in the packed layouts (I_z rows of
//      2 * ceil(c / 64) words, I_p rows of ceil(k / 32) words) and, when asked for, to global
//      memory as the packed factors.
//   2. Wavefronts take the tile's rows in turn.  A lane owns 8 (16-bit types) or 4 (fp32)
//      consecutive columns per step: it rebuilds the 32-bit mask word over them (OR of the I_z
//      words selected by the set bits of the row's I_p words, all from LDS), counts the ones,
//      loads its 16 bytes of W and adds |w| for every column with w kept by magnitude and
//      pruned by the mask.  Per-lane sums are kept in double; lanes, then wavefronts, are added
//      in a fixed order.
// The kernel is bound by the single sweep over W (HBM); the factor reads are k (r + c) floats
// per tile against r c weights.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "lrbi_internal.hpp"

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

template <typename T>
__global__ __launch_bounds__(kEvalThreads) void threshold_eval_kernel(Geom g, const T *__restrict__ W, int64_t ldw,
                                                                      float w_threshold,
                                                                      const float *__restrict__ Mp,
                                                                      const float *__restrict__ Mz,
                                                                      const float *__restrict__ Tp,
                                                                      const float *__restrict__ Tz,
                                                                      uint32_t *__restrict__ IpOut,
                                                                      uint32_t *__restrict__ IzOut,
                                                                      unsigned long long *__restrict__ Kept,
                                                                      double *__restrict__ Cost, int w_vec_ok)
{
    constexpr int VEC = Mag<T>::VEC;
    extern __shared__ uint4 lrbi_dyn_smem[];
    uint32_t *iz = reinterpret_cast<uint32_t *>(lrbi_dyn_smem); // [k][izw]
    uint32_t *ip = iz + g.k * g.izw;                            // [r][ipw]
    static __shared__ double wave_cost[kEvalWaves];
    static __shared__ unsigned long long wave_kept[kEvalWaves];

    const int64_t t = blockIdx.x;
    const int ti = (int)(t / g.tile_cols), tj = (int)(t - (int64_t)ti * g.tile_cols);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float tp = Tp[t], tz = Tz[t];

    // ---- 1. binary factors of the tile
    const float *mz = Mz + t * (int64_t)g.k * g.c;
    for (int idx = tid; idx < g.k * g.izw; idx += kEvalThreads) {
        const int l = idx / g.izw, wq = idx - l * g.izw;
        uint32_t bits = 0u;
        const int j0 = 32 * wq;
#pragma unroll 8
        for (int b = 0; b < 32; ++b)
            if (j0 + b < g.c && mz[(int64_t)l * g.c + j0 + b] >= tz) bits |= 1u << b;
        iz[idx] = bits;
        if (IzOut) IzOut[(t * g.k + l) * (int64_t)g.izw + wq] = bits;
    }
    const float *mp = Mp + t * (int64_t)g.r * g.k;
    for (int idx = tid; idx < g.r * g.ipw; idx += kEvalThreads) {
        const int i = idx / g.ipw, wq = idx - i * g.ipw;
        uint32_t bits = 0u;
        const int l0 = 32 * wq;
        for (int b = 0; b < 32; ++b)
            if (l0 + b < g.k && mp[(int64_t)i * g.k + l0 + b] >= tp) bits |= 1u << b;
        ip[idx] = bits;
        if (IpOut) IpOut[(t * g.r + i) * (int64_t)g.ipw + wq] = bits;
    }
    __syncthreads();

    // ---- 2. rows of the tile: ones of I_a, and magnitudes kept by pruning but cleared by I_a
    double cost = 0.0;
    unsigned long long kept = 0ull;
    const int64_t col0 = (int64_t)tj * g.c;
    for (int i = wave; i < g.r; i += kEvalWaves) {
        const T *wrow = W + ((int64_t)ti * g.r + i) * ldw + col0;
        const uint32_t *ipr = ip + i * g.ipw;
        for (int j = lane * VEC; j < g.c; j += 64 * VEC) {
            // mask bits of columns j .. j + VEC - 1 (inside one 32-bit word, VEC divides 32)
            uint32_t word = 0u;
            for (int q = 0; q < g.ipw; ++q) {
                uint32_t sel = ipr[q];
                while (sel) {
                    const int l = __builtin_ctz(sel) + 32 * q;
                    sel &= sel - 1u;
                    word |= iz[l * g.izw + (j >> 5)];
                }
            }
            const int nvalid = (g.c - j < VEC) ? g.c - j : VEC;
            const uint32_t valid = (nvalid >= 32) ? 0xFFFFFFFFu : ((1u << nvalid) - 1u);
            const uint32_t bits = (word >> (j & 31)) & valid;
            kept += (unsigned long long)__builtin_popcount(bits);
            if (bits == valid) continue; // nothing pruned here
            uint32_t w4[4] = {0u, 0u, 0u, 0u};
            const bool vec = w_vec_ok && (j + VEC <= g.c) && (((col0 + j) % VEC) == 0);
            if (vec) {
                const uint4 v = *reinterpret_cast<const uint4 *>(wrow + j);
                w4[0] = v.x; w4[1] = v.y; w4[2] = v.z; w4[3] = v.w;
            } else if (sizeof(T) == 4) {
                const uint32_t *wr = reinterpret_cast<const uint32_t *>(wrow);
#pragma unroll
                for (int e = 0; e < 4; ++e) w4[e] = (e < nvalid) ? wr[j + e] : 0u;
            } else {
                const uint16_t *wr = reinterpret_cast<const uint16_t *>(wrow);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (e < nvalid) w4[e >> 1] |= (uint32_t)wr[j + e] << (16 * (e & 1));
            }
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float a = piece_abs<T>(w4, e);
                if (e < nvalid && !((bits >> e) & 1u) && a >= w_threshold) cost += (double)a;
            }
        }
    }
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
        Cost[t] = c;
        Kept[t] = kk;
    }
}

size_t threshold_eval_lds_bytes(const Geom &g)
{
    return ((size_t)g.k * g.izw + (size_t)g.r * g.ipw) * 4;
}

template <typename T>
static int launch_eval_t(const Geom &g, const void *dW, int64_t ldw, float w_threshold, const float *dMp,
                         const float *dMz, const float *dTp, const float *dTz, void *dIp, void *dIz, uint64_t *dKept,
                         double *dCost, hipStream_t stream)
{
    const int64_t tiles = (int64_t)g.tile_rows * g.tile_cols;
    if (tiles > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    const size_t smem = (threshold_eval_lds_bytes(g) + 15) / 16 * 16;
    const int w_vec_ok = (((uintptr_t)dW & 15) == 0) && (ldw % Mag<T>::VEC == 0);
    auto kern = threshold_eval_kernel<T>;
    if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
        return LRBI_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(kEvalThreads), smem, stream, g, (const T *)dW, ldw,
                       w_threshold, dMp, dMz, dTp, dTz, (uint32_t *)dIp, (uint32_t *)dIz,
                       (unsigned long long *)dKept, dCost, w_vec_ok);
    LRBI_CHECK_LAUNCH();
    return LRBI_OK;
}

int launch_threshold_eval(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, float w_threshold,
                          const float *dMp, const float *dMz, const float *dTp, const float *dTz, void *dIp, void *dIz,
                          uint64_t *dKept, double *dCost, hipStream_t stream)
{
    switch (dt) {
    case LRBI_F32: return launch_eval_t<float>(g, dW, ldw, w_threshold, dMp, dMz, dTp, dTz, dIp, dIz, dKept, dCost, stream);
    case LRBI_F16: return launch_eval_t<__half>(g, dW, ldw, w_threshold, dMp, dMz, dTp, dTz, dIp, dIz, dKept, dCost, stream);
    case LRBI_BF16:
        return launch_eval_t<__hip_bfloat16>(g, dW, ldw, w_threshold, dMp, dMz, dTp, dTz, dIp, dIz, dKept, dCost, stream);
    default: return LRBI_ERR_DTYPE;
    }
}

} // namespace lrbi
