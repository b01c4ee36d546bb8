// Fused masked product on the vector ALUs: Y = (W o I_a) X for small batches
// (matrix-vector and a few columns) and for fp32, where the work is bound by
// streaming W from HBM once and no matrix-core path applies.
//
// One wavefront owns one row of W at a time.  For each segment of 2048 columns
// the 64 lanes first rebuild the 64 mask words of that segment from the factors
// (Eq. 3; one word per lane) and park them in a wave-private LDS strip; then the
// lanes sweep the segment with 16-byte loads of W, pick their 8 (or 4) mask bits
// out of the strip, and accumulate only the kept weights in fp32 (select, never
// multiply: a pruned weight's stored value cannot reach Y).  A wave reduction
// finishes the row.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "lrbi_internal.hpp"

namespace lrbi {

static constexpr int kGemvThreads = 256;
static constexpr int kGemvWaves = kGemvThreads / 64;
static constexpr int kSegWords = 64;             // mask words per segment (one per lane)
static constexpr int kSegCols = kSegWords * 32;  // 2048 columns

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int VEC = 4;
    __device__ static float to_f32(float v) { return v; }
    __device__ static float from_f32(float v) { return v; }
};
template <> struct Elem<__half> {
    static constexpr int VEC = 8;
    __device__ static float to_f32(__half v) { return __half2float(v); }
    __device__ static __half from_f32(float v) { return __float2half_rn(v); }
};
template <> struct Elem<__hip_bfloat16> {
    static constexpr int VEC = 8;
    __device__ static float to_f32(__hip_bfloat16 v) { return __bfloat162float(v); }
    __device__ static __hip_bfloat16 from_f32(float v) { return __float2bfloat16(v); } // nearest-even
};

template <typename T, int NB>
__global__ __launch_bounds__(kGemvThreads) void valu_gemm_kernel(Geom g, const T *__restrict__ W, int64_t ldw,
                                                                 const uint32_t *__restrict__ Ip,
                                                                 const uint32_t *__restrict__ Iz,
                                                                 const T *__restrict__ X, int64_t ldx, int N,
                                                                 T *__restrict__ Y, int64_t ldy, int w_vec_ok,
                                                                 int x_vec_ok)
{
    constexpr int VEC = Elem<T>::VEC;
    static __shared__ uint32_t strip[kGemvWaves][kSegWords];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * kGemvWaves + wave;
    if (row >= g.m) return; // whole wavefront leaves together; no block-wide barrier below
    const int ti = (int)(row / g.r);
    const int il = (int)(row - (int64_t)ti * g.r);
    const T *wrow = W + row * ldw;
    const int n = (int)g.n;

    for (int q0 = 0; q0 < N; q0 += NB) {
        float acc[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[b] = 0.f;
        const int nb = (N - q0 < NB) ? N - q0 : NB;

        for (int seg = 0; seg < n; seg += kSegCols) {
            // lanes rebuild the mask words of this segment (wave-private strip)
            __builtin_amdgcn_wave_barrier();
            strip[wave][lane] = decode_word(g, Ip, Iz, ti, il, (seg >> 5) + lane);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

            const int seg_end = (seg + kSegCols < n) ? seg + kSegCols : n;
            for (int j = seg + lane * VEC; j < seg_end; j += 64 * VEC) {
                const int rel = j - seg;
                const uint32_t bits = (strip[wave][rel >> 5] >> (rel & 31)) & ((1u << VEC) - 1u);
                if (bits == 0u) continue; // nothing kept in this piece: skip the W load as well
                T wv[VEC];
                if (w_vec_ok && j + VEC <= n) {
                    *reinterpret_cast<uint4 *>(wv) = *reinterpret_cast<const uint4 *>(wrow + j);
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) wv[e] = (j + e < n) ? wrow[j + e] : Elem<T>::from_f32(0.f);
                }
                if (NB == 1 && x_vec_ok && j + VEC <= n) {
                    T xv[VEC];
                    *reinterpret_cast<uint4 *>(xv) = *reinterpret_cast<const uint4 *>(X + j);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const float w = ((bits >> e) & 1u) ? Elem<T>::to_f32(wv[e]) : 0.f;
                        acc[0] = fmaf(w, Elem<T>::to_f32(xv[e]), acc[0]);
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        if (((bits >> e) & 1u) && j + e < n) {
                            const float w = Elem<T>::to_f32(wv[e]);
                            const T *xr = X + (int64_t)(j + e) * ldx + q0;
#pragma unroll
                            for (int b = 0; b < NB; ++b)
                                if (b < nb) acc[b] = fmaf(w, Elem<T>::to_f32(xr[b]), acc[b]);
                        }
                    }
                }
            }
        }
        // wave reduction, fixed order
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float v = acc[b];
#pragma unroll
            for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, 64);
            if (lane == 0 && b < nb) Y[row * ldy + q0 + b] = Elem<T>::from_f32(v);
        }
    }
}

template <typename T>
static int launch_valu_t(const Geom &g, const void *dW, int64_t ldw, const uint32_t *dIp, const uint32_t *dIz,
                         const void *dX, int64_t ldx, int64_t N, void *dY, int64_t ldy, hipStream_t stream)
{
    constexpr int VEC = Elem<T>::VEC;
    const int64_t blocks = (g.m + kGemvWaves - 1) / kGemvWaves;
    if (blocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    const int w_vec_ok = (((uintptr_t)dW & 15) == 0) && (ldw % VEC == 0);
    // contiguous x vector: one column with unit stride between consecutive j
    const int x_vec_ok = (N == 1) && (ldx == 1) && (((uintptr_t)dX & 15) == 0);
    const dim3 grid((unsigned)blocks), block(kGemvThreads);
    if (N == 1)
        LRBI_LAUNCH((valu_gemm_kernel<T, 1>), grid, block, 0, stream, g, (const T *)dW, ldw, dIp, dIz,
                           (const T *)dX, ldx, (int)N, (T *)dY, ldy, w_vec_ok, x_vec_ok);
    else
        LRBI_LAUNCH((valu_gemm_kernel<T, 4>), grid, block, 0, stream, g, (const T *)dW, ldw, dIp, dIz,
                           (const T *)dX, ldx, (int)N, (T *)dY, ldy, w_vec_ok, x_vec_ok);
    return LRBI_OK;
}

int launch_valu_gemm(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, const uint32_t *dIp,
                     const uint32_t *dIz, const void *dX, int64_t ldx, int64_t N, void *dY, int64_t ldy,
                     hipStream_t stream)
{
    switch (dt) {
    case LRBI_F32: return launch_valu_t<float>(g, dW, ldw, dIp, dIz, dX, ldx, N, dY, ldy, stream);
    case LRBI_F16: return launch_valu_t<__half>(g, dW, ldw, dIp, dIz, dX, ldx, N, dY, ldy, stream);
    case LRBI_BF16: return launch_valu_t<__hip_bfloat16>(g, dW, ldw, dIp, dIz, dX, ldx, N, dY, ldy, stream);
    default: return LRBI_ERR_DTYPE;
    }
}

} // namespace lrbi
