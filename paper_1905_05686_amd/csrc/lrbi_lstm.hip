// One LSTM step on a masked gate matrix: the gate product z = (W o I_a) [x_t; h_{t-1}] runs on the matrix-core
// kernels of lrbi_gemm_mfma.hip, which leave the fp32 partial planes of their slices in the workspace; the kernel
// here adds the planes (slice order) and applies the cell equations in the same pass, so the pre-activations never
// go through HBM in the storage dtype and no separate reduction or gate kernel runs.
//
// The paper evaluates an LSTM (Sec. 4) without printing cell equations; the usual ones are used:
// rows of W are [i; f; g; o] blocks of H = m / 4 rows, no bias,
//   c_t = sigm(z_f) c_{t-1} + sigm(z_i) tanh(z_g),   h_t = sigm(z_o) tanh(c_t),
// c kept in fp32, h rounded (nearest-even) to the storage dtype.
#include <math.h>

#include "lrbi_internal.hpp"
#include "lrbi_mfma_common.hpp"

namespace lrbi {

__device__ __forceinline__ float sigm(float z) { return 1.f / (1.f + expf(-z)); }

// One lane per (hidden unit j, batch column b): consecutive lanes take consecutive b, so every plane row is read in
// one piece; the 4 x slices loads of a lane are independent of each other.
template <typename Tag>
__global__ __launch_bounds__(256) void lstm_cell_kernel(const float *__restrict__ P, int slices, int64_t m, int64_t ldp,
                                                        int B, float *__restrict__ C, int64_t ldc,
                                                        uint16_t *__restrict__ H1, int64_t ldh1,
                                                        uint16_t *__restrict__ H2, int64_t ldh2)
{
    const int64_t H = m / 4;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= H * B) return;
    const int64_t j = e / B;
    const int b = (int)(e - j * B);
    float z[4] = {0.f, 0.f, 0.f, 0.f}; // gates i, f, g, o; planes added in slice order
    for (int k = 0; k < slices; ++k) {
        const float *plane = P + ((int64_t)k * m + j) * ldp + b;
#pragma unroll
        for (int gate = 0; gate < 4; ++gate) z[gate] += plane[gate * H * ldp];
    }
    const float c = sigm(z[1]) * C[j * ldc + b] + sigm(z[0]) * tanhf(z[2]);
    const float h = sigm(z[3]) * tanhf(c);
    C[j * ldc + b] = c;
    const uint16_t hs = cvt_store(Tag{}, h);
    H1[j * ldh1 + b] = hs;
    if (H2) H2[j * ldh2 + b] = hs;
}

int launch_lstm_cell(lrbi_dtype dt, const float *dPlanes, int slices, int64_t m, int64_t ldp, int64_t B, float *dC,
                     int64_t ldc, void *dH1, int64_t ldh1, void *dH2, int64_t ldh2, hipStream_t stream)
{
    const int64_t items = (m / 4) * B;
    const int64_t blocks = (items + 255) / 256;
    if (blocks > 0x7FFFFFFF) return LRBI_ERR_SHAPE;
    if (dt == LRBI_F16)
        LRBI_LAUNCH(lstm_cell_kernel<F16Tag>, dim3((unsigned)blocks), dim3(256), 0, stream, dPlanes, slices, m, ldp,
                           (int)B, dC, ldc, (uint16_t *)dH1, ldh1, (uint16_t *)dH2, ldh2);
    else if (dt == LRBI_BF16)
        LRBI_LAUNCH(lstm_cell_kernel<BF16Tag>, dim3((unsigned)blocks), dim3(256), 0, stream, dPlanes, slices, m, ldp,
                           (int)B, dC, ldc, (uint16_t *)dH1, ldh1, (uint16_t *)dH2, ldh2);
    else
        return LRBI_ERR_DTYPE;
    return LRBI_OK;
}

} // namespace lrbi
