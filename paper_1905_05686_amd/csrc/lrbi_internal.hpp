// Internal declarations shared by the host entry points and the gfx950 kernels.
// Nothing here is part of the C ABI (that is include/lrbi.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <map>
#include <mutex>
#include <tuple>
#include <utility>

#include "lrbi.h"

namespace lrbi {

// Geometry of one problem, precomputed on the host and passed by value to kernels.
struct Geom {
    int64_t m, n;      // rows / columns of W
    int32_t r, c, k;   // tile rows, tile columns, rank
    int32_t tile_cols; // ceil(n / c)
    int32_t tile_rows; // ceil(m / r)
    int32_t ragged;    // r does not divide m or c does not divide n: the last tile row / column is cut off
    int32_t ipw;       // 32-bit words per packed I_p row  = ceil(k / 32)
    int32_t izw;       // 32-bit words per packed I_z row  = 2 * ceil(c / 64)
};

int validate_desc(const lrbi_desc *d);
Geom make_geom(const lrbi_desc *d);

// kernel launchers (each returns an lrbi_status)
int launch_decode(const Geom &g, uint32_t flags, const uint32_t *dIp, const uint32_t *dIz, void *dMask,
                  int64_t pitch_bytes, hipStream_t stream);
int launch_valu_gemm(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, const uint32_t *dIp,
                     const uint32_t *dIz, const void *dX, int64_t ldx, int64_t N, void *dY, int64_t ldy,
                     hipStream_t stream);

// candidate evaluation of Algorithm 1 (lrbi_alg1.hip)
struct EvalPlan {
    int bands;         // row bands per tile (workgroups per tile)
    int rows_per_band;
    uint64_t workspace_bytes;
};
// how the cost of a candidate sees the magnitudes (Sec. 3.2: the cost keeps its definition, on manipulated magnitudes)
struct CostManip {
    bool squared;  // method 2: sum of squared magnitudes
    double scale;  // method 3: the amplification, common to every counted weight; 1 otherwise
};
EvalPlan plan_threshold_eval(const Geom &g);
size_t threshold_eval_lds_bytes(const Geom &g);
int launch_threshold_eval(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, float w_threshold, CostManip manip,
                          const float *dMp, const float *dMz, const float *dTp, const float *dTz, void *dIp, void *dIz,
                          uint64_t *dKept, double *dCost, void *dWorkspace, hipStream_t stream);

// threshold search of Algorithm 1 (lrbi_alg1.hip): workspace layout (byte offsets) and sizes
struct SearchPlan {
    int np, nz;                 // entries of one tile's M_p, M_z
    int64_t stride_p, stride_z; // floats between two tiles' sorted factors in the workspace
    uint64_t off_sorted_mp, off_sorted_mz, off_state, off_tp, off_tz, off_kept, off_cost, off_eval, bytes;
};
SearchPlan plan_search(const Geom &g);
int launch_search(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, float w_threshold, CostManip manip,
                  const float *dMp,
                  const float *dMz, double target_sparsity, int n_sp, const double *sp_values, int steps,
                  int64_t tolerance, float *dTpBest, float *dTzBest, uint64_t *dKeptBest, double *dCostBest, void *dIp,
                  void *dIz, void *dWorkspace, hipStream_t stream);

// backward pass through the masking layer (lrbi_backward.hip)
struct BwdPlan {
    bool mfma;     // matrix-core kernel (f16 / bf16, aligned operands, N > 4); otherwise the vector-ALU kernel
    int bq;        // batch columns per workgroup
    int slices;    // slices over the rows of W (partial planes through the workspace when > 1)
    int64_t iper;  // rows of W per slice
    uint64_t workspace_bytes;
};
BwdPlan plan_gemm_t(const Geom &g, lrbi_dtype dt, int64_t N, bool aligned);
int launch_gemm_t(const Geom &g, const BwdPlan &plan, lrbi_dtype dt, const void *dW, int64_t ldw, const uint32_t *dIp,
                  const uint32_t *dIz, const void *dDY, int64_t lddy, int64_t N, void *dDX, int64_t lddx,
                  void *dWorkspace, hipStream_t stream);
// the pipelined transposed product (lrbi_gemm_pipe_t.hip)
bool pipe_t_ok(const Geom &g, const void *dW, int64_t ldw, const void *dIz, const void *dDY, int64_t lddy, int64_t N);
int pipe_t_slices(const Geom &g, int64_t N, int max_slices, int64_t *iper);
int launch_pipe_t_gemm(const Geom &g, int slices, int64_t iper, lrbi_dtype dt, const void *dW, int64_t ldw,
                       const uint32_t *dIp, const uint32_t *dIz, const void *dDY, int64_t lddy, int64_t N, void *dDX,
                       int64_t lddx, void *dWorkspace, hipStream_t stream);
int launch_grad(const Geom &g, lrbi_dtype dt, bool mfma, const void *dDY, int64_t lddy, const void *dX, int64_t ldx,
                int64_t N, const uint32_t *dIp, const uint32_t *dIz, void *dDW, int64_t lddw, hipStream_t stream);

struct MfmaPlan {
    int tile;     // tile variant id (1-based, see lrbi_gemm_mfma.hip)
    int bm, bn;   // workgroup tile
    int splitk;   // number of slices of the n range
    int64_t kper; // columns of W per slice (multiple of the kernel's BK)
    uint64_t workspace_bytes;
    // leave the fp32 planes of the slices in the workspace ([slice][m][ldp], ldp = N rounded up to 4) and skip the
    // reduction into Y: a fused consumer (the LSTM cell kernel) adds and uses them
    bool planes_only = false;
};
MfmaPlan plan_mfma(const Geom &g, uint32_t flags, int64_t N);
// Where the tile kernel leaves the decoded mask as a by-product (rows of 16-byte pieces, one bit per weight), or {nullptr, 0}.
struct MaskOut {
    void *ptr;
    int64_t pitch16; // 16-byte pieces per mask row
};
int launch_mfma_gemm(const Geom &g, const MfmaPlan &plan, lrbi_dtype dt, const void *dW, int64_t ldw,
                     const uint32_t *dIp, const uint32_t *dIz, const void *dX, int64_t ldx, int64_t N,
                     void *dY, int64_t ldy, void *dWorkspace, hipStream_t stream, MaskOut mo = {nullptr, 0});
// true when launch_mfma_gemm would run the kernel that can leave the mask behind (and so honours MaskOut)
bool mfma_gemm_emits_mask(const Geom &g, const MfmaPlan &plan, const void *dW, int64_t ldw, const void *dIz,
                          const void *dX, int64_t ldx, int64_t N);

// row-streaming kernel for narrow batches (lrbi_gemm_stream.hip)
bool stream_ok(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, const void *dX, int64_t ldx, int64_t N, int cus);
int launch_stream_lstm(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, const uint32_t *dIp,
                       const uint32_t *dIz, const void *dXH, int64_t B, float *dC, int64_t ldc, void *dH1, int64_t ldh1,
                       void *dH2, int64_t ldh2, int cus, hipStream_t stream);
int launch_stream_gemm(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, const uint32_t *dIp,
                       const uint32_t *dIz, const void *dX, int64_t N, void *dY, int64_t ldy, float *dP, int64_t ldp,
                       int cus, hipStream_t stream, MaskOut mo = {nullptr, 0});

// a 3 x 3 convolution with padding 1 read as a product (lrbi_gemm_pipe.hip): the activation is zero-padded,
// [batch][H + 2][Wd + 2][cin] with channels fastest; reduction index = (kh * 3 + kw) * cin + ci
struct ConvGeom {
    int cin, H, Wd; // channels, output height and width
};
bool pipe_conv_ok(const Geom &g, const ConvGeom &cg, int64_t batch, const void *dIz, const void *dAct, int64_t ldw);
int launch_pipe_conv(const Geom &g, const MfmaPlan &plan, lrbi_dtype dt, const ConvGeom &cg, const void *dW, int64_t ldw,
                     const uint32_t *dIp, const uint32_t *dIz, const void *dAct, int64_t N, void *dY, int64_t ldy,
                     void *dWorkspace, hipStream_t stream);

int launch_mfma_conv(const Geom &g, const MfmaPlan &plan, lrbi_dtype dt, const ConvGeom &cg, const void *dW, int64_t ldw,
                     const uint32_t *dIp, const uint32_t *dIz, const void *dAct, int64_t N, void *dY, int64_t ldy,
                     void *dWorkspace, hipStream_t stream);

// software-pipelined tile kernel (lrbi_gemm_pipe.hip)
bool pipe_shape_ok(const Geom &g);
bool pipe_ok(const Geom &g, const void *dIz, const void *dX, int64_t ldw, int64_t ldx, int64_t N);
int launch_pipe_gemm(const Geom &g, const MfmaPlan &plan, lrbi_dtype dt, int pf, const void *dW, int64_t ldw,
                     const uint32_t *dIp, const uint32_t *dIz, const void *dX, int64_t ldx, int64_t N, void *dY,
                     int64_t ldy, void *dWorkspace, hipStream_t stream, MaskOut mo = {nullptr, 0});

// non-negative factorisation of the magnitude matrix (lrbi_nmf.hip)
uint64_t nmf_workspace_bytes(const Geom &g);
int launch_nmf(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, int method, float w_threshold, float amplify,
               float *dMp, float *dMz, int iters, float eps, void *dWorkspace, hipStream_t stream);

// LSTM cell on the fp32 planes of a gate product (lrbi_lstm.hip)
int launch_lstm_cell(lrbi_dtype dt, const float *dPlanes, int slices, int64_t m, int64_t ldp, int64_t B, float *dC,
                     int64_t ldc, void *dH1, int64_t ldh1, void *dH2, int64_t ldh2, hipStream_t stream);

// register budget of a kernel, as resident wavefronts per SIMD (a host-only build ignores it)
#if defined(__HIP__)
#define LRBI_WAVES_PER_SIMD(n) __attribute__((amdgpu_waves_per_eu(n, n)))
#else
#define LRBI_WAVES_PER_SIMD(n)
#endif

// Kernel launch with its own status: hipLaunchKernel returns the error of this launch, so an error that an
// earlier HIP call of the caller left behind on this thread is neither reported as ours nor cleared.
template <typename... P, size_t... I>
inline hipError_t launch_kernel_impl(void (*kern)(P...), dim3 grid, dim3 block, size_t smem, hipStream_t stream,
                                     std::tuple<P...> &vals, std::index_sequence<I...>)
{
    void *ptrs[sizeof...(P) ? sizeof...(P) : 1] = {(void *)&std::get<I>(vals)...};
    return hipLaunchKernel((const void *)kern, grid, block, ptrs, smem, stream);
}
template <typename... P, typename... A>
inline hipError_t launch_kernel(void (*kern)(P...), dim3 grid, dim3 block, size_t smem, hipStream_t stream, A &&...args)
{
    static_assert(sizeof...(P) == sizeof...(A), "kernel argument count");
    std::tuple<P...> vals(static_cast<P>(args)...); // converted to the kernel's parameter types, by value
    return launch_kernel_impl(kern, grid, block, smem, stream, vals, std::index_sequence_for<P...>{});
}
#define LRBI_LAUNCH(kern, grid, block, smem, stream, ...)                                                   \
    do {                                                                                                    \
        if (::lrbi::launch_kernel(kern, grid, block, smem, stream, __VA_ARGS__) != hipSuccess)              \
            return LRBI_ERR_LAUNCH;                                                                         \
    } while (0)

// Raises a kernel's dynamic LDS limit; asked of the runtime once per (device, kernel, size reached), not per call.
inline hipError_t set_max_lds(const void *kern, int bytes)
{
    static std::mutex mu;
    static std::map<std::pair<int, const void *>, int> granted;
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) device = 0;
    std::lock_guard<std::mutex> lock(mu);
    int &have = granted[std::make_pair(device, kern)];
    if (have >= bytes) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) have = bytes;
    return e;
}
// Compute units of the device `stream` belongs to (the persistent kernels size their grids by it); looked up once
// per device.
inline int compute_units_of(hipStream_t stream)
{
    static std::mutex mu;
    static std::map<int, int> known;
    int device = 0;
    if (hipStreamGetDevice(stream, &device) != hipSuccess && hipGetDevice(&device) != hipSuccess) device = 0;
    std::lock_guard<std::mutex> lock(mu);
    int &cus = known[device];
    if (cus <= 0) {
        int v = 0;
        cus = (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && v > 0) ? v : 256;
    }
    return cus;
}
#define LRBI_SET_MAX_LDS(kern, bytes)                                                                       \
    do {                                                                                                    \
        if (::lrbi::set_max_lds((const void *)(kern), (int)(bytes)) != hipSuccess) return LRBI_ERR_LAUNCH;  \
    } while (0)

#if defined(__HIPCC__)
// ---------------------------------------------------------------------------
// Device helpers for Eq. 3 on packed factors.
// ---------------------------------------------------------------------------

// 32 consecutive bits of a packed I_z row starting at bit offset `off`
// (off may be negative: the window starts before the row; off > -32).
// Words beyond the row read as zero.
__device__ __forceinline__ uint32_t iz_window(const uint32_t *__restrict__ zr, int izw, int off)
{
    if (off >= 0) {
        const int q = off >> 5, s = off & 31;
        const uint32_t a = (q < izw) ? zr[q] : 0u;
        const uint32_t b = (q + 1 < izw) ? zr[q + 1] : 0u;
        return s ? ((a >> s) | (b << (32 - s))) : a;
    }
    return zr[0] << (-off);
}

// bits [lo, hi) of a 32-bit word set, 0 <= lo, hi <= 32
__device__ __forceinline__ uint32_t bit_range(int lo, int hi)
{
    if (hi <= lo) return 0u;
    const uint32_t upper = (hi >= 32) ? 0xFFFFFFFFu : ((1u << hi) - 1u);
    const uint32_t lower = (lo >= 32) ? 0xFFFFFFFFu : ((1u << lo) - 1u);
    return upper & ~lower;
}

// One 32-bit word of the decoded mask: bits j = 32*w .. 32*w+31 of mask row
// (ti * r + il).  Generic in r, c, k; bits at or beyond column n come out zero.
// Row i of a tile's mask is the OR of the I_z rows selected by row i of I_p (Eq. 3).
__device__ __forceinline__ uint32_t decode_word(const Geom &g, const uint32_t *__restrict__ Ip,
                                                const uint32_t *__restrict__ Iz, int ti, int il, int w)
{
    const int64_t j0 = (int64_t)w * 32;
    if (j0 >= g.n) return 0u;
    const int64_t j1 = (j0 + 32 < g.n) ? j0 + 32 : g.n;
    int tj = (int)(j0 / g.c);
    uint32_t acc = 0u;
    for (int64_t tbeg = (int64_t)tj * g.c; tbeg < j1; tbeg += g.c, ++tj) {
        const int64_t t = (int64_t)ti * g.tile_cols + tj;
        const uint32_t *ip = Ip + (t * g.r + il) * g.ipw;
        const uint32_t *izt = Iz + t * g.k * (int64_t)g.izw;
        const int off = (int)(j0 - tbeg); // -32 < off < c
        const uint32_t valid = bit_range(off < 0 ? -off : 0, (g.c - off < 32) ? g.c - off : 32);
        uint32_t v = 0u;
        for (int iw = 0; iw < g.ipw; ++iw) {
            uint32_t sel = ip[iw];
            while (sel) {
                const int l = __builtin_ctz(sel) + 32 * iw;
                sel &= sel - 1u;
                v |= iz_window(izt + (int64_t)l * g.izw, g.izw, off);
            }
        }
        acc |= v & valid;
    }
    // a tile cut off at the right edge: whatever its I_z holds beyond column n stays out
    if (j1 - j0 < 32) acc &= bit_range(0, (int)(j1 - j0));
    return acc;
}
#endif // __HIPCC__

} // namespace lrbi
