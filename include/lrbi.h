/*
 * lrbi.h - low-rank binary index (LRBI) inference path for AMD MI355X (gfx950).
 *
 * C ABI of the library built from paper_1905_05686_amd/csrc.  It implements the
 * inference side of "Network Pruning for Low-Rank Binary Indexing"
 * (arXiv 1905.05686): the pruning mask of a weight matrix is stored, tile by
 * tile, as two small binary factors and rebuilt on the fly as their Boolean
 * product; the mask is applied to the weights and the layer product is taken.
 *
 * Notation follows the paper: W is m x n, a tile is r x c, the rank is k,
 * I_p is r x k and I_z is k x c per tile, the decoded mask is I_a (1 = weight
 * kept, 0 = weight pruned; Sec. 2, Eq. 2).
 *
 * General rules for every entry point
 *   - Returns LRBI_OK (0) or a negative lrbi_status.  Nothing throws or aborts.
 *     Arguments are validated before any GPU work is queued.
 *   - The library allocates nothing, frees nothing, keeps no global state and
 *     never synchronises.  Every buffer belongs to the caller.
 *   - Pointers named d* are DEVICE pointers valid on the device of `stream`;
 *     pointers named h* are HOST pointers.  `stream` is a hipStream_t passed as
 *     void* (NULL = the default stream).  GPU work is queued on it and has not
 *     finished when the call returns; inputs and outputs must stay alive and
 *     unmodified until it has.
 *   - An out-of-bounds buffer is outside the contract: sizes are stated below
 *     and the library trusts them.
 *
 * Logical layout
 *   Tiles are numbered row-major: t = ti * ceil(n / c) + tj, T = ceil(m / r) * ceil(n / c).
 *   Mask bit (i, j) of W belongs to tile (i / r, j / c) at (i mod r, j mod c).
 *   Every tile stores factors of the same rank k (Sec. 3.1).
 *   Edge tiles: when r does not divide m (c does not divide n) the last tile row
 *   (column) is cut off at the matrix edge.  Such a tile keeps full-size factors
 *   in the layouts below and only their first m - ti r rows of I_p and first
 *   n - tj c columns of I_z are used; the kernels ignore the rest, and
 *   lrbi_pack_factors / lrbi_threshold_eval / lrbi_search_thresholds write it as
 *   zero.  (The paper's tilings all divide; this is the library's reading.)  The
 *   tuned kernels need dividing tiles: shapes with edge tiles run on the general
 *   kernels, with the same results.
 *   Per-tile rank (end of Sec. 3.1: every submatrix may choose its own rank): tile t of rank
 *   k_t <= k has zero columns l >= k_t in I_p and zero rows l >= k_t in I_z;
 *   lrbi_pack_factors_ranked writes them so, lrbi_index_bits_ranked counts only k_t.
 *
 * Packed layouts (defined as byte images, little-endian bit order: bit b of a
 * row sits in byte b >> 3 at position b & 7)
 *   I_p packed: T * r rows of ip_row_bytes = 4 * ceil(k / 32) bytes; row
 *               (t, i) holds bits l = 0 .. k-1 of (I_p,t)[i, :].  Pad bits zero.
 *   I_z packed: T * k rows of iz_row_bytes = 8 * ceil(c / 64) bytes; row
 *               (t, l) holds bits j = 0 .. c-1 of (I_z,t)[l, :].  Pad bits zero.
 *   Mask      : m rows of mask_pitch_bytes; row i holds bits j = 0 .. n-1.
 *   lrbi_index_bits reports the two packed sizes.
 */
#ifndef LRBI_H
#define LRBI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LRBI_MAX_RANK 256

typedef struct lrbi_desc {
    int64_t m, n;   /* rows and columns of W                                   */
    int32_t r, c;   /* tile rows and columns; edge tiles are cut off at m, n    */
    int32_t k;      /* rank of every tile, 1 <= k <= LRBI_MAX_RANK             */
    uint32_t flags; /* 0, or LRBI_FLAG_* bits (kernel choice overrides)        */
} lrbi_desc;

/* desc.flags: force a kernel family in lrbi_masked_gemm (default: by N, dtype). */
#define LRBI_FLAG_PATH_MASK   0x0000000Fu
#define LRBI_FLAG_PATH_AUTO   0x00000000u
#define LRBI_FLAG_PATH_VALU   0x00000001u /* bandwidth-bound vector-ALU kernel    */
#define LRBI_FLAG_PATH_MFMA   0x00000002u /* matrix-core kernel (f16 / bf16 only) */
#define LRBI_FLAG_PATH_STREAM 0x00000003u /* row-streaming kernels (W read once, any tile shape): f16 / bf16, N = 1 or a
                                             multiple of 4 up to 32, X contiguous (ldx = N) and 16-byte aligned, W rows
                                             16-byte aligned.  Chosen by the library for such calls when the matrix has
                                             rows for half the compute units, or when its rows are short (64 KB of W per
                                             16 rows on tile shapes the panel kernels take, 256 KB on others); not for
                                             N = 16, 24, 32 on those tile shapes when rows are long (above 128 KB per 16
                                             rows) and there is at most one workgroup per compute unit */
/* desc.flags bits 8..15: split of the n (reduction) range over workgroups for the
 * MFMA path, 0 = chosen by the library.  Values > 1 need a workspace. */
#define LRBI_FLAG_SPLITK_SHIFT 8
#define LRBI_FLAG_SPLITK_MASK  0x0000FF00u
/* desc.flags bits 16..19: MFMA tile variant, 0 = chosen by the library. */
#define LRBI_FLAG_TILE_SHIFT 16
#define LRBI_FLAG_TILE_MASK  0x000F0000u
/* desc.flags: force the generic decode kernel in lrbi_decode_mask. */
#define LRBI_FLAG_DECODE_GENERIC 0x00100000u

typedef enum lrbi_dtype { LRBI_F32 = 0, LRBI_F16 = 1, LRBI_BF16 = 2 } lrbi_dtype;

typedef enum lrbi_status {
    LRBI_OK = 0,
    LRBI_ERR_NULL = -1,      /* a required pointer is NULL                       */
    LRBI_ERR_SHAPE = -2,     /* non-positive size, or beyond an entry point's limit */
    LRBI_ERR_RANK = -3,      /* k outside 1 .. LRBI_MAX_RANK, tile rank outside 0 .. k */
    LRBI_ERR_DTYPE = -4,     /* unknown dtype, or dtype not served by forced path */
    LRBI_ERR_PITCH = -5,     /* pitch / leading dimension too small or misaligned */
    LRBI_ERR_ALIGN = -6,     /* a pointer is not aligned as stated               */
    LRBI_ERR_LAUNCH = -7,    /* the HIP runtime refused a launch                 */
    LRBI_ERR_WORKSPACE = -8, /* forced split needs a larger workspace            */
    LRBI_ERR_FLAGS = -9      /* unknown bits in desc.flags                       */
} lrbi_status;

/* Text for a status code; never NULL, static storage. */
const char *lrbi_strerror(int status);

/*
 * Index size accounting (Sec. 2.2: compression ratio mn / (k(m+n)); Sec. 3.1:
 * every tile is factorised on its own with the same rank; Tables 1 and 3).
 * Host only.  Any out pointer may be NULL.
 *   lrbi_bits   = k * (ceil(n / c) * m + ceil(m / r) * n): bits of the factor pair of all
 *                 tiles, edge tiles counted with the rows / columns they use
 *                 (= T * k * (r + c) when the tiles divide the matrix)
 *   dense_bits  = m * n                bits of the plain binary mask
 *   packed_ip_bytes / packed_iz_bytes  sizes of the packed factor buffers above
 */
int lrbi_index_bits(const lrbi_desc *desc, uint64_t *lrbi_bits, uint64_t *dense_bits,
                    uint64_t *packed_ip_bytes, uint64_t *packed_iz_bytes);

/* The same with a rank per tile (hTileRank [T], 0 <= k_t <= k): sum over tiles of k_t (r_t + c_t). */
int lrbi_index_bits_ranked(const lrbi_desc *desc, const int32_t *hTileRank, uint64_t *lrbi_bits);

/*
 * CSR index size under this library's stated accounting (the paper compares
 * against CSR in Tables 1 and 3 without giving a formula):
 *   bits = nnz * idx_bits + (m + 1) * ptr_bits.        Host only.
 */
int lrbi_csr_bits(uint64_t nnz, int64_t m, int32_t idx_bits, int32_t ptr_bits, uint64_t *bits);

/*
 * Pack factors given one byte per bit into the packed layouts (host only).
 *   hIp01 [T][r][k], hIz01 [T][k][c]: any non-zero byte is a set bit.
 *   hIp_packed: packed_ip_bytes, 4-byte aligned.  hIz_packed: packed_iz_bytes,
 *   8-byte aligned.  Both are fully overwritten (pad bits zero; also zero: what a
 *   cut-off edge tile leaves outside the matrix).
 */
int lrbi_pack_factors(const lrbi_desc *desc, const uint8_t *hIp01, const uint8_t *hIz01,
                      void *hIp_packed, void *hIz_packed);

/*
 * The same for tiles of different ranks (end of Sec. 3.1): hTileRank [T], 0 <= k_t <= k.  The inputs
 * keep the uniform shapes [T][r][k] and [T][k][c]; ranks l >= k_t of tile t are not read and
 * are packed as zero, so every entry point sees a tile of rank k_t.
 */
int lrbi_pack_factors_ranked(const lrbi_desc *desc, const int32_t *hTileRank, const uint8_t *hIp01,
                             const uint8_t *hIz01, void *hIp_packed, void *hIz_packed);

/*
 * Unpack a packed mask (host only): hM01 [m][n] receives 0 / 1 bytes.
 * mask_pitch_bytes >= ceil(n / 8).
 */
int lrbi_unpack_mask(const lrbi_desc *desc, const void *hMask, int64_t mask_pitch_bytes,
                     uint8_t *hM01);

/*
 * Decode the mask of every tile: I_a,t = I_p,t (x) I_z,t with the Boolean
 * product of Eq. 3, (I_a)_{i,j} = OR_l (I_p)_{i,l} AND (I_z)_{l,j}, each tile
 * independently (Sec. 3.1), written as the one-bit-per-weight binary index form
 * (Fig. 1).
 *   dIp_packed, dIz_packed: packed factors (4- and 8-byte aligned).
 *   dMask: m * mask_pitch_bytes bytes, 16-byte aligned; mask_pitch_bytes is a
 *   multiple of 16 and >= ceil(n / 8).  In every row the first
 *   16 * ceil(n / 128) bytes are written (bits >= n as zero); bytes beyond that
 *   up to the pitch are left untouched.
 * One kernel launch on `stream`.
 */
int lrbi_decode_mask(const lrbi_desc *desc, const void *dIp_packed, const void *dIz_packed,
                     void *dMask, int64_t mask_pitch_bytes, void *stream);

/*
 * Workspace the masked product may use for (desc, dtype, N): partial sums when
 * the reduction over n is split across workgroups.  Host only.  *bytes may be 0.
 */
int lrbi_masked_gemm_workspace_bytes(const lrbi_desc *desc, lrbi_dtype dtype, int64_t N,
                                     uint64_t *bytes);

/*
 * Fused masked layer product Y = (W o I_a) X: the mask of Eq. 3 is rebuilt from
 * the factors inside the kernel (it never goes through HBM), applied to W as a
 * masking layer (Sec. 2, Sec. 2.2: a pruned weight contributes nothing, whatever
 * value is stored under it, NaN and Inf included), and multiplied with X.
 *   dW: m x n row-major, leading dimension ldw >= n (elements).
 *   dX: n x N row-major, ldx >= N.   dY: m x N row-major, ldy >= N; overwritten.
 *   W, X, Y share `dtype`.  Products are accumulated in fp32 (order unspecified
 *   but fixed: two calls with the same arguments give identical bits) and
 *   rounded to nearest-even on store.
 *   Pointers must be aligned to the element size; 16-byte aligned W / X / Y with
 *   ldw, ldx, ldy multiples of 8 (f16 / bf16) or 4 (f32) elements take the fast
 *   vector paths, anything else a slower scalar path with the same results.
 *   dWorkspace / workspace_bytes: optional scratch (16-byte aligned).  With NULL
 *   or fewer bytes than lrbi_masked_gemm_workspace_bytes reports, the library
 *   uses an unsplit kernel (slower for small m * N), unless desc.flags forces a
 *   split, which then fails with LRBI_ERR_WORKSPACE.
 * One or two kernel launches on `stream`.
 */
int lrbi_masked_gemm(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                     const void *dIp_packed, const void *dIz_packed, const void *dX, int64_t ldx,
                     int64_t N, void *dY, int64_t ldy, void *dWorkspace, uint64_t workspace_bytes,
                     void *stream);

/*
 * Rows a1-a6 of the hot path in one call: the decoded mask (Eq. 3, layout and pitch rules of lrbi_decode_mask)
 * AND the fused masked product Y = (W o I_a) X (arguments of lrbi_masked_gemm, workspace as sized by
 * lrbi_masked_gemm_workspace_bytes).  For f16 / bf16 layers this is one product launch (plus the split reduction
 * when the plan splits) on the kernels that rebuild the mask in a form they can store on the way, so that the
 * stand-alone decode kernel and its launch drop out: the pipelined tile kernel (c % 128 == 0, or c % 64 == 0 with
 * n % 128 == 0; r % 128 == 0, k <= 64, no cut-off tiles, N > 32, X and W readable in 16-byte pieces), the generic
 * tile kernel (any tile shape and rank, cut-off tiles, N > 4, W readable in 16-byte pieces), and the row-streaming
 * kernels for narrow batches (N = 1 or a multiple of 4 up to 32, any tile shape).  Every other case (fp32, the
 * staged panel kernels, unaligned W) runs lrbi_decode_mask and then lrbi_masked_gemm on `stream`.  Results are
 * bit-identical to those two calls.
 * Errors: those of the two entry points.
 */
int lrbi_decode_and_gemm(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                         const void *dIp_packed, const void *dIz_packed, const void *dX, int64_t ldx, int64_t N,
                         void *dY, int64_t ldy, void *dMask, int64_t mask_pitch_bytes, void *dWorkspace,
                         uint64_t workspace_bytes, void *stream);

/*
 * The masked product of a 3 x 3 convolution layer with padding 1 and stride 1 (the convolution layers of Sec. 4's
 * ResNet32 and AlexNet rows), without the unfolded input matrix: Y = (W o I_a) X where column (b, oh, ow) of X would
 * hold the 9 * cin input values under the filter at output pixel (oh, ow) of image b.  The kernel gathers them from
 * the activation itself.  The paper leaves the 2-D view of a 4-D filter bank open ("reshaping the original binary
 * index matrix can be varied", Sec. 3.1); here
 *   W is m x (9 * cin) with column index (kh * 3 + kw) * cin + ci (filter tap major, channel minor), desc.n = 9 * cin,
 *   and the factors describe that matrix;
 *   dActPadded: the input activation with a zero border of one pixel, [batch][H + 2][Wd + 2][cin], channels
 *   fastest, same dtype as W, 16-byte aligned; the producer of the activation writes the interior and keeps the
 *   border zero (the entry point neither checks nor writes it);
 *   dY: m x (batch * H * Wd) row-major, column index (b * H + oh) * Wd + ow, ldy >= batch * H * Wd.
 * Same arithmetic contract as lrbi_masked_gemm (fp32 accumulation, fixed order, nearest-even store, pruned weights
 * contribute nothing).  Served shapes: f16 / bf16, tile sizes that are multiples of 128 dividing m and 9 * cin,
 * rank <= 64, cin a multiple of 64, 16-byte aligned W rows and I_z; anything else returns LRBI_ERR_SHAPE /
 * LRBI_ERR_ALIGN (the caller can still unfold X and call lrbi_masked_gemm).  Workspace as for lrbi_masked_gemm.
 * One or two kernel launches on `stream`.
 */
int lrbi_masked_conv3x3_workspace_bytes(const lrbi_desc *desc, lrbi_dtype dtype, int64_t batch, int64_t H, int64_t Wd,
                                        uint64_t *bytes);
int lrbi_masked_conv3x3(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                        const void *dIp_packed, const void *dIz_packed, const void *dActPadded, int64_t batch,
                        int64_t H, int64_t Wd, int64_t cin, void *dY, int64_t ldy, void *dWorkspace,
                        uint64_t workspace_bytes, void *stream);

/*
 * lrbi_masked_gemm for callers that cannot allocate device memory and have no workspace to hand over: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, results
 * (identical bits) and launches as lrbi_masked_gemm called with a workspace of
 * lrbi_masked_gemm_workspace_bytes bytes, but the partial sums of a split reduction go to a scratch array
 * of LRBI_STATIC_SCRATCH_BYTES bytes that is part of the library image on every GPU it runs on (held until
 * the process ends).  The call allocates and frees nothing, on the host side or the device side of HIP.
 *   Limit: shapes whose workspace query exceeds LRBI_STATIC_SCRATCH_BYTES return LRBI_ERR_WORKSPACE before
 *   any launch (all five paper-shaped configurations fit: the largest, 4096 x 9216 at N = 128, needs 16 MiB).
 *   The device of `stream` must be the current device (the scratch array is looked up per current device).
 *   All calls on one GPU share that GPU's array: two calls that may overlap in time (different streams, or
 *   graph branches without an edge between them) race on it; calls ordered by one stream do not.
 *   Nothing in the array needs to start at zero: every partial sum is written before it is read.
 */
#define LRBI_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
int lrbi_masked_gemm_static(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                            const void *dIp_packed, const void *dIz_packed, const void *dX, int64_t ldx,
                            int64_t N, void *dY, int64_t ldy, void *stream);

/*
 * One candidate of Algorithm 1 (Sec. 2.1), evaluated for every tile in one launch:
 * the real-valued non-negative factors M_p (r x k) and M_z (k x c) of a tile are turned
 * into binary factors with the tile's thresholds, (I_p)_{i,l} = 1 iff (M_p)_{i,l} >= T_p
 * and (I_z)_{l,j} = 1 iff (M_z)_{l,j} >= T_z; the mask I_a = I_p (x) I_z of Eq. 3 is
 * formed on chip; and the two quantities the search needs come back per tile:
 *   dKept[t]  number of ones of I_a in tile t (its sparsity is S_a = 1 - kept / (r c)),
 *   dCost[t]  sum of M_{i,j} over the tile's entries that magnitude pruning keeps
 *             (I_{i,j} = 1 iff |W_{i,j}| >= w_threshold, Eq. 1 -> Eq. 2) but I_a prunes,
 *             the cost function of Sec. 2.1.  M is the magnitude matrix the factorisation saw
 *             (Sec. 3.2 manipulates the magnitudes and keeps this definition of the cost):
 *             method 1: |W|; 2: |W|^2; 3: `amplify` * |W| where |W| >= w_threshold (which holds
 *             for every entry the cost counts).  Pass the method and amplification given to
 *             lrbi_nmf.  method outside 1 .. 3, or method 3 with amplify not positive and
 *             finite: LRBI_ERR_SHAPE.  amplify is ignored for methods 1 and 2.
 * (lrbi_search_thresholds below runs the sweep over S_p and the bisection on S_z around it.)
 *   dW: m x n row-major, ldw >= n elements, of `dtype`; magnitudes are taken exactly.
 *   dMp: [T][r][k] float, dMz: [T][k][c] float, dTp, dTz: [T] float (T = tiles, row-major
 *   tile order); comparisons are made in single precision.
 *   dIp_packed, dIz_packed: when not NULL, receive the packed binary factors (layouts
 *   above), e.g. for the final conversion with the best thresholds; both or neither.
 *   dKept: [T] uint64, dCost: [T] double (sums accumulated in double, fixed order:
 *   identical bits from call to call).
 * Limits: 4 * (k * 2 * ceil(c / 64) + r * ceil(k / 32)) bytes of factor bits must fit
 * in 64 KiB of on-chip memory (LRBI_ERR_SHAPE otherwise).
 *   dWorkspace / workspace_bytes: optional scratch (8-byte aligned) of at least
 *   lrbi_threshold_eval_workspace_bytes bytes.  With it, a layer of few large tiles is
 *   spread over more workgroups (row bands per tile, partial results added in band order
 *   by a second launch); with NULL or too few bytes one workgroup serves a whole tile.
 *   Results are identical either way for dKept and the packed factors; dCost may differ in
 *   the last bits between the two arrangements (different, each fixed, summation orders).
 * One or two kernel launches on `stream`.
 */
int lrbi_threshold_eval(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                        float w_threshold, int32_t method, float amplify, const float *dMp, const float *dMz, const float *dTp,
                        const float *dTz, void *dIp_packed, void *dIz_packed, uint64_t *dKept,
                        double *dCost, void *dWorkspace, uint64_t workspace_bytes, void *stream);

/* Scratch lrbi_threshold_eval can use for this geometry.  Host only.  *bytes may be 0. */
int lrbi_threshold_eval_workspace_bytes(const lrbi_desc *desc, uint64_t *bytes);

/*
 * The threshold search of Algorithm 1 (Sec. 2.1) for every tile of a layer, entirely on
 * the device: for each S_p of the caller's list (the sweep of the outer loop), T_p is the
 * entry of the tile's ascending-sorted M_p at index round(S_p r k) (+inf at r k: I_p all
 * zero), and S_z is found by bisection on [0, 1], starting from Eq. 7 solved for S_z,
 * S_z = (S^(1/k) - S_p) / (1 - S_p) clipped to [0, 1] (0 when S_p = 1); each of the `steps`
 * probes converts with (T_p, T_z), forms I_a (Eq. 3) and takes its number of ones and
 * its cost exactly as lrbi_threshold_eval does; more ones than round((1 - S) r c) moves
 * the lower end of the interval to the probe, otherwise the upper end, and the next probe is
 * the midpoint.  The probe whose count of ones is closest to that target (the first such)
 * stands for its S_p; it is eligible when it is within `tolerance` ones of the target.
 * Per tile the result is the eligible candidate of least cost (the first in list order on
 * ties); when no S_p has an eligible candidate, the one closest to the target.
 *   dW, ldw, w_threshold, method, amplify, dMp, dMz: as for lrbi_threshold_eval.  M_p, M_z must hold no NaN.
 *   target_sparsity: S, in (0, 1).  sp_values: HOST array of n_sp values in [0, 1].
 *   dTp, dTz [T] float, dKept [T] uint64, dCost [T] double: the winning thresholds of every
 *   tile with their number of ones and cost.  dIp_packed, dIz_packed: when not NULL, the
 *   binary factors converted with the winning thresholds; both or neither.
 *   dWorkspace: required, 16-byte aligned, at least lrbi_search_workspace_bytes bytes (the
 *   sorted factors, per-tile search state, and the evaluation's own scratch).
 * Limits: those of lrbi_threshold_eval (a factor of up to 16384 entries per tile is sorted in
 * on-chip memory, a larger one in the workspace, more slowly); LRBI_ERR_SHAPE otherwise, and
 * for n_sp < 1, steps < 1, tolerance < 0, S outside (0, 1) or an S_p outside [0, 1].
 * Costs of candidates that differ by less than the rounding of a double-precision sum may
 * rank either way.  2 + n_sp (1 + steps .. 2 steps) + (0 .. 2) launches on `stream` (a tile's
 * search state is advanced inside the evaluation launches); the host does not wait for the device.
 */
int lrbi_search_thresholds(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                           float w_threshold, int32_t method, float amplify, const float *dMp,
                           const float *dMz, double target_sparsity, const double *sp_values, int32_t n_sp,
                           int32_t steps, int64_t tolerance, float *dTp, float *dTz,
                           uint64_t *dKept, double *dCost, void *dIp_packed, void *dIz_packed,
                           void *dWorkspace, uint64_t workspace_bytes, void *stream);

/* Scratch lrbi_search_thresholds needs for this geometry.  Host only. */
int lrbi_search_workspace_bytes(const lrbi_desc *desc, uint64_t *bytes);

/*
 * Backward pass through the masking layer (Sec. 2: the decoded index is a binary masking layer
 * on W, so retraining with it sends gradients through the kept weights only).  With
 * Y = (W o I_a) X (lrbi_masked_gemm) and dY the gradient with respect to Y, m x N:
 *
 * lrbi_masked_gemm_t: dX = (W o I_a)^T dY, n x N, the gradient with respect to X.  The mask is
 *   rebuilt from the factors inside the kernel and applied as a select (a pruned weight's stored
 *   value, NaN and Inf included, never reaches dX).
 *   dW: m x n row-major, ldw >= n.  dDY: m x N row-major, lddy >= N.  dDX: n x N row-major,
 *   lddx >= N; overwritten.  All of `dtype`; fp32 accumulation in a fixed order (identical bits
 *   from call to call), rounded to nearest-even on store.  Pointers aligned to the element size;
 *   f16 / bf16 with 16-byte aligned W, ldw % 8 == 0 and n % 8 == 0 run on the matrix cores at
 *   any N, everything else on a plain (and for large m slow) vector-ALU kernel with the same results.
 *   dWorkspace / workspace_bytes: optional scratch (16-byte aligned) of at least
 *   lrbi_masked_gemm_t_workspace_bytes bytes: partial sums when the reduction over m is split
 *   across workgroups; with NULL or too few bytes it is not split (slower for small n * N).
 *   One or two kernel launches on `stream`.
 *
 * lrbi_masked_grad: dW = (dY X^T) o I_a, m x n, the gradient with respect to W: entry (i, j) is
 *   sum_q dY[i, q] X[j, q] where I_a keeps the weight and exactly 0 where it prunes it.
 *   dDY: m x N, lddy >= N.  dX: n x N, ldx >= N.  dDW: m x n, lddw >= n; overwritten (every
 *   entry is written).  Same dtype, accumulation and rounding rules as above; f16 / bf16 run on
 *   the matrix cores at any N (16-byte aligned dY, X with lddy, ldx, N multiples of 8, and
 *   16-byte aligned dW rows, take the vector paths inside it).  One kernel launch on `stream`.
 */
int lrbi_masked_gemm_t_workspace_bytes(const lrbi_desc *desc, lrbi_dtype dtype, int64_t N,
                                       uint64_t *bytes);
int lrbi_masked_gemm_t(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                       const void *dIp_packed, const void *dIz_packed, const void *dDY,
                       int64_t lddy, int64_t N, void *dDX, int64_t lddx, void *dWorkspace,
                       uint64_t workspace_bytes, void *stream);
int lrbi_masked_grad(const lrbi_desc *desc, lrbi_dtype dtype, const void *dDY, int64_t lddy,
                     const void *dX, int64_t ldx, int64_t N, const void *dIp_packed,
                     const void *dIz_packed, void *dDW, int64_t lddw, void *stream);

/*
 * One LSTM step on a masked gate matrix (the paper's LSTM model, Sec. 4; it prints no cell
 * equations, the usual ones are used).  desc: W is m x n with m = 4 H (row blocks i, f, g, o of
 * H rows each) and n = the length of the stacked input [x_t; h_{t-1}].  Per call:
 *   z = (W o I_a) XH                         (as lrbi_masked_gemm, kept in fp32)
 *   c = sigm(z_f) c + sigm(z_i) tanh(z_g)    (dC, H x B fp32, updated in place)
 *   h = sigm(z_o) tanh(c)                    (rounded to `dtype`, written to dH1 and, when not
 *                                             NULL, dH2: e.g. the h rows of this layer's next
 *                                             input and the x rows of the next layer's input)
 * The gate product leaves the fp32 partial sums of its slices in the workspace and one more
 * kernel adds them and applies the cell equations; z is never rounded to `dtype`.
 *   dtype: LRBI_F16 or LRBI_BF16 (LRBI_ERR_DTYPE otherwise).  dW 16-byte aligned, ldw % 8 == 0,
 *   n % 8 == 0 (LRBI_ERR_ALIGN otherwise).  dXH: n x B, ldxh >= B.  dC: ldc >= B.  dH1 / dH2: H x B,
 *   ldh1 / ldh2 >= B; they may point into the buffer dXH points into (the product has finished
 *   reading it when they are written).  dWorkspace: required, 16-byte aligned, at least
 *   lrbi_lstm_step_workspace_bytes bytes (LRBI_ERR_WORKSPACE otherwise).  m % 4 != 0 is
 *   LRBI_ERR_SHAPE.  Two kernel launches on `stream`; a single one (product and cell equations
 *   in one kernel, nothing through the workspace, same results bit for bit) when neither dH1
 *   nor dH2 overlaps the n x B input, B is a multiple of 4 up to 32, H and the tile height r are
 *   multiples of 4 and the shape is one the row-streaming product kernel serves: a caller that
 *   alternates between two input buffers per layer gets that form.
 */
int lrbi_lstm_step_workspace_bytes(const lrbi_desc *desc, lrbi_dtype dtype, int64_t B, uint64_t *bytes);
int lrbi_lstm_step(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                   const void *dIp_packed, const void *dIz_packed, const void *dXH, int64_t ldxh,
                   int64_t B, float *dC, int64_t ldc, void *dH1, int64_t ldh1, void *dH2,
                   int64_t ldh2, void *dWorkspace, uint64_t workspace_bytes, void *stream);

/*
 * Non-negative factorisation of the magnitude matrix, every tile on its own (Algorithm 1's first
 * step, Sec. 2.1: M = |W| ~ M_p M_z with M_p (r x k), M_z (k x c) >= 0, minimising the Frobenius
 * distance).  The paper uses an off-the-shelf library and names no algorithm; this entry point
 * runs `iters` multiplicative updates of Lee and Seung for that objective from the caller's
 * starting point, M_z first, then M_p:
 *     M_z <- M_z * (M_p^T M) / (M_p^T M_p M_z + eps),   M_p <- M_p * (M M_z^T) / (M_p M_z M_z^T + eps)
 * Its result feeds lrbi_search_thresholds.
 *   method (Sec. 3.2, weight-magnitude manipulation, applied to |W| on the fly): 1 none, 2 squared,
 *   3 multiplied by `amplify` (the paper's 1 / (1 - S)) where |W| >= w_threshold.  W must be finite.
 *   dW: m x n of `dtype`, ldw >= n.  dMp [T][r][k], dMz [T][k][c] float: on entry the (positive,
 *   e.g. uniform random) starting point, on return the factors; the rows / columns a cut-off edge
 *   tile does not use are left as given.  eps > 0.  fp32 arithmetic, fixed summation order.
 *   dWorkspace: required, 16-byte aligned, at least lrbi_nmf_workspace_bytes bytes (a second copy of
 *   both factors and one k x k matrix per tile).  Any rank the descriptor allows (up to LRBI_MAX_RANK);
 *   method outside 1 .. 3, iters < 0 or eps <= 0 are LRBI_ERR_SHAPE.  2 + 4 iters (+ 2) kernel launches
 *   on `stream`.
 */
int lrbi_nmf_workspace_bytes(const lrbi_desc *desc, uint64_t *bytes);
int lrbi_nmf(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw, int32_t method,
             float w_threshold, float amplify, float *dMp, float *dMz, int32_t iters, float eps,
             void *dWorkspace, uint64_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LRBI_H */
