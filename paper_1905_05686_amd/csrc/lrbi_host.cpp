// Host side of the LRBI library: descriptor validation, index-size accounting,
// factor packing, workspace queries, and argument checks + dispatch of every GPU entry point.
#include <string.h>

#include "lrbi_internal.hpp"

namespace lrbi {

int validate_desc(const lrbi_desc *d)
{
    if (!d) return LRBI_ERR_NULL;
    if (d->m <= 0 || d->n <= 0 || d->r <= 0 || d->c <= 0) return LRBI_ERR_SHAPE;
    // columns are indexed with 32-bit integers inside the kernels
    if (d->n > (int64_t)0x7FFFFF00 || d->m > (int64_t)0x7FFFFF00) return LRBI_ERR_SHAPE;
    if (d->k < 1 || d->k > LRBI_MAX_RANK) return LRBI_ERR_RANK;
    const uint32_t known = LRBI_FLAG_PATH_MASK | LRBI_FLAG_SPLITK_MASK | LRBI_FLAG_TILE_MASK |
                           LRBI_FLAG_DECODE_GENERIC;
    if (d->flags & ~known) return LRBI_ERR_FLAGS;
    const uint32_t path = d->flags & LRBI_FLAG_PATH_MASK;
    if (path > LRBI_FLAG_PATH_STREAM) return LRBI_ERR_FLAGS;
    return LRBI_OK;
}

Geom make_geom(const lrbi_desc *d)
{
    Geom g;
    g.m = d->m;
    g.n = d->n;
    g.r = d->r;
    g.c = d->c;
    g.k = d->k;
    g.tile_cols = (int32_t)((d->n + d->c - 1) / d->c);
    g.tile_rows = (int32_t)((d->m + d->r - 1) / d->r);
    g.ragged = (d->m % d->r != 0 || d->n % d->c != 0) ? 1 : 0;
    g.ipw = (d->k + 31) / 32;
    g.izw = 2 * ((d->c + 63) / 64);
    return g;
}

static inline bool aligned_to(const void *p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

} // namespace lrbi

using namespace lrbi;

extern "C" const char *lrbi_strerror(int status)
{
    switch (status) {
    case LRBI_OK: return "ok";
    case LRBI_ERR_NULL: return "a required pointer is NULL";
    case LRBI_ERR_SHAPE: return "bad shape: a size is not positive or exceeds a limit of the entry point";
    case LRBI_ERR_RANK: return "rank k outside 1..LRBI_MAX_RANK";
    case LRBI_ERR_DTYPE: return "unknown dtype or dtype not served by the forced kernel path";
    case LRBI_ERR_PITCH: return "pitch or leading dimension too small or misaligned";
    case LRBI_ERR_ALIGN: return "pointer not aligned as required";
    case LRBI_ERR_LAUNCH: return "HIP runtime refused the kernel launch";
    case LRBI_ERR_WORKSPACE: return "workspace too small for the forced split";
    case LRBI_ERR_FLAGS: return "unknown bits in desc.flags";
    default: return "unknown lrbi status";
    }
}

extern "C" int lrbi_index_bits(const lrbi_desc *desc, uint64_t *lrbi_bits, uint64_t *dense_bits,
                               uint64_t *packed_ip_bytes, uint64_t *packed_iz_bytes)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    const Geom g = make_geom(desc);
    const uint64_t tiles = (uint64_t)g.tile_rows * (uint64_t)g.tile_cols;
    // every tile column stores m rows of I_p, every tile row n columns of I_z (edge tiles are cut off)
    if (lrbi_bits)
        *lrbi_bits = (uint64_t)g.k * ((uint64_t)g.tile_cols * (uint64_t)g.m + (uint64_t)g.tile_rows * (uint64_t)g.n);
    if (dense_bits) *dense_bits = (uint64_t)g.m * (uint64_t)g.n;
    if (packed_ip_bytes) *packed_ip_bytes = tiles * (uint64_t)g.r * (uint64_t)g.ipw * 4u;
    if (packed_iz_bytes) *packed_iz_bytes = tiles * (uint64_t)g.k * (uint64_t)g.izw * 4u;
    return LRBI_OK;
}

extern "C" int lrbi_csr_bits(uint64_t nnz, int64_t m, int32_t idx_bits, int32_t ptr_bits, uint64_t *bits)
{
    if (!bits) return LRBI_ERR_NULL;
    if (m <= 0 || idx_bits <= 0 || ptr_bits < 0) return LRBI_ERR_SHAPE;
    *bits = nnz * (uint64_t)idx_bits + (uint64_t)(m + 1) * (uint64_t)ptr_bits;
    return LRBI_OK;
}

// Packs 0/1 factors; bits that no mask entry uses are written as zero: ranks at or beyond a tile's
// own rank, rows of I_p and columns of I_z that a cut-off edge tile leaves outside the matrix.
static int pack_impl(const lrbi_desc *desc, const int32_t *hTileRank, const uint8_t *hIp01, const uint8_t *hIz01,
                     void *hIp_packed, void *hIz_packed)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!hIp01 || !hIz01 || !hIp_packed || !hIz_packed) return LRBI_ERR_NULL;
    if (!aligned_to(hIp_packed, 4) || !aligned_to(hIz_packed, 8)) return LRBI_ERR_ALIGN;
    const Geom g = make_geom(desc);
    const int64_t tiles = (int64_t)g.tile_rows * g.tile_cols;
    if (hTileRank)
        for (int64_t t = 0; t < tiles; ++t)
            if (hTileRank[t] < 0 || hTileRank[t] > g.k) return LRBI_ERR_RANK;
    uint8_t *ip = (uint8_t *)hIp_packed;
    uint8_t *iz = (uint8_t *)hIz_packed;
    const int64_t ip_row = (int64_t)g.ipw * 4, iz_row = (int64_t)g.izw * 4;
    memset(ip, 0, (size_t)(tiles * g.r * ip_row));
    memset(iz, 0, (size_t)(tiles * g.k * iz_row));
    for (int64_t t = 0; t < tiles; ++t) {
        const int64_t ti = t / g.tile_cols, tj = t - ti * g.tile_cols;
        const int64_t rt = (g.m - ti * g.r < g.r) ? g.m - ti * g.r : g.r;
        const int64_t ct = (g.n - tj * g.c < g.c) ? g.n - tj * g.c : g.c;
        const int kt = hTileRank ? hTileRank[t] : g.k;
        for (int64_t i = 0; i < rt; ++i) {
            const uint8_t *src = hIp01 + (t * g.r + i) * g.k;
            uint8_t *dst = ip + (t * g.r + i) * ip_row;
            for (int l = 0; l < kt; ++l)
                if (src[l]) dst[l >> 3] |= (uint8_t)(1u << (l & 7));
        }
        for (int64_t l = 0; l < kt; ++l) {
            const uint8_t *src = hIz01 + (t * g.k + l) * g.c;
            uint8_t *dst = iz + (t * g.k + l) * iz_row;
            for (int j = 0; j < ct; ++j)
                if (src[j]) dst[j >> 3] |= (uint8_t)(1u << (j & 7));
        }
    }
    return LRBI_OK;
}

extern "C" int lrbi_pack_factors(const lrbi_desc *desc, const uint8_t *hIp01, const uint8_t *hIz01,
                                 void *hIp_packed, void *hIz_packed)
{
    return pack_impl(desc, nullptr, hIp01, hIz01, hIp_packed, hIz_packed);
}

extern "C" int lrbi_pack_factors_ranked(const lrbi_desc *desc, const int32_t *hTileRank, const uint8_t *hIp01,
                                        const uint8_t *hIz01, void *hIp_packed, void *hIz_packed)
{
    if (!hTileRank) return LRBI_ERR_NULL;
    return pack_impl(desc, hTileRank, hIp01, hIz01, hIp_packed, hIz_packed);
}

extern "C" int lrbi_index_bits_ranked(const lrbi_desc *desc, const int32_t *hTileRank, uint64_t *lrbi_bits)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!hTileRank || !lrbi_bits) return LRBI_ERR_NULL;
    const Geom g = make_geom(desc);
    uint64_t bits = 0;
    for (int64_t ti = 0; ti < g.tile_rows; ++ti) {
        const uint64_t rt = (uint64_t)((g.m - ti * g.r < g.r) ? g.m - ti * g.r : g.r);
        for (int64_t tj = 0; tj < g.tile_cols; ++tj) {
            const uint64_t ct = (uint64_t)((g.n - tj * g.c < g.c) ? g.n - tj * g.c : g.c);
            const int32_t kt = hTileRank[ti * g.tile_cols + tj];
            if (kt < 0 || kt > g.k) return LRBI_ERR_RANK;
            bits += (uint64_t)kt * (rt + ct);
        }
    }
    *lrbi_bits = bits;
    return LRBI_OK;
}

extern "C" int lrbi_unpack_mask(const lrbi_desc *desc, const void *hMask, int64_t mask_pitch_bytes,
                                uint8_t *hM01)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!hMask || !hM01) return LRBI_ERR_NULL;
    if (mask_pitch_bytes < (desc->n + 7) / 8) return LRBI_ERR_PITCH;
    const uint8_t *src = (const uint8_t *)hMask;
    for (int64_t i = 0; i < desc->m; ++i) {
        const uint8_t *row = src + i * mask_pitch_bytes;
        uint8_t *out = hM01 + i * desc->n;
        for (int64_t j = 0; j < desc->n; ++j) out[j] = (uint8_t)((row[j >> 3] >> (j & 7)) & 1u);
    }
    return LRBI_OK;
}

extern "C" int lrbi_decode_mask(const lrbi_desc *desc, const void *dIp_packed, const void *dIz_packed,
                                void *dMask, int64_t mask_pitch_bytes, void *stream)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!dIp_packed || !dIz_packed || !dMask) return LRBI_ERR_NULL;
    if (!aligned_to(dIp_packed, 4) || !aligned_to(dIz_packed, 8) || !aligned_to(dMask, 16))
        return LRBI_ERR_ALIGN;
    if (mask_pitch_bytes % 16 != 0 || mask_pitch_bytes < (desc->n + 7) / 8) return LRBI_ERR_PITCH;
    const Geom g = make_geom(desc);
    return launch_decode(g, desc->flags, (const uint32_t *)dIp_packed, (const uint32_t *)dIz_packed, dMask,
                         mask_pitch_bytes, (hipStream_t)stream);
}

static int elem_size(lrbi_dtype dt)
{
    switch (dt) {
    case LRBI_F32: return 4;
    case LRBI_F16: return 2;
    case LRBI_BF16: return 2;
    default: return 0;
    }
}

// true when the matrix-core kernel serves this call
static bool use_mfma(const lrbi_desc *desc, lrbi_dtype dt, int64_t N)
{
    const uint32_t path = desc->flags & LRBI_FLAG_PATH_MASK;
    if (dt == LRBI_F32) return false;
    if (path == LRBI_FLAG_PATH_MFMA) return true;
    if (path == LRBI_FLAG_PATH_VALU) return false;
    // below five columns the product is a bandwidth-bound matrix-vector sweep; the row-streaming kernels take one and
    // four columns ahead of this choice, and for two or three columns of a large matrix the tile kernel's split over n
    // beats the sweep (HBM-cold 4096 x 9216: 34 against 83-95 us; 6000 x 3000 in 300 x 300 tiles: 26.5 against 37.3 us)
    return N > 4 || (N >= 2 && (int64_t)desc->m * desc->n >= ((int64_t)1 << 23)); // (level at 2048 x 2048, the sweep ahead at 1024 x 1024)
}

extern "C" int lrbi_masked_gemm_workspace_bytes(const lrbi_desc *desc, lrbi_dtype dtype, int64_t N,
                                                uint64_t *bytes)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!bytes) return LRBI_ERR_NULL;
    if (elem_size(dtype) == 0) return LRBI_ERR_DTYPE;
    if (N <= 0) return LRBI_ERR_SHAPE;
    if ((desc->flags & LRBI_FLAG_PATH_MASK) == LRBI_FLAG_PATH_MFMA && dtype == LRBI_F32) return LRBI_ERR_DTYPE;
    *bytes = 0;
    if (use_mfma(desc, dtype, N)) {
        const Geom g = make_geom(desc);
        *bytes = plan_mfma(g, desc->flags, N).workspace_bytes;
    }
    return LRBI_OK;
}

extern "C" int lrbi_masked_gemm(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                                const void *dIp_packed, const void *dIz_packed, const void *dX, int64_t ldx,
                                int64_t N, void *dY, int64_t ldy, void *dWorkspace, uint64_t workspace_bytes,
                                void *stream)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!dW || !dIp_packed || !dIz_packed || !dX || !dY) return LRBI_ERR_NULL;
    const int es = elem_size(dtype);
    if (es == 0) return LRBI_ERR_DTYPE;
    if (N <= 0 || N > (int64_t)0x7FFFFF00) return LRBI_ERR_SHAPE;
    if (ldw < desc->n || ldx < N || ldy < N) return LRBI_ERR_PITCH;
    if (!aligned_to(dIp_packed, 4) || !aligned_to(dIz_packed, 8)) return LRBI_ERR_ALIGN;
    if (!aligned_to(dW, (uintptr_t)es) || !aligned_to(dX, (uintptr_t)es) || !aligned_to(dY, (uintptr_t)es))
        return LRBI_ERR_ALIGN;
    if ((desc->flags & LRBI_FLAG_PATH_MASK) == LRBI_FLAG_PATH_MFMA && dtype == LRBI_F32) return LRBI_ERR_DTYPE;
    const Geom g = make_geom(desc);
    hipStream_t s = (hipStream_t)stream;
    {
        // narrow batches of the 16-bit types: W streamed once, whatever the tile shape
        const uint32_t path = desc->flags & LRBI_FLAG_PATH_MASK;
        if (path == LRBI_FLAG_PATH_AUTO || path == LRBI_FLAG_PATH_STREAM) {
            const int cus = (path == LRBI_FLAG_PATH_STREAM) ? 0 : compute_units_of(s); // forced: any number of rows
            if (stream_ok(g, dtype, dW, ldw, dX, ldx, N, cus))
                return launch_stream_gemm(g, dtype, dW, ldw, (const uint32_t *)dIp_packed, (const uint32_t *)dIz_packed,
                                          dX, N, dY, ldy, nullptr, 0, cus, s);
            if (path == LRBI_FLAG_PATH_STREAM) return (dtype == LRBI_F32) ? LRBI_ERR_DTYPE : LRBI_ERR_ALIGN;
        }
    }
    bool mfma = use_mfma(desc, dtype, N);
    if (mfma) {
        // the matrix-core kernel loads W in 16-byte pieces; anything else goes to the vector-ALU kernel
        const bool w_vec = aligned_to(dW, 16) && (ldw % 8 == 0) && (desc->n % 8 == 0);
        if (!w_vec) {
            if ((desc->flags & LRBI_FLAG_PATH_MASK) == LRBI_FLAG_PATH_MFMA) return LRBI_ERR_ALIGN;
            mfma = false;
        }
    }
    if (!mfma)
        return launch_valu_gemm(g, dtype, dW, ldw, (const uint32_t *)dIp_packed, (const uint32_t *)dIz_packed,
                                dX, ldx, N, dY, ldy, s);
    MfmaPlan plan = plan_mfma(g, desc->flags, N);
    if (plan.splitk > 1) {
        const bool ws_ok = dWorkspace && aligned_to(dWorkspace, 16) && workspace_bytes >= plan.workspace_bytes;
        if (!ws_ok) {
            if (desc->flags & LRBI_FLAG_SPLITK_MASK) return LRBI_ERR_WORKSPACE;
            // no scratch: fall back to one slice over the whole n range
            plan = plan_mfma(g, (desc->flags & ~LRBI_FLAG_SPLITK_MASK) | (1u << LRBI_FLAG_SPLITK_SHIFT), N);
        }
    }
    return launch_mfma_gemm(g, plan, dtype, dW, ldw, (const uint32_t *)dIp_packed, (const uint32_t *)dIz_packed,
                            dX, ldx, N, dY, ldy, dWorkspace, s);
}

extern "C" int lrbi_decode_and_gemm(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                                    const void *dIp_packed, const void *dIz_packed, const void *dX, int64_t ldx,
                                    int64_t N, void *dY, int64_t ldy, void *dMask, int64_t mask_pitch_bytes,
                                    void *dWorkspace, uint64_t workspace_bytes, void *stream)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!dW || !dIp_packed || !dIz_packed || !dX || !dY || !dMask) return LRBI_ERR_NULL;
    const int es = elem_size(dtype);
    if (es == 0) return LRBI_ERR_DTYPE;
    if (N <= 0 || N > (int64_t)0x7FFFFF00) return LRBI_ERR_SHAPE;
    if (ldw < desc->n || ldx < N || ldy < N) return LRBI_ERR_PITCH;
    if (mask_pitch_bytes % 16 != 0 || mask_pitch_bytes < (desc->n + 7) / 8) return LRBI_ERR_PITCH;
    if (!aligned_to(dIp_packed, 4) || !aligned_to(dIz_packed, 8) || !aligned_to(dMask, 16)) return LRBI_ERR_ALIGN;
    if (!aligned_to(dW, (uintptr_t)es) || !aligned_to(dX, (uintptr_t)es) || !aligned_to(dY, (uintptr_t)es))
        return LRBI_ERR_ALIGN;
    // Narrow batches on the row-streaming kernels (tried first, as in lrbi_masked_gemm): a workgroup rebuilds the
    // whole mask of its rows in LDS before its first product and stores it from there.
    {
        const uint32_t path = desc->flags & LRBI_FLAG_PATH_MASK;
        if (path == LRBI_FLAG_PATH_AUTO || path == LRBI_FLAG_PATH_STREAM) {
            const Geom g = make_geom(desc);
            const int cus = (path == LRBI_FLAG_PATH_STREAM) ? 0 : compute_units_of((hipStream_t)stream);
            if (stream_ok(g, dtype, dW, ldw, dX, ldx, N, cus))
                return launch_stream_gemm(g, dtype, dW, ldw, (const uint32_t *)dIp_packed, (const uint32_t *)dIz_packed,
                                          dX, N, dY, ldy, nullptr, 0, cus, (hipStream_t)stream,
                                          MaskOut{dMask, mask_pitch_bytes / 16});
            if (path == LRBI_FLAG_PATH_STREAM) return (dtype == LRBI_F32) ? LRBI_ERR_DTYPE : LRBI_ERR_ALIGN;
        }
    }
    // One launch when the pipelined or the generic tile kernel serves the product: they rebuild every mask word for
    // their own use and store it on the way (the workgroups of the first block of batch columns do).
    if (use_mfma(desc, dtype, N) && aligned_to(dW, 16) && ldw % 8 == 0 && desc->n % 8 == 0) {
        const Geom g = make_geom(desc);
        MfmaPlan plan = plan_mfma(g, desc->flags, N);
        if (plan.splitk > 1) {
            const bool ws_ok = dWorkspace && aligned_to(dWorkspace, 16) && workspace_bytes >= plan.workspace_bytes;
            if (!ws_ok) {
                if (desc->flags & LRBI_FLAG_SPLITK_MASK) return LRBI_ERR_WORKSPACE;
                plan = plan_mfma(g, (desc->flags & ~LRBI_FLAG_SPLITK_MASK) | (1u << LRBI_FLAG_SPLITK_SHIFT), N);
            }
        }
        if (mfma_gemm_emits_mask(g, plan, dW, ldw, dIz_packed, dX, ldx, N))
            return launch_mfma_gemm(g, plan, dtype, dW, ldw, (const uint32_t *)dIp_packed,
                                    (const uint32_t *)dIz_packed, dX, ldx, N, dY, ldy, dWorkspace, (hipStream_t)stream,
                                    MaskOut{dMask, mask_pitch_bytes / 16});
    }
    // every other shape: the two entry points one after the other on the same stream
    const int rc1 = lrbi_decode_mask(desc, dIp_packed, dIz_packed, dMask, mask_pitch_bytes, stream);
    if (rc1 != LRBI_OK) return rc1;
    return lrbi_masked_gemm(desc, dtype, dW, ldw, dIp_packed, dIz_packed, dX, ldx, N, dY, ldy, dWorkspace,
                            workspace_bytes, stream);
}

// plan of the convolution form: the pipelined tile kernel, whatever the tile flag says
static MfmaPlan plan_conv(const lrbi_desc *desc, int64_t N)
{
    const uint32_t flags = (desc->flags & ~LRBI_FLAG_TILE_MASK) | (14u << LRBI_FLAG_TILE_SHIFT);
    return plan_mfma(make_geom(desc), flags, N);
}

extern "C" int lrbi_masked_conv3x3_workspace_bytes(const lrbi_desc *desc, lrbi_dtype dtype, int64_t batch, int64_t H,
                                                   int64_t Wd, uint64_t *bytes)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!bytes) return LRBI_ERR_NULL;
    if (dtype != LRBI_F16 && dtype != LRBI_BF16) return LRBI_ERR_DTYPE;
    if (batch <= 0 || H <= 0 || Wd <= 0 || batch * H * Wd > (int64_t)0x7FFFFF00) return LRBI_ERR_SHAPE;
    *bytes = plan_conv(desc, batch * H * Wd).workspace_bytes;
    return LRBI_OK;
}

extern "C" int lrbi_masked_conv3x3(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                                   const void *dIp_packed, const void *dIz_packed, const void *dActPadded, int64_t batch,
                                   int64_t H, int64_t Wd, int64_t cin, void *dY, int64_t ldy, void *dWorkspace,
                                   uint64_t workspace_bytes, void *stream)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!dW || !dIp_packed || !dIz_packed || !dActPadded || !dY) return LRBI_ERR_NULL;
    if (dtype != LRBI_F16 && dtype != LRBI_BF16) return LRBI_ERR_DTYPE;
    if (batch <= 0 || H <= 0 || Wd <= 0 || cin <= 0 || H > 32766 || Wd > 32766 || cin > (1 << 20)) return LRBI_ERR_SHAPE;
    if (batch * H * Wd > (int64_t)0x7FFFFF00 || desc->n != 9 * cin) return LRBI_ERR_SHAPE;
    const int64_t N = batch * H * Wd;
    if (ldw < desc->n || ldy < N) return LRBI_ERR_PITCH;
    if (!aligned_to(dIp_packed, 4) || !aligned_to(dIz_packed, 16) || !aligned_to(dW, 16) || ldw % 8 != 0 ||
        !aligned_to(dActPadded, 16) || !aligned_to(dY, 2))
        return LRBI_ERR_ALIGN;
    const Geom g = make_geom(desc);
    const ConvGeom cg = {(int)cin, (int)H, (int)Wd};
    if (!pipe_conv_ok(g, cg, batch, dIz_packed, dActPadded, ldw)) return LRBI_ERR_SHAPE;
    MfmaPlan plan = plan_conv(desc, N);
    if (plan.splitk > 1) {
        const bool ws_ok = dWorkspace && aligned_to(dWorkspace, 16) && workspace_bytes >= plan.workspace_bytes;
        if (!ws_ok) {
            if (desc->flags & LRBI_FLAG_SPLITK_MASK) return LRBI_ERR_WORKSPACE;
            lrbi_desc one = *desc; // no scratch: one slice over the whole reduction range
            one.flags = (desc->flags & ~LRBI_FLAG_SPLITK_MASK) | (1u << LRBI_FLAG_SPLITK_SHIFT);
            plan = plan_conv(&one, N);
        }
    }
    return launch_mfma_conv(g, plan, dtype, cg, dW, ldw, (const uint32_t *)dIp_packed, (const uint32_t *)dIz_packed,
                            dActPadded, N, dY, ldy, dWorkspace, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------
// lrbi_masked_gemm_static: the fused masked product for callers that cannot allocate.  The partial sums of a
// split reduction live in `scratch`, a device array that is part of the library's code object: every GPU the
// library runs on holds its own copy from the moment the code object is loaded there until the process ends.
// In host code the array's name only stands for the symbol; its address on a device is asked of the runtime once
// per device (with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[LRBI_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex scratch_mu;
void *scratch_ptr[kMaxDevices]; // per device: address of that device's copy of `scratch`, nullptr until asked

// address of the current device's scratch array; nullptr when the runtime cannot tell
void *scratch_of_current_device()
{
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_ptr[device]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        scratch_ptr[device] = p;
    }
    return scratch_ptr[device];
}
} // namespace

extern "C" int lrbi_masked_gemm_static(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                                       const void *dIp_packed, const void *dIz_packed, const void *dX, int64_t ldx,
                                       int64_t N, void *dY, int64_t ldy, void *stream)
{
    uint64_t need = 0;
    const int rc = lrbi_masked_gemm_workspace_bytes(desc, dtype, N, &need);
    if (rc != LRBI_OK) return rc;
    if (need > (uint64_t)LRBI_STATIC_SCRATCH_BYTES) return LRBI_ERR_WORKSPACE;
    void *ws = nullptr;
    if (need) {
        ws = scratch_of_current_device();
        if (!ws) return LRBI_ERR_LAUNCH;
    }
    return lrbi_masked_gemm(desc, dtype, dW, ldw, dIp_packed, dIz_packed, dX, ldx, N, dY, ldy, ws,
                            ws ? (uint64_t)LRBI_STATIC_SCRATCH_BYTES : 0u, stream);
}

// Sec. 3.2: methods 1 .. 3; the amplification must be a positive finite number for method 3
static bool cost_manip_of(int32_t method, float amplify, CostManip *out)
{
    if (method < 1 || method > 3) return false;
    if (method == 3 && !(amplify > 0.f && amplify <= 3.0e38f)) return false;
    out->squared = method == 2;
    out->scale = method == 3 ? (double)amplify : 1.0;
    return true;
}

extern "C" int lrbi_threshold_eval(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                                   float w_threshold, int32_t method, float amplify, const float *dMp, const float *dMz, const float *dTp,
                                   const float *dTz, void *dIp_packed, void *dIz_packed, uint64_t *dKept,
                                   double *dCost, void *dWorkspace, uint64_t workspace_bytes, void *stream)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!dW || !dMp || !dMz || !dTp || !dTz || !dKept || !dCost) return LRBI_ERR_NULL;
    if ((dIp_packed == nullptr) != (dIz_packed == nullptr)) return LRBI_ERR_NULL;
    const int es = elem_size(dtype);
    if (es == 0) return LRBI_ERR_DTYPE;
    if (ldw < desc->n) return LRBI_ERR_PITCH;
    if (!aligned_to(dW, (uintptr_t)es) || !aligned_to(dMp, 4) || !aligned_to(dMz, 4) || !aligned_to(dTp, 4) ||
        !aligned_to(dTz, 4) || !aligned_to(dKept, 8) || !aligned_to(dCost, 8))
        return LRBI_ERR_ALIGN;
    if (dIp_packed && (!aligned_to(dIp_packed, 4) || !aligned_to(dIz_packed, 8))) return LRBI_ERR_ALIGN;
    CostManip manip;
    if (!cost_manip_of(method, amplify, &manip)) return LRBI_ERR_SHAPE;
    const Geom g = make_geom(desc);
    if (threshold_eval_lds_bytes(g) > 64 * 1024) return LRBI_ERR_SHAPE;
    const EvalPlan plan = plan_threshold_eval(g);
    const bool ws_ok = dWorkspace && aligned_to(dWorkspace, 8) && workspace_bytes >= plan.workspace_bytes;
    return launch_threshold_eval(g, dtype, dW, ldw, w_threshold, manip, dMp, dMz, dTp, dTz, dIp_packed, dIz_packed, dKept,
                                 dCost, (plan.bands > 1 && ws_ok) ? dWorkspace : nullptr, (hipStream_t)stream);
}

extern "C" int lrbi_threshold_eval_workspace_bytes(const lrbi_desc *desc, uint64_t *bytes)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!bytes) return LRBI_ERR_NULL;
    *bytes = plan_threshold_eval(make_geom(desc)).workspace_bytes;
    return LRBI_OK;
}

extern "C" int lrbi_search_thresholds(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                                      float w_threshold, int32_t method, float amplify, const float *dMp,
                                      const float *dMz, double target_sparsity,
                                      const double *sp_values, int32_t n_sp, int32_t steps, int64_t tolerance,
                                      float *dTp, float *dTz, uint64_t *dKept, double *dCost, void *dIp_packed,
                                      void *dIz_packed, void *dWorkspace, uint64_t workspace_bytes, void *stream)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!dW || !dMp || !dMz || !sp_values || !dTp || !dTz || !dKept || !dCost || !dWorkspace) return LRBI_ERR_NULL;
    if ((dIp_packed == nullptr) != (dIz_packed == nullptr)) return LRBI_ERR_NULL;
    const int es = elem_size(dtype);
    if (es == 0) return LRBI_ERR_DTYPE;
    if (ldw < desc->n) return LRBI_ERR_PITCH;
    if (n_sp < 1 || steps < 1 || tolerance < 0) return LRBI_ERR_SHAPE;
    CostManip manip;
    if (!cost_manip_of(method, amplify, &manip)) return LRBI_ERR_SHAPE;
    if (!(target_sparsity > 0.0 && target_sparsity < 1.0)) return LRBI_ERR_SHAPE;
    for (int32_t a = 0; a < n_sp; ++a)
        if (!(sp_values[a] >= 0.0 && sp_values[a] <= 1.0)) return LRBI_ERR_SHAPE;
    if (!aligned_to(dW, (uintptr_t)es) || !aligned_to(dMp, 4) || !aligned_to(dMz, 4) || !aligned_to(dTp, 4) ||
        !aligned_to(dTz, 4) || !aligned_to(dKept, 8) || !aligned_to(dCost, 8) || !aligned_to(dWorkspace, 16))
        return LRBI_ERR_ALIGN;
    if (dIp_packed && (!aligned_to(dIp_packed, 4) || !aligned_to(dIz_packed, 8))) return LRBI_ERR_ALIGN;
    const Geom g = make_geom(desc);
    if (threshold_eval_lds_bytes(g) > 64 * 1024) return LRBI_ERR_SHAPE;
    const SearchPlan plan = plan_search(g);
    if (workspace_bytes < plan.bytes) return LRBI_ERR_WORKSPACE;
    return launch_search(g, dtype, dW, ldw, w_threshold, manip, dMp, dMz, target_sparsity, n_sp, sp_values, steps, tolerance,
                         dTp, dTz, dKept, dCost, dIp_packed, dIz_packed, dWorkspace, (hipStream_t)stream);
}

extern "C" int lrbi_search_workspace_bytes(const lrbi_desc *desc, uint64_t *bytes)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!bytes) return LRBI_ERR_NULL;
    *bytes = plan_search(make_geom(desc)).bytes;
    return LRBI_OK;
}

// the matrix-core backward kernels load W (and write dW) in 16-byte pieces
static bool w_pieces_ok(const lrbi_desc *desc, const void *dW, int64_t ldw)
{
    return aligned_to(dW, 16) && (ldw % 8 == 0) && (desc->n % 8 == 0);
}

extern "C" int lrbi_masked_gemm_t_workspace_bytes(const lrbi_desc *desc, lrbi_dtype dtype, int64_t N, uint64_t *bytes)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!bytes) return LRBI_ERR_NULL;
    if (elem_size(dtype) == 0) return LRBI_ERR_DTYPE;
    if (N <= 0) return LRBI_ERR_SHAPE;
    *bytes = plan_gemm_t(make_geom(desc), dtype, N, desc->n % 8 == 0).workspace_bytes;
    return LRBI_OK;
}

extern "C" int lrbi_masked_gemm_t(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                                  const void *dIp_packed, const void *dIz_packed, const void *dDY, int64_t lddy,
                                  int64_t N, void *dDX, int64_t lddx, void *dWorkspace, uint64_t workspace_bytes,
                                  void *stream)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!dW || !dIp_packed || !dIz_packed || !dDY || !dDX) return LRBI_ERR_NULL;
    const int es = elem_size(dtype);
    if (es == 0) return LRBI_ERR_DTYPE;
    if (N <= 0 || N > (int64_t)0x7FFFFF00) return LRBI_ERR_SHAPE;
    if (ldw < desc->n || lddy < N || lddx < N) return LRBI_ERR_PITCH;
    if (!aligned_to(dIp_packed, 4) || !aligned_to(dIz_packed, 8)) return LRBI_ERR_ALIGN;
    if (!aligned_to(dW, (uintptr_t)es) || !aligned_to(dDY, (uintptr_t)es) || !aligned_to(dDX, (uintptr_t)es))
        return LRBI_ERR_ALIGN;
    const Geom g = make_geom(desc);
    // the matrix-core kernel addresses a slab of 64 rows with 32-bit byte offsets
    const bool small_pitch = ldw < ((int64_t)1 << 24) && lddy < ((int64_t)1 << 24);
    BwdPlan plan = plan_gemm_t(g, dtype, N, w_pieces_ok(desc, dW, ldw) && small_pitch);
    if (plan.slices > 1) {
        const bool ws_ok = dWorkspace && aligned_to(dWorkspace, 16) && workspace_bytes >= plan.workspace_bytes;
        if (!ws_ok) { // no scratch: one slice over all rows of W
            plan.slices = 1;
            plan.iper = g.m;
        }
    }
    return launch_gemm_t(g, plan, dtype, dW, ldw, (const uint32_t *)dIp_packed, (const uint32_t *)dIz_packed, dDY, lddy,
                         N, dDX, lddx, dWorkspace, (hipStream_t)stream);
}

extern "C" int lrbi_masked_grad(const lrbi_desc *desc, lrbi_dtype dtype, const void *dDY, int64_t lddy, const void *dX,
                                int64_t ldx, int64_t N, const void *dIp_packed, const void *dIz_packed, void *dDW,
                                int64_t lddw, void *stream)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!dDY || !dX || !dIp_packed || !dIz_packed || !dDW) return LRBI_ERR_NULL;
    const int es = elem_size(dtype);
    if (es == 0) return LRBI_ERR_DTYPE;
    if (N <= 0 || N > (int64_t)0x7FFFFF00) return LRBI_ERR_SHAPE;
    if (lddw < desc->n || lddy < N || ldx < N) return LRBI_ERR_PITCH;
    if (!aligned_to(dIp_packed, 4) || !aligned_to(dIz_packed, 8)) return LRBI_ERR_ALIGN;
    if (!aligned_to(dDW, (uintptr_t)es) || !aligned_to(dDY, (uintptr_t)es) || !aligned_to(dX, (uintptr_t)es))
        return LRBI_ERR_ALIGN;
    const Geom g = make_geom(desc);
    // matrix cores for the 16-bit types at any batch (below 8 columns the slab is mostly zero fill, and the tile kernel
    // still writes dW seven times faster than the vector-ALU kernel: 4096 x 9216 at one column 23 against 152 us); dW
    // rows need not be 16-byte aligned (the kernel then writes element by element)
    const bool mfma = dtype != LRBI_F32;
    return launch_grad(g, dtype, mfma, dDY, lddy, dX, ldx, N, (const uint32_t *)dIp_packed,
                       (const uint32_t *)dIz_packed, dDW, lddw, (hipStream_t)stream);
}

// plan of the gate product of an LSTM step: always the matrix-core kernels, planes left in the workspace
static MfmaPlan plan_lstm(const lrbi_desc *desc, int64_t B)
{
    MfmaPlan plan = plan_mfma(make_geom(desc), desc->flags, B);
    plan.planes_only = true;
    const uint64_t ldp = (uint64_t)((B + 3) / 4 * 4);
    plan.workspace_bytes = (uint64_t)plan.splitk * (uint64_t)desc->m * ldp * 4u;
    return plan;
}

extern "C" int lrbi_lstm_step_workspace_bytes(const lrbi_desc *desc, lrbi_dtype dtype, int64_t B, uint64_t *bytes)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!bytes) return LRBI_ERR_NULL;
    if (dtype != LRBI_F16 && dtype != LRBI_BF16) return LRBI_ERR_DTYPE;
    if (B <= 0 || desc->m % 4 != 0) return LRBI_ERR_SHAPE;
    *bytes = plan_lstm(desc, B).workspace_bytes;
    return LRBI_OK;
}

extern "C" int lrbi_lstm_step(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw,
                              const void *dIp_packed, const void *dIz_packed, const void *dXH, int64_t ldxh, int64_t B,
                              float *dC, int64_t ldc, void *dH1, int64_t ldh1, void *dH2, int64_t ldh2,
                              void *dWorkspace, uint64_t workspace_bytes, void *stream)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!dW || !dIp_packed || !dIz_packed || !dXH || !dC || !dH1 || !dWorkspace) return LRBI_ERR_NULL;
    if (dtype != LRBI_F16 && dtype != LRBI_BF16) return LRBI_ERR_DTYPE;
    if (B <= 0 || B > (int64_t)0x7FFFFF00 || desc->m % 4 != 0) return LRBI_ERR_SHAPE;
    if (ldw < desc->n || ldxh < B || ldc < B || ldh1 < B || (dH2 && ldh2 < B)) return LRBI_ERR_PITCH;
    if (!aligned_to(dIp_packed, 4) || !aligned_to(dIz_packed, 8)) return LRBI_ERR_ALIGN;
    if (!aligned_to(dW, 16) || ldw % 8 != 0 || desc->n % 8 != 0) return LRBI_ERR_ALIGN; // the matrix-core kernels' W loads
    if (!aligned_to(dXH, 2) || !aligned_to(dC, 4) || !aligned_to(dH1, 2) || !aligned_to(dH2, 2) ||
        !aligned_to(dWorkspace, 16))
        return LRBI_ERR_ALIGN;
    const Geom g = make_geom(desc);
    const MfmaPlan plan = plan_lstm(desc, B);
    if (workspace_bytes < plan.workspace_bytes) return LRBI_ERR_WORKSPACE;
    if ((desc->flags & LRBI_FLAG_PATH_MASK) == LRBI_FLAG_PATH_AUTO) {
        // narrow batches: the row-streaming kernel leaves the fp32 pre-activations as a single plane
        const int cus = compute_units_of((hipStream_t)stream);
        if (stream_ok(g, dtype, dW, ldw, dXH, ldxh, B, cus)) {
            // One kernel (product and cell equations) when h does not go into the buffer the product reads: there
            // other workgroups would still be reading what the first ones overwrite.
            const char *x0 = (const char *)dXH, *x1 = x0 + ((desc->n - 1) * ldxh + B) * 2;
            const int64_t Hh = desc->m / 4;
            auto overlaps_input = [&](const void *p, int64_t ld) {
                if (!p) return false;
                const char *h0 = (const char *)p, *h1 = h0 + ((Hh - 1) * ld + B) * 2;
                return h0 < x1 && x0 < h1;
            };
            if (B > 1 && !overlaps_input(dH1, ldh1) && !overlaps_input(dH2, ldh2)) {
                const int rcf = launch_stream_lstm(g, dtype, dW, ldw, (const uint32_t *)dIp_packed,
                                                   (const uint32_t *)dIz_packed, dXH, B, dC, ldc, dH1, ldh1, dH2, ldh2, cus,
                                                   (hipStream_t)stream);
                if (rcf != LRBI_ERR_SHAPE) return rcf; // done, or a launch error; LRBI_ERR_SHAPE: not served, go on
            }
            const int64_t ldp = (B + 3) / 4 * 4;
            const int rc1 = launch_stream_gemm(g, dtype, dW, ldw, (const uint32_t *)dIp_packed, (const uint32_t *)dIz_packed,
                                               dXH, B, nullptr, 0, (float *)dWorkspace, ldp, cus, (hipStream_t)stream);
            if (rc1 != LRBI_OK) return rc1;
            return launch_lstm_cell(dtype, (const float *)dWorkspace, 1, desc->m, ldp, B, dC, ldc, dH1, ldh1, dH2, ldh2,
                                    (hipStream_t)stream);
        }
    }
    const int rc2 = launch_mfma_gemm(g, plan, dtype, dW, ldw, (const uint32_t *)dIp_packed, (const uint32_t *)dIz_packed,
                                     dXH, ldxh, B, nullptr, 0, dWorkspace, (hipStream_t)stream);
    if (rc2 != LRBI_OK) return rc2;
    return launch_lstm_cell(dtype, (const float *)dWorkspace, plan.splitk, desc->m, (B + 3) / 4 * 4, B, dC, ldc, dH1, ldh1,
                            dH2, ldh2, (hipStream_t)stream);
}

extern "C" int lrbi_nmf_workspace_bytes(const lrbi_desc *desc, uint64_t *bytes)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!bytes) return LRBI_ERR_NULL;
    *bytes = nmf_workspace_bytes(make_geom(desc));
    return LRBI_OK;
}

extern "C" int lrbi_nmf(const lrbi_desc *desc, lrbi_dtype dtype, const void *dW, int64_t ldw, int32_t method,
                        float w_threshold, float amplify, float *dMp, float *dMz, int32_t iters, float eps,
                        void *dWorkspace, uint64_t workspace_bytes, void *stream)
{
    const int rc = validate_desc(desc);
    if (rc != LRBI_OK) return rc;
    if (!dW || !dMp || !dMz || !dWorkspace) return LRBI_ERR_NULL;
    const int es = elem_size(dtype);
    if (es == 0) return LRBI_ERR_DTYPE;
    if (method < 1 || method > 3 || iters < 0 || !(eps > 0.f)) return LRBI_ERR_SHAPE;
    if (ldw < desc->n) return LRBI_ERR_PITCH;
    if (!aligned_to(dW, (uintptr_t)es) || !aligned_to(dMp, 4) || !aligned_to(dMz, 4) || !aligned_to(dWorkspace, 16))
        return LRBI_ERR_ALIGN;
    const Geom g = make_geom(desc);
    if (workspace_bytes < nmf_workspace_bytes(g)) return LRBI_ERR_WORKSPACE;
    if (iters == 0) return LRBI_OK;
    return launch_nmf(g, dtype, dW, ldw, method, w_threshold, amplify, dMp, dMz, iters, eps, dWorkspace,
                      (hipStream_t)stream);
}
