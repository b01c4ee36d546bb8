// Fused masked product for narrow batches (N <= 32 columns of X, f16 / bf16): Y = (W o I_a) X with W streamed from
// HBM exactly once at the rate the memory delivers it.  Any tile shape: the mask words come from the general
// decode (Eq. 3), so tiles need not line up with anything.
//
// A workgroup of eight wavefronts owns BM (16 or 8) rows of one tile row of W and walks all n columns in slabs of
// KS (256 or 512) columns; BM * KS * 2 bytes = 8 KB of W per slab either way.
//   * First the mask of the workgroup's rows, all n columns of it, is rebuilt: the tile row's packed I_z and the
//     rows' I_p words are copied into LDS, then every lane decodes 32-bit mask words from there (Eq. 3; no dependent
//     global load per word) into an LDS array.  The first slabs of W are already on their way meanwhile.
//   * Slab loop: every wavefront copies its share of the slab NS - 1 slabs ahead -- one 1 KB piece of W (a row, or two
//     half rows) and up to two 1 KB pieces of the slab's 256 x N or 512 x N part of X -- from global memory straight
//     into an LDS ring of NS stages (load-to-LDS, 16 bytes per lane, no registers).  Many wavefronts with few
//     loads each is what the memory pipeline wants: measured on the box, a wavefront gets no more than about four
//     such loads to overlap, however many it has issued.  Every wavefront issues the same number of copy
//     instructions for every slab (addresses past the matrix are clamped, never skipped), so "my share of slab s has
//     landed" is a fixed bound on its count of outstanding loads, and one barrier per slab makes that true of the
//     whole slab and hands the oldest stage back.
//   * Arithmetic: 16x16x32 MFMAs, A = 16 rows x 32 columns of W read from LDS with the pruned weights zeroed by
//     select on the bit pattern, B = the matching 32 x 16 piece of X.  Wavefront w takes the slab's 32-column steps
//     w (and w + 8); the eight partial accumulators are added through LDS at the end, in wavefront order.
// X stays in its [k][N] order in LDS: for N = 1 an operand is 16 consecutive bytes of it, otherwise the transposing
// LDS read delivers 8 consecutive k of one column per lane (needs N % 4 == 0 for its 8-byte alignment).
//
// A single column over rows of at most 8192 columns takes the second kernel of this file instead (a row of W goes
// straight into the registers of its wavefront); the mask of the rows is rebuilt the same way in both.
#include <type_traits>

#include "lrbi_internal.hpp"
#include "lrbi_lds_dma.hpp"
#include "lrbi_mfma_common.hpp"

namespace lrbi {

static constexpr int ST_WAVES = 8;
static constexpr int ST_THREADS = ST_WAVES * 64;
static constexpr int ST_W_INSTR = 8;              // 1 KB copy instructions per W slab: one per wavefront
static constexpr int ST_WPIECE = 1024 + 16;       // LDS bytes per such piece (16 bytes of skew against bank conflicts)
static constexpr int ST_WSTAGE = ST_W_INSTR * ST_WPIECE;
static constexpr int ST_FP_ROWS = 16;             // I_p rows per tile held in LDS
// bytes of W per workgroup up to which a grid of fewer workgroups than half the compute units is still served: tile
// shapes that the panel kernels take, and every other shape (the generic tile kernel)
static constexpr int ST_LONE_ROWS_BYTES_PANEL = 64 * 1024, ST_LONE_ROWS_BYTES = 256 * 1024;
static constexpr int ST_FZ_MAX_BYTES = 40 * 1024; // packed I_z of one tile row that the kernel is willing to hold in LDS
static constexpr int ST_X_PAD = 64;               // the transposing read of the last k rows may run this far past the slab

typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ f32x4 mfma_16x16x32(F16Tag, u32x4 a, u32x4 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0,
                                                  0);
}
__device__ __forceinline__ f32x4 mfma_16x16x32(BF16Tag, u32x4 a, u32x4 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
}

// wait until at most n of this wavefront's loads are outstanding (n known only at run time; waiting for a few
// loads more than asked is harmless, so above 15 the count is rounded down to a multiple of four)
__device__ __forceinline__ void wait_loads_at_most(int n)
{
    switch (n < 16 ? n : 12 + (n >> 2)) {
    case 0: wait_loads<0>(); break;
    case 1: wait_loads<1>(); break;
    case 2: wait_loads<2>(); break;
    case 3: wait_loads<3>(); break;
    case 4: wait_loads<4>(); break;
    case 5: wait_loads<5>(); break;
    case 6: wait_loads<6>(); break;
    case 7: wait_loads<7>(); break;
    case 8: wait_loads<8>(); break;
    case 9: wait_loads<9>(); break;
    case 10: wait_loads<10>(); break;
    case 11: wait_loads<11>(); break;
    case 12: wait_loads<12>(); break;
    case 13: wait_loads<13>(); break;
    case 14: wait_loads<14>(); break;
    case 15: wait_loads<15>(); break;
    case 16: wait_loads<16>(); break; // 16 .. 19
    case 17: wait_loads<20>(); break;
    case 18: wait_loads<24>(); break;
    case 19: wait_loads<28>(); break;
    case 20: wait_loads<32>(); break;
    case 21: wait_loads<36>(); break;
    case 22: wait_loads<40>(); break;
    case 23: wait_loads<44>(); break;
    case 24: wait_loads<48>(); break;
    case 25: wait_loads<52>(); break;
    case 26: wait_loads<56>(); break;
    case 27: wait_loads<60>(); break;
    default: wait_loads<0>(); break;
    }
}

struct StreamArgs {
    const uint16_t *W;
    int64_t ldw;
    const uint32_t *Ip, *Iz;
    const uint16_t *X;
    int N;
    uint16_t *Y;   // storage-dtype output [m][ldy], or null
    int64_t ldy;
    float *P;      // fp32 output [m][ldp] (the pre-activations of a fused consumer), or null
    int64_t ldp;
    int x_instr;   // copy instructions per X slab
    int x_stage;   // LDS bytes per X stage
    uint32_t x_pieces; // 16-byte pieces of X in all
    int blocks_per_tile_row; // workgroups per tile row (BM rows each, the last one may be short)
    int fz_words;  // packed I_z words of one tile row
    int fz_pad;    // the same rounded up to whole copy instructions (64 words, or 64 16-byte pieces)
    int fz_vec;    // the tile rows' slices of I_z are 16-byte aligned whole numbers of 16-byte pieces
    int fp_pitch;  // LDS words per tile for the I_p words of 16 rows: 16 * ipw rounded up to whole copy instructions
    int ms_pitch;  // mask words per row in LDS (odd, at least 8 per slab)
    uint32_t *mask_out;   // not null: the rows' mask also goes to global memory, in the stand-alone decode's layout
    int64_t mask_pitch32; // 32-bit words per row of that mask
    int mask_words;       // words per row that the decode writes: whole 16-byte pieces up to column n
    uint32_t izw_magic; // floor(2^32 / izw) + 1: an index below 2^16 times this, upper 32 bits, is the index / izw
};


// The mask of a workgroup's rows, first half: the tile row's packed I_z and the rows' I_p words into LDS.
// Linear copies, spread evenly over the wavefronts (a wavefront's copies complete in order and only a few of
// them overlap, so the wavefront with the most of them sets the time): I_z in 16-byte pieces when its slices
// allow, else word by word; the I_p words of tile tj by wavefront tj % 8.
__device__ __forceinline__ void stage_row_factors(const Geom &g, const StreamArgs &a, uint32_t *Fz, uint32_t *Fp, int ti,
                                                  int il0, int rows_here, int wave, int lane)
{
    const uint32_t *zsrc = a.Iz + (int64_t)ti * g.tile_cols * g.k * (int64_t)g.izw;
    if (a.fz_vec) {
        const int pieces = a.fz_words >> 2;
        for (int p0 = wave * 64; p0 < pieces; p0 += ST_THREADS) {
            int p = p0 + lane;
            if (p >= pieces) p = pieces - 1; // the copy instruction's slots past the end are part of the pad
            load_to_lds16(lds_address(Fz + 4 * p0), zsrc, 16u * (uint32_t)p);
        }
    } else {
        for (int w0 = wave * 64; w0 < a.fz_words; w0 += ST_THREADS) {
            int w = w0 + lane;
            if (w >= a.fz_words) w = a.fz_words - 1;
            load_to_lds4(lds_address(Fz + w0), zsrc, 4u * (uint32_t)w);
        }
    }
    // per tile, the I_p rows il0 .. il0 + rows_here - 1 (slots past them are filled with the last row, never used)
    const int live = rows_here * g.ipw;
    for (int tj = wave; tj < g.tile_cols; tj += ST_WAVES) {
        const uint32_t *psrc = a.Ip + (((int64_t)ti * g.tile_cols + tj) * g.r + il0) * g.ipw;
        for (int e0 = 0; e0 < a.fp_pitch; e0 += 64) {
            int e = e0 + lane;
            if (e >= live) e = live - 1;
            load_to_lds4(lds_address(Fp + tj * a.fp_pitch + e0), psrc, 4u * (uint32_t)e);
        }
    }
}

// Second half: Eq. 3 from the factors in LDS.  Wavefront w takes rows w, w + 8, ...; its lanes take the (tile, 32-bit
// word of the tile's I_z rows) pairs of the row, 64 at a time.  An item ORs the word of every I_z row that its I_p row
// selects and then ORs the result into the row's mask (cleared by the caller) at the tile's bit position (two words
// when the tile does not start on a word boundary; neighbouring tiles may share a word, hence LDS atomics).  No item
// looks at more than one tile, so tile edges need no special cases.  The tile of an item is its index divided by
// izw: a multiplication by izw_magic = floor(2^32 / izw) + 1 (exact for the item counts that fit LDS; izw = 1 apart).
template <int BM>
__device__ __forceinline__ void decode_row_masks(const Geom &g, const StreamArgs &a, const uint32_t *Fz,
                                                 const uint32_t *Fp, uint32_t *Ms, int rows_here, int n, int wave,
                                                 int lane)
{
    const uint32_t items = (uint32_t)g.tile_cols * (uint32_t)g.izw;
    for (int rl = wave; rl < BM && rl < rows_here; rl += ST_WAVES) {
        for (uint32_t j = lane; j < items; j += 64) {
            const uint32_t tj = (g.izw == 1) ? j : __umulhi(j, a.izw_magic);
            const uint32_t wz = j - tj * (uint32_t)g.izw;
            const int in_tile = (int)wz * 32;
            const int col0 = (int)tj * g.c + in_tile;
            if (in_tile >= g.c || col0 >= n) continue;
            uint32_t v = 0u;
            const uint32_t *zcol = Fz + (size_t)tj * g.k * g.izw + wz; // this word of the tile's I_z rows
            for (int iw = 0; iw < g.ipw; ++iw) {
                uint32_t sel = Fp[tj * a.fp_pitch + rl * g.ipw + iw];
                // four selected rows per round, their reads independent of one another; when fewer are left the
                // last one is read again (an OR with the same word changes nothing)
                while (sel) {
                    const int l0 = __builtin_ctz(sel);
                    sel &= sel - 1u;
                    const int l1 = sel ? __builtin_ctz(sel) : l0;
                    sel &= sel - 1u;
                    const int l2 = sel ? __builtin_ctz(sel) : l1;
                    sel &= sel - 1u;
                    const int l3 = sel ? __builtin_ctz(sel) : l2;
                    sel &= sel - 1u;
                    const uint32_t z0 = zcol[(32 * iw + l0) * g.izw], z1 = zcol[(32 * iw + l1) * g.izw];
                    const uint32_t z2 = zcol[(32 * iw + l2) * g.izw], z3 = zcol[(32 * iw + l3) * g.izw];
                    v |= (z0 | z1) | (z2 | z3);
                }
            }
            // columns past the tile's width (pad bits of the packed rows) and past n (a cut-off last tile) stay out
            const int lim = (g.c - in_tile < n - col0) ? g.c - in_tile : n - col0;
            if (lim < 32) v &= (1u << lim) - 1u;
            if (v == 0u) continue;
            uint32_t *dst = Ms + rl * a.ms_pitch + (col0 >> 5);
            const int sh = col0 & 31;
            __hip_atomic_fetch_or(dst, v << sh, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (sh && (v >> (32 - sh)))
                __hip_atomic_fetch_or(dst + 1, v >> (32 - sh), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
}

// The rows' mask as the stand-alone decode leaves it in global memory (one bit per weight, pad bits zero): the
// workgroup has just rebuilt exactly these words in LDS.  Call behind the barrier that publishes them.
__device__ __forceinline__ void store_row_masks(const StreamArgs &a, const uint32_t *Ms, int64_t m0, int rows_here, int tid)
{
    if (!a.mask_out) return;
    for (int i = tid; i < rows_here * a.mask_words; i += ST_THREADS) {
        const int row = i / a.mask_words, w = i - row * a.mask_words;
        a.mask_out[(m0 + row) * a.mask_pitch32 + w] = Ms[row * a.ms_pitch + w];
    }
}

template <typename Tag, int NS, int BM, int KS>
__global__ __launch_bounds__(ST_THREADS) void stream_gemm_kernel(Geom g, StreamArgs a)
{
    static_assert(BM * KS * 2 == ST_W_INSTR * 1024, "a W slab is eight 1 KB pieces");
    constexpr int ROWS_PER_PIECE = 1024 / (KS * 2); // 2 half rows (KS = 256) or 1 row (KS = 512)
    constexpr int STEPS = KS / 32;                  // MFMA steps per slab: 8 or 16
    extern __shared__ uint4 lrbi_dyn_smem[];
    unsigned char *smem = (unsigned char *)lrbi_dyn_smem;
    unsigned char *Wst = smem;                                  // [NS][ST_WSTAGE]
    unsigned char *Xst = smem + NS * ST_WSTAGE;                  // [NS][x_stage]
    uint32_t *Ms = (uint32_t *)(Xst + (size_t)NS * a.x_stage);   // [BM][ms_pitch]: the rows' whole mask
    uint32_t *Fz = Ms + BM * a.ms_pitch;                         // [tile_cols][k][izw]
    uint32_t *Fp = Fz + a.fz_pad;                                // [tile_cols][fp_pitch]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ti = blockIdx.x / a.blocks_per_tile_row;           // tile row
    const int il0 = (blockIdx.x - ti * a.blocks_per_tile_row) * BM; // first row within the tile
    const int64_t m0 = (int64_t)ti * g.r + il0;
    // rows of this workgroup: at most BM, cut at the end of the tile and of the matrix
    int rows_here = BM;
    if (g.r - il0 < rows_here) rows_here = g.r - il0;
    if (g.m - m0 < rows_here) rows_here = (int)(g.m - m0);
    if (rows_here <= 0) return; // a tile row cut off by the end of the matrix: the whole workgroup leaves
    const int n = (int)g.n;
    const int N = a.N;
    const int nslabs = (n + KS - 1) / KS;

    // ---- this wavefront's share of a slab's copies ----
    const uint16_t *wbase = a.W + m0 * a.ldw; // uniform; lanes add 32-bit byte offsets
    // piece `wave` of the W slab: KS = 512: row `wave`; KS = 256: rows 2 wave (lanes 0-31) and 2 wave + 1 (lanes 32-63).
    // Past the last row or column the address is clamped, never skipped: such values meet a zero mask bit or land
    // in rows that are never stored.
    int my_row = wave * ROWS_PER_PIECE + (ROWS_PER_PIECE == 2 ? (lane >> 5) : 0);
    if (my_row >= rows_here) my_row = rows_here - 1;
    const int my_col = 8 * (ROWS_PER_PIECE == 2 ? (lane & 31) : lane);
    const int my_x_instr = (a.x_instr > wave ? 1 : 0) + (a.x_instr > wave + ST_WAVES ? 1 : 0);
    const int my_per_slab = 1 + my_x_instr; // copy instructions of this wavefront per slab
    auto copy_slab = [&](int slab) {
        const int stage = slab % NS;
        const int k0 = slab * KS;
        int col = k0 + my_col;
        if (col > n - 8) col = n - 8;
        load_to_lds16(lds_address(Wst + stage * ST_WSTAGE + wave * ST_WPIECE), wbase,
                      (uint32_t)(((int64_t)my_row * a.ldw + col) * 2));
        const uint32_t x_lds = lds_address(Xst + (size_t)stage * a.x_stage);
        const uint32_t first = (uint32_t)(((int64_t)k0 * N * 2) >> 4); // 16-byte piece of X the slab starts at
        for (int i = wave; i < a.x_instr; i += ST_WAVES) {
            uint32_t piece = first + 64u * i + lane;
            if (piece >= a.x_pieces) piece = a.x_pieces - 1u; // stays inside X; meets zeroed weights only
            load_to_lds16(x_lds + 1024u * i, a.X, piece * 16u);
        }
    };

    // ---- the mask of the workgroup's rows ----
    auto stage_factors = [&]() { stage_row_factors(g, a, Fz, Fp, ti, il0, rows_here, wave, lane); };
    auto decode_rows = [&]() { decode_row_masks<BM>(g, a, Fz, Fp, Ms, rows_here, n, wave, lane); };

    // ---- arithmetic ----
    const int row16 = lane & 15, kg = lane >> 4; // operand row / column, and which 8 of a step's 32 reduction indices
    const int arow = row16 & (BM - 1);           // BM = 8: rows 8-15 of the operand repeat rows 0-7 and are dropped
    f32x4 acc[2];
    acc[0] = f32x4{0.f, 0.f, 0.f, 0.f};
    acc[1] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int nblocks = (N > 16) ? 2 : 1; // 16-column blocks of Y

    auto multiply_slab = [&](int slab) {
        const int stage = slab % NS;
        const unsigned char *ws = Wst + stage * ST_WSTAGE + (arow / ROWS_PER_PIECE) * ST_WPIECE +
                                  (arow % ROWS_PER_PIECE) * (KS * 2);
        const unsigned char *xs = Xst + (size_t)stage * a.x_stage;
        const unsigned char *mb = (const unsigned char *)(Ms + arow * a.ms_pitch + slab * STEPS);
#pragma unroll
        for (int h = 0; h < STEPS / ST_WAVES; ++h) {
            const int step = wave + ST_WAVES * h;    // 32 columns of the slab
            const int kk = step * 32 + 8 * kg;       // this lane's 8 reduction indices
            const u32x4 wf = *reinterpret_cast<const u32x4 *>(ws + kk * 2);
            const u32x4 am = apply_mask8(wf, mb[step * 4 + kg]);
            if (N == 1) {
                const u32x4 xf = *reinterpret_cast<const u32x4 *>(xs + kk * 2); // every column of the block sees x
                acc[0] = mfma_16x16x32(Tag{}, am, xf, acc[0]);
            } else {
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) { // static indices: the accumulators must stay in registers
                    if (cb >= nblocks) break;
                    // lane s of a 16-lane group addresses row s / 4 (then + 4), columns 4 (s % 4) .. + 3 of the block
                    const unsigned char *p = xs + ((size_t)(kk + (row16 >> 2)) * N + cb * 16 + 4 * (row16 & 3)) * 2;
                    const u32x2 lo = lds_read_tr16_v((const uint16_t *)p);
                    const u32x2 hi = lds_read_tr16_v((const uint16_t *)(p + (size_t)4 * N * 2));
                    const u32x4 xf = {lo.x, lo.y, hi.x, hi.y};
                    acc[cb] = mfma_16x16x32(Tag{}, am, xf, acc[cb]);
                }
            }
        }
    };

#define LRBI_BARRIER()                                      \
    do {                                                    \
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  \
        __builtin_amdgcn_s_barrier();                       \
        asm volatile("" ::: "memory");                      \
    } while (0)

    // The factor copies go first and are waited for by count: the slab copies issued after them stay in flight.
    stage_factors();
    // Only the first two slabs are asked for behind the factor copies, the rest of the ring once the factors are in:
    // a compute unit serves its requests in order, and a second workgroup's factor copies would otherwise queue
    // behind the first one's whole ring.  (Slabs past the end copy clamped addresses: same count.)
    constexpr int EARLY = NS - 1 < 2 ? NS - 1 : 2;
    for (int s = 0; s < EARLY; ++s) copy_slab(s);
    for (int i = tid; i < BM * a.ms_pitch; i += ST_THREADS) Ms[i] = 0u;
    wait_loads_at_most(EARLY * my_per_slab);
    LRBI_BARRIER();
    for (int s = EARLY; s < NS - 1; ++s) copy_slab(s);
    decode_rows();
    for (int s = 0; s < nslabs; ++s) {
        wait_loads_at_most((NS - 2) * my_per_slab); // my share of slab s is in; slabs s + 1 .. s + NS - 2 may be on their way
        LRBI_BARRIER(); // the first one also publishes the mask words
        copy_slab(s + NS - 1); // into the stage of slab s - 1, which every wavefront has left
        multiply_slab(s);
    }
    wait_loads<0>(); // nothing may still be landing when the stages are reused below
    store_row_masks(a, Ms, m0, rows_here, tid); // (behind the loop: a store inside it would enter the counted waits)
    LRBI_BARRIER();

    // wavefronts' partial accumulators -> LDS; lane holds rows 4 kg + v, column row16 of each 16 x 16 block
    float *red = (float *)smem; // [8][2][16][16]
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[((wave * 2 + cb) * 16 + 4 * kg + v) * 16 + row16] = acc[cb][v];
    LRBI_BARRIER();
#undef LRBI_BARRIER
    for (int e = tid; e < 16 * 16 * nblocks; e += ST_THREADS) {
        const int cb = e >> 8, rr = (e >> 4) & 15, cc = e & 15;
        const int col = cb * 16 + cc;
        const int64_t row = m0 + rr;
        if (col >= N || rr >= rows_here) continue;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < ST_WAVES; ++w) v += red[((w * 2 + cb) * 16 + rr) * 16 + cc];
        if (a.P) a.P[row * a.ldp + col] = v;
        if (a.Y) a.Y[row * a.ldy + col] = cvt_store(Tag{}, v);
    }
}


// ---------------------------------------------------------------------------
// One column (N = 1), rows of at most 8192 columns: W goes from global memory straight into registers
// ---------------------------------------------------------------------------
// A workgroup of eight wavefronts owns eight rows of one tile row, one row per wavefront.  Every wavefront asks for
// its whole row at once (P loads of 1 KB, 16 bytes per lane), behind the copies of the factors and of x into LDS, so
// the whole matrix is requested within the first microsecond and the mask of the rows is rebuilt (as above) while W
// is on its way; no stage ring, no barrier per slab.  Then per row: select by mask byte, 2-element dot products in
// fp32 against x from LDS, a butterfly sum over the lanes.
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_acc(F16Tag, uint32_t w, uint32_t x, float c)
{
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w), __builtin_bit_cast(f16x2, x), c, false);
}
__device__ __forceinline__ float dot2_acc(BF16Tag, uint32_t w, uint32_t x, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, x), c, false);
}

// Sum over the 64 lanes, valid in lane 63: butterflies inside the groups of four, mirrored halves and rows of 16 (after
// which every lane of a row holds the row's sum), then row 0's sum into row 1 and row 2's into row 3, then row 1's
// into rows 2 and 3.  Cross-lane operands of the vector ALU, no LDS traffic; the order of the additions is fixed.
__device__ __forceinline__ float wave_sum_to_last_lane(float v)
{
    auto from = [](float x, auto ctrl, auto rows) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value,
                                                                     decltype(rows)::value, 0xF, false));
    };
    using std::integral_constant;
    v += from(v, integral_constant<int, 0xB1>{}, integral_constant<int, 0xF>{});  // quad_perm [1,0,3,2]
    v += from(v, integral_constant<int, 0x4E>{}, integral_constant<int, 0xF>{});  // quad_perm [2,3,0,1]
    v += from(v, integral_constant<int, 0x141>{}, integral_constant<int, 0xF>{}); // row_half_mirror
    v += from(v, integral_constant<int, 0x140>{}, integral_constant<int, 0xF>{}); // row_mirror
    v += from(v, integral_constant<int, 0x142>{}, integral_constant<int, 0xA>{}); // row_bcast15 into rows 1 and 3
    v += from(v, integral_constant<int, 0x143>{}, integral_constant<int, 0xC>{}); // row_bcast31 into rows 2 and 3
    return v;
}

static constexpr int RV_ROWS = 8;      // rows per workgroup: one per wavefront
static constexpr int RV_MAX_PIECES = 16; // 1 KB pieces of a row held in registers: rows of up to 8192 columns

template <typename Tag, int P>
__global__ __launch_bounds__(ST_THREADS) void rowvec_gemm_kernel(Geom g, StreamArgs a)
{
    static_assert(RV_ROWS == ST_WAVES && P <= RV_MAX_PIECES, "one row per wavefront");
    extern __shared__ uint4 lrbi_dyn_smem[];
    unsigned char *smem = (unsigned char *)lrbi_dyn_smem;
    unsigned char *Xs = smem;                               // x: P KB, column j at byte 2 j
    uint32_t *Ms = (uint32_t *)(smem + P * 1024);           // [8][ms_pitch]: the rows' whole mask
    uint32_t *Fz = Ms + RV_ROWS * a.ms_pitch;               // [tile_cols][k][izw]
    uint32_t *Fp = Fz + a.fz_pad;                           // [tile_cols][fp_pitch]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ti = blockIdx.x / a.blocks_per_tile_row;
    const int il0 = (blockIdx.x - ti * a.blocks_per_tile_row) * RV_ROWS;
    const int64_t m0 = (int64_t)ti * g.r + il0;
    int rows_here = RV_ROWS;
    if (g.r - il0 < rows_here) rows_here = g.r - il0;
    if (g.m - m0 < rows_here) rows_here = (int)(g.m - m0);
    if (rows_here <= 0) return; // a tile row cut off by the end of the matrix: the whole workgroup leaves
    const int n = (int)g.n;

    // copies into LDS first: the loads of W below are then the youngest of the wavefront, and "at most P loads
    // outstanding" means that every copy has landed
    stage_row_factors(g, a, Fz, Fp, ti, il0, rows_here, wave, lane);
    for (int i = wave; i < P; i += ST_WAVES) {
        uint32_t piece = 64u * i + lane;
        if (piece >= a.x_pieces) piece = a.x_pieces - 1u; // stays inside x; such columns are cleared below
        load_to_lds16(lds_address(Xs + 1024 * i), a.X, piece * 16u);
    }
    // this wavefront's row (a wavefront past the last row repeats that row and stores nothing); columns past n - 8
    // read the row's last piece instead: their mask bits are zero
    const int my_row = wave < rows_here ? wave : rows_here - 1;
    const char *wrow = (const char *)(a.W + (m0 + my_row) * a.ldw);
    // The first half of the row is asked for now, the second half once the mask is there: a wavefront cannot issue
    // further loads while the memory pipeline is full, and it must get to the mask rebuild while W streams in.
    constexpr int H = P / 2;
    u32x4 w[P];
    auto load_piece = [&](int p) {
        int col = p * 512 + lane * 8;
        if (col > n - 8) col = n - 8;
        return *reinterpret_cast<const u32x4 *>(wrow + (size_t)col * 2);
    };
#pragma unroll
    for (int p = 0; p < H; ++p) w[p] = load_piece(p);
    for (int i = tid; i < RV_ROWS * a.ms_pitch; i += ST_THREADS) Ms[i] = 0u;
    wait_loads<H>();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    decode_row_masks<RV_ROWS>(g, a, Fz, Fp, Ms, rows_here, n, wave, lane);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int p = H; p < P; ++p) w[p] = load_piece(p);
    store_row_masks(a, Ms, m0, rows_here, tid);

    const unsigned char *mb = (const unsigned char *)(Ms + my_row * a.ms_pitch);
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f; // four chains, added in a fixed order
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const u32x4 am = apply_mask8(w[p], mb[p * 64 + lane]);
        u32x4 xv = *reinterpret_cast<const u32x4 *>(Xs + p * 1024 + lane * 16);
        if (p * 512 + lane * 8 >= n) xv = u32x4{0u, 0u, 0u, 0u};
        a0 = dot2_acc(Tag{}, am.x, xv.x, a0);
        a1 = dot2_acc(Tag{}, am.y, xv.y, a1);
        a2 = dot2_acc(Tag{}, am.z, xv.z, a2);
        a3 = dot2_acc(Tag{}, am.w, xv.w, a3);
    }
    const float acc = wave_sum_to_last_lane((a0 + a1) + (a2 + a3));
    if (lane == 63 && wave < rows_here) {
        const int64_t row = m0 + wave;
        if (a.P) a.P[row * a.ldp] = acc;
        if (a.Y) a.Y[row * a.ldy] = cvt_store(Tag{}, acc);
    }
}

// ---------------------------------------------------------------------------
// LSTM step in one kernel: gate product and cell equations
// ---------------------------------------------------------------------------
// The ring kernel above with another choice of rows: a workgroup owns four hidden units j0 .. j0 + 3 and, of W's four
// row blocks [i; f; g; o] of H rows each, the rows of exactly these units (operand row 4 gate + unit: W row
// gate * H + j0 + unit), so that after the sum over the wavefronts it holds all four pre-activations of its units and
// applies the cell equations itself (the same arithmetic as lstm_cell_kernel): no plane of pre-activations, no second
// launch.  The four groups of rows lie in four tile rows: each one's packed I_z is copied into LDS (four copies of
// what the ring kernel stages), the rows' I_p words are gathered with one address per lane, and the rows' mask is
// rebuilt as above.  Needs H % 4 == 0 and r % 4 == 0 (the four rows of a gate then lie in one tile), and h outputs
// that do not alias the input: other workgroups still read it.
struct LstmFuse {
    int64_t H;
    float *C;
    int64_t ldc;
    uint16_t *H1;
    int64_t ldh1;
    uint16_t *H2;
    int64_t ldh2;
    int fp_words; // I_p words per tile column in LDS: 16 rows x ipw
    int fp_instr; // copy instructions for all of them
};

__device__ __forceinline__ float lstm_sigm(float z) { return 1.f / (1.f + expf(-z)); }

template <typename Tag, int NS>
__global__ __launch_bounds__(ST_THREADS) void stream_lstm_kernel(Geom g, StreamArgs a, LstmFuse f)
{
    constexpr int BM = 16, KS = 256;
    constexpr int ROWS_PER_PIECE = 2;
    constexpr int STEPS = KS / 32;
    extern __shared__ uint4 lrbi_dyn_smem[];
    unsigned char *smem = (unsigned char *)lrbi_dyn_smem;
    unsigned char *Wst = smem;                                  // [NS][ST_WSTAGE]
    unsigned char *Xst = smem + NS * ST_WSTAGE;                  // [NS][x_stage]
    uint32_t *Ms = (uint32_t *)(Xst + (size_t)NS * a.x_stage);   // [16][ms_pitch]: the rows' whole mask
    uint32_t *Fz = Ms + BM * a.ms_pitch;                         // [4 gates][fz_pad]: [tile_cols][k][izw] each
    uint32_t *Fp = Fz + 4 * a.fz_pad;                            // [tile_cols][16 rows][ipw]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t j0 = (int64_t)blockIdx.x * 4;
    const int units_here = (int)((f.H - j0 < 4) ? f.H - j0 : 4); // (H % 4 == 0: always 4; kept for safety)
    const int n = (int)g.n;
    const int N = a.N;
    const int nslabs = (n + KS - 1) / KS;

    // operand row rr = 4 gate + unit -> row of W, its tile row and its row inside the tile
    auto w_row = [&](int rr) -> int64_t {
        const int gate = rr >> 2;
        int unit = rr & 3;
        if (unit >= units_here) unit = units_here - 1; // repeats a row; its results are dropped
        return (int64_t)gate * f.H + j0 + unit;
    };

    // ---- this wavefront's share of a slab's copies: piece `wave` of the W slab = operand rows 2 wave (lanes 0-31)
    // and 2 wave + 1 (lanes 32-63), 512 bytes each; columns past n - 8 are clamped (they meet zero mask bits)
    const uint32_t my_wrow_off = (uint32_t)(w_row(wave * ROWS_PER_PIECE + (lane >> 5)) * a.ldw * 2); // below 2^32: host
    const int my_col = 8 * (lane & 31);
    const int my_x_instr = (a.x_instr > wave ? 1 : 0) + (a.x_instr > wave + ST_WAVES ? 1 : 0);
    const int my_per_slab = 1 + my_x_instr;
    auto copy_slab = [&](int slab) {
        const int stage = slab % NS;
        const int k0 = slab * KS;
        int col = k0 + my_col;
        if (col > n - 8) col = n - 8;
        load_to_lds16(lds_address(Wst + stage * ST_WSTAGE + wave * ST_WPIECE), a.W, my_wrow_off + (uint32_t)col * 2u);
        const uint32_t x_lds = lds_address(Xst + (size_t)stage * a.x_stage);
        const uint32_t first = (uint32_t)(((int64_t)k0 * N * 2) >> 4);
        for (int i = wave; i < a.x_instr; i += ST_WAVES) {
            uint32_t piece = first + 64u * i + lane;
            if (piece >= a.x_pieces) piece = a.x_pieces - 1u;
            load_to_lds16(x_lds + 1024u * i, a.X, piece * 16u);
        }
    };

    // ---- factor copies: per gate the packed I_z of its tile row (as the ring kernel's, spread over the wavefronts),
    // then the I_p words: entry e = (tile column, operand row, word), one per lane and copy instruction
    auto stage_factors = [&]() {
        // (the copy instructions of the four gates in one list, dealt round the wavefronts: the wavefront with the
        // most copies sets the time)
        const int per_instr = a.fz_vec ? 256 : 64; // words per copy instruction
        const int instr_per_gate = (a.fz_words + per_instr - 1) / per_instr;
        for (int q = wave; q < 4 * instr_per_gate; q += ST_WAVES) {
            const int gate = q / instr_per_gate, chunk = q - gate * instr_per_gate;
            const int ti = (int)(w_row(4 * gate) / g.r);
            const uint32_t *zsrc = a.Iz + (int64_t)ti * g.tile_cols * g.k * (int64_t)g.izw;
            uint32_t *dst = Fz + gate * a.fz_pad + chunk * per_instr;
            if (a.fz_vec) {
                const int pieces = a.fz_words >> 2;
                int p = chunk * 64 + lane;
                if (p >= pieces) p = pieces - 1;
                load_to_lds16(lds_address(dst), zsrc, 16u * (uint32_t)p);
            } else {
                int w = chunk * 64 + lane;
                if (w >= a.fz_words) w = a.fz_words - 1;
                load_to_lds4(lds_address(dst), zsrc, 4u * (uint32_t)w);
            }
        }
        const int entries = g.tile_cols * f.fp_words;
        for (int i = wave; i < f.fp_instr; i += ST_WAVES) {
            int e = i * 64 + lane;
            if (e >= entries) e = entries - 1;
            const int tj = e / f.fp_words, rem = e - tj * f.fp_words;
            const int rr = rem / g.ipw, iw = rem - rr * g.ipw;
            const int64_t row = w_row(rr);
            const int ti = (int)(row / g.r);
            const int il = (int)(row - (int64_t)ti * g.r);
            const int64_t word = ((((int64_t)ti * g.tile_cols + tj) * g.r) + il) * g.ipw + iw; // below 2^30: host
            load_to_lds4(lds_address(Fp + i * 64), a.Ip, (uint32_t)word * 4u);
        }
    };
    // Eq. 3 from the factors in LDS: wavefront w takes operand rows w and w + 8, its lanes the (tile, word) pairs
    auto decode_rows = [&]() {
        const uint32_t items = (uint32_t)g.tile_cols * (uint32_t)g.izw;
        for (int rl = wave; rl < BM; rl += ST_WAVES) {
            if ((rl & 3) >= units_here) continue;
            const uint32_t *fz = Fz + (rl >> 2) * a.fz_pad;
            for (uint32_t j = lane; j < items; j += 64) {
                const uint32_t tj = (g.izw == 1) ? j : __umulhi(j, a.izw_magic);
                const uint32_t wz = j - tj * (uint32_t)g.izw;
                const int in_tile = (int)wz * 32;
                const int col0 = (int)tj * g.c + in_tile;
                if (in_tile >= g.c || col0 >= n) continue;
                uint32_t v = 0u;
                const uint32_t *zcol = fz + (size_t)tj * g.k * g.izw + wz;
                for (int iw = 0; iw < g.ipw; ++iw) {
                    uint32_t sel = Fp[tj * f.fp_words + rl * g.ipw + iw];
                    while (sel) {
                        const int l0 = __builtin_ctz(sel);
                        sel &= sel - 1u;
                        const int l1 = sel ? __builtin_ctz(sel) : l0;
                        sel &= sel - 1u;
                        const int l2 = sel ? __builtin_ctz(sel) : l1;
                        sel &= sel - 1u;
                        const int l3 = sel ? __builtin_ctz(sel) : l2;
                        sel &= sel - 1u;
                        const uint32_t z0 = zcol[(32 * iw + l0) * g.izw], z1 = zcol[(32 * iw + l1) * g.izw];
                        const uint32_t z2 = zcol[(32 * iw + l2) * g.izw], z3 = zcol[(32 * iw + l3) * g.izw];
                        v |= (z0 | z1) | (z2 | z3);
                    }
                }
                const int lim = (g.c - in_tile < n - col0) ? g.c - in_tile : n - col0;
                if (lim < 32) v &= (1u << lim) - 1u;
                if (v == 0u) continue;
                uint32_t *dst = Ms + rl * a.ms_pitch + (col0 >> 5);
                const int sh = col0 & 31;
                __hip_atomic_fetch_or(dst, v << sh, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                if (sh && (v >> (32 - sh)))
                    __hip_atomic_fetch_or(dst + 1, v >> (32 - sh), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
    };

    // ---- arithmetic: as the ring kernel's
    const int row16 = lane & 15, kg = lane >> 4;
    f32x4 acc[2];
    acc[0] = f32x4{0.f, 0.f, 0.f, 0.f};
    acc[1] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int nblocks = (N > 16) ? 2 : 1;
    auto multiply_slab = [&](int slab) {
        const int stage = slab % NS;
        const unsigned char *ws = Wst + stage * ST_WSTAGE + (row16 / ROWS_PER_PIECE) * ST_WPIECE +
                                  (row16 % ROWS_PER_PIECE) * (KS * 2);
        const unsigned char *xs = Xst + (size_t)stage * a.x_stage;
        const unsigned char *mb = (const unsigned char *)(Ms + row16 * a.ms_pitch + slab * STEPS);
        const int step = wave;
        const int kk = step * 32 + 8 * kg;
        const u32x4 wf = *reinterpret_cast<const u32x4 *>(ws + kk * 2);
        const u32x4 am = apply_mask8(wf, mb[step * 4 + kg]);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            if (cb >= nblocks) break;
            const unsigned char *p = xs + ((size_t)(kk + (row16 >> 2)) * N + cb * 16 + 4 * (row16 & 3)) * 2;
            const u32x2 lo = lds_read_tr16_v((const uint16_t *)p);
            const u32x2 hi = lds_read_tr16_v((const uint16_t *)(p + (size_t)4 * N * 2));
            const u32x4 xf = {lo.x, lo.y, hi.x, hi.y};
            acc[cb] = mfma_16x16x32(Tag{}, am, xf, acc[cb]);
        }
    };

#define LRBI_BARRIER()                                      \
    do {                                                    \
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  \
        __builtin_amdgcn_s_barrier();                       \
        asm volatile("" ::: "memory");                      \
    } while (0)

    stage_factors();
    constexpr int EARLY = NS - 1 < 2 ? NS - 1 : 2;
    for (int s = 0; s < EARLY; ++s) copy_slab(s);
    for (int i = tid; i < BM * a.ms_pitch; i += ST_THREADS) Ms[i] = 0u;
    wait_loads_at_most(EARLY * my_per_slab);
    LRBI_BARRIER();
    for (int s = EARLY; s < NS - 1; ++s) copy_slab(s);
    decode_rows();
    for (int s = 0; s < nslabs; ++s) {
        wait_loads_at_most((NS - 2) * my_per_slab);
        LRBI_BARRIER();
        copy_slab(s + NS - 1);
        multiply_slab(s);
    }
    wait_loads<0>();
    LRBI_BARRIER();

    // wavefronts' partial accumulators -> LDS; lane holds operand rows 4 kg + v, column row16 of each 16 x 16 block
    float *red = (float *)smem; // [8][2][16][16]
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[((wave * 2 + cb) * 16 + 4 * kg + v) * 16 + row16] = acc[cb][v];
    LRBI_BARRIER();
#undef LRBI_BARRIER
    // one lane per (unit, batch column): the four pre-activations (sums over the wavefronts, in wavefront order),
    // then c = sigm(z_f) c + sigm(z_i) tanh(z_g), h = sigm(z_o) tanh(c)
    for (int e = tid; e < units_here * N; e += ST_THREADS) {
        const int unit = e / N, b = e - unit * N;
        const int cb = b >> 4, cc = b & 15;
        float z[4];
#pragma unroll
        for (int gate = 0; gate < 4; ++gate) {
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < ST_WAVES; ++w) v += red[((w * 2 + cb) * 16 + 4 * gate + unit) * 16 + cc];
            z[gate] = v;
        }
        const int64_t j = j0 + unit;
        const float c = lstm_sigm(z[1]) * f.C[j * f.ldc + b] + lstm_sigm(z[0]) * tanhf(z[2]);
        const float h = lstm_sigm(z[3]) * tanhf(c);
        f.C[j * f.ldc + b] = c;
        const uint16_t hs = cvt_store(Tag{}, h);
        f.H1[j * f.ldh1 + b] = hs;
        if (f.H2) f.H2[j * f.ldh2 + b] = hs;
    }
}

// The kernel serves: f16 / bf16, N = 1 or a multiple of 4 up to 32, X contiguous ([n][N] with ldx = N) and 16-byte
// aligned, W rows 16-byte aligned, n a multiple of 8, a tile row's packed I_z small enough for LDS, and enough rows to
// give every compute unit a workgroup or so.
struct StreamPlan {
    int ns;       // ring stages
    int bm, ks;   // rows per workgroup and columns per slab: (16, 256), or (8, 512) for a single column
    size_t lds;
    unsigned grid;
    int rv_pieces; // above 0: the single-column kernel that holds a row in registers, with this many 1 KB pieces
    StreamArgs a; // the geometry-derived fields only
};

static bool plan_stream(const Geom &g, int64_t N, int cus, StreamPlan &p)
{
    StreamArgs &a = p.a;
    // one column: eight rows per workgroup, so that twice as many workgroups (and copying wavefronts) share the
    // chip, and 512-column slabs: a wavefront's piece is 1 KB of one row
    p.bm = (N == 1) ? 8 : 16;
    p.ks = (N == 1) ? 512 : 256;
    const int slab_bytes = p.ks * (int)N * 2;
    a.x_instr = (slab_bytes + 1023) / 1024;
    a.x_stage = a.x_instr * 1024 + ST_X_PAD;
    a.x_pieces = (uint32_t)(((uint64_t)g.n * (uint64_t)N * 2u) >> 4);
    a.blocks_per_tile_row = (g.r + p.bm - 1) / p.bm;
    const int64_t fz_words = (int64_t)g.tile_cols * g.k * g.izw;
    if (fz_words * 4 > ST_FZ_MAX_BYTES) return false;
    a.fz_words = (int)fz_words;
    a.izw_magic = (g.izw > 1) ? (uint32_t)((((uint64_t)1 << 32) / (uint64_t)g.izw) + 1u) : 0u;
    a.fz_pad = (a.fz_words + 255) / 256 * 256; // whole copy instructions of either width
    a.fp_pitch = (ST_FP_ROWS * g.ipw + 63) / 64 * 64;
    const int nslabs = (int)((g.n + p.ks - 1) / p.ks);
    a.ms_pitch = nslabs * (p.ks / 32) + 1;
    const int64_t grid = (int64_t)g.tile_rows * a.blocks_per_tile_row;
    // Few workgroups (small m) each walk a whole row length alone, at the latency of their own ring: worth it while a
    // workgroup's rows are short (measured, 800 x 400 at rank 145 and 20 columns: 6.9 us against 29 + 4 us on the
    // tile kernel with its split reduction; 256 x 2304 at 4 columns: 8.8 against 19.7 us; against the panel kernels
    // on their tile shapes it breaks even at 128 KB per workgroup: 128 x 4096 at 8 columns 11.0 against 10.4 us)
    if (grid > 0x7FFFFFFF) return false;
    const bool panel_shape = (g.c % 128) == 0 && (g.r % 128) == 0 && g.k <= FAST_MAX_K && !g.ragged;
    if (grid < cus / 2 && (int64_t)p.bm * g.n * 2 > (panel_shape ? ST_LONE_ROWS_BYTES_PANEL : ST_LONE_ROWS_BYTES)) return false;
    // At most one workgroup per compute unit walking long rows, on a tile shape and batch that the panel kernels take
    // with 16-byte X loads: their split over n keeps more loads in flight (HBM-cold W, N = 32: 2048 x 9216 18.6 against
    // 25.8 us, 4096 x 9216 24.1 against 27.6 us; 4096 x 4096, 128 KB per workgroup: 15.2 against 14.1 us, left here)
    if (panel_shape && N >= 16 && N % 8 == 0 && grid <= cus && (int64_t)p.bm * g.n * 2 > 2 * ST_LONE_ROWS_BYTES_PANEL)
        return false;
    p.grid = (unsigned)grid;
    p.rv_pieces = 0;
    if (N == 1 && g.n <= RV_MAX_PIECES * 512) {
        int pieces = 2;
        while (pieces * 512 < g.n) pieces *= 2;
        const int ms_pitch = pieces * 16 + 1;
        const size_t lds = (size_t)pieces * 1024 +
                           ((size_t)RV_ROWS * ms_pitch + a.fz_pad + (size_t)g.tile_cols * a.fp_pitch) * 4;
        if (lds <= 64 * 1024) {
            p.rv_pieces = pieces;
            a.ms_pitch = ms_pitch;
            p.ns = 0;
            p.lds = lds;
            return true;
        }
    }
    const size_t fixed = ((size_t)p.bm * a.ms_pitch + a.fz_pad + (size_t)g.tile_cols * a.fp_pitch) * 4;
    // two workgroups per compute unit when there are more workgroups than compute units, else the deepest ring;
    // a wavefront issues at most three copies per slab, so its 6-bit load counter never limits the depth
    const size_t budget = (grid > cus) ? 80 * 1024 : 160 * 1024;
    for (int ns : {6, 4, 3}) {
        const size_t lds = (size_t)ns * (ST_WSTAGE + a.x_stage) + fixed;
        if (lds <= budget) {
            p.ns = ns;
            p.lds = lds;
            return true;
        }
    }
    return false;
}

bool stream_ok(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, const void *dX, int64_t ldx, int64_t N, int cus)
{
    if (dt != LRBI_F16 && dt != LRBI_BF16) return false;
    if (!(N == 1 || (N % 4 == 0 && N <= 32))) return false;
    if (ldx != N || ((uintptr_t)dX & 15) != 0) return false;
    if (((uintptr_t)dW & 15) != 0 || ldw % 8 != 0 || g.n % 8 != 0 || g.n < 8) return false;
    if (ldw >= ((int64_t)1 << 26) || g.n >= ((int64_t)1 << 30)) return false;       // 32-bit byte offsets within 16 rows
    if ((uint64_t)g.n * (uint64_t)N * 2u >= ((uint64_t)1 << 32)) return false;       // and within X
    StreamPlan p;
    return plan_stream(g, N, cus, p);
}

template <typename Tag, int NS, int BM, int KS>
static int launch_stream_t(const Geom &g, const StreamPlan &p, hipStream_t stream)
{
    auto kern = stream_gemm_kernel<Tag, NS, BM, KS>;
    LRBI_SET_MAX_LDS(kern, p.lds);
    LRBI_LAUNCH(kern, dim3(p.grid), dim3(ST_THREADS), p.lds, stream, g, p.a);
    return LRBI_OK;
}

template <typename Tag, int BM, int KS> static int launch_stream_ns(const Geom &g, const StreamPlan &p, hipStream_t stream)
{
    switch (p.ns) {
    case 6: return launch_stream_t<Tag, 6, BM, KS>(g, p, stream);
    case 4: return launch_stream_t<Tag, 4, BM, KS>(g, p, stream);
    default: return launch_stream_t<Tag, 3, BM, KS>(g, p, stream);
    }
}

template <typename Tag, int P> static int launch_rowvec_t(const Geom &g, const StreamPlan &p, hipStream_t stream)
{
    auto kern = rowvec_gemm_kernel<Tag, P>;
    LRBI_SET_MAX_LDS(kern, p.lds);
    LRBI_LAUNCH(kern, dim3(p.grid), dim3(ST_THREADS), p.lds, stream, g, p.a);
    return LRBI_OK;
}

template <typename Tag> static int launch_stream_shape(const Geom &g, const StreamPlan &p, hipStream_t stream)
{
    switch (p.rv_pieces) {
    case 0: break;
    case 2: return launch_rowvec_t<Tag, 2>(g, p, stream);
    case 4: return launch_rowvec_t<Tag, 4>(g, p, stream);
    case 8: return launch_rowvec_t<Tag, 8>(g, p, stream);
    default: return launch_rowvec_t<Tag, 16>(g, p, stream);
    }
    return (p.bm == 8) ? launch_stream_ns<Tag, 8, 512>(g, p, stream) : launch_stream_ns<Tag, 16, 256>(g, p, stream);
}

// dY (storage dtype) and / or dP (fp32) receive the product; the caller has checked stream_ok() with the same cus
int launch_stream_gemm(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, const uint32_t *dIp,
                       const uint32_t *dIz, const void *dX, int64_t N, void *dY, int64_t ldy, float *dP, int64_t ldp,
                       int cus, hipStream_t stream, MaskOut mo)
{
    StreamPlan p;
    if (!plan_stream(g, N, cus, p)) return LRBI_ERR_SHAPE;
    StreamArgs &a = p.a;
    a.W = (const uint16_t *)dW;
    a.ldw = ldw;
    a.Ip = dIp;
    a.Iz = dIz;
    a.X = (const uint16_t *)dX;
    a.N = (int)N;
    a.Y = (uint16_t *)dY;
    a.ldy = ldy;
    a.P = dP;
    a.ldp = ldp;
    a.fz_vec = ((((uintptr_t)dIz) & 15) == 0 && (a.fz_words & 3) == 0) ? 1 : 0;
    a.mask_out = (uint32_t *)mo.ptr;
    a.mask_pitch32 = mo.pitch16 * 4;
    a.mask_words = (int)((g.n + 127) / 128 * 4);
    if (dt == LRBI_F16) return launch_stream_shape<F16Tag>(g, p, stream);
    if (dt == LRBI_BF16) return launch_stream_shape<BF16Tag>(g, p, stream);
    return LRBI_ERR_DTYPE;
}

// The fused LSTM step serves what the ring kernel serves at 4 to 32 columns (the caller has checked stream_ok()), when
// in addition H = m / 4 and the tile height are multiples of 4, offsets fit 32 bits and LDS holds four tile rows' I_z.
// Returns LRBI_ERR_SHAPE otherwise: the caller then runs the product and the cell kernel one after the other.
template <typename Tag, int NS>
static int launch_stream_lstm_t(const Geom &g, const StreamPlan &p, const LstmFuse &f, hipStream_t stream)
{
    auto kern = stream_lstm_kernel<Tag, NS>;
    LRBI_SET_MAX_LDS(kern, p.lds);
    LRBI_LAUNCH(kern, dim3(p.grid), dim3(ST_THREADS), p.lds, stream, g, p.a, f);
    return LRBI_OK;
}

int launch_stream_lstm(const Geom &g, lrbi_dtype dt, const void *dW, int64_t ldw, const uint32_t *dIp,
                       const uint32_t *dIz, const void *dXH, int64_t B, float *dC, int64_t ldc, void *dH1, int64_t ldh1,
                       void *dH2, int64_t ldh2, int cus, hipStream_t stream)
{
    if (B < 4 || B > 32 || B % 4 != 0) return LRBI_ERR_SHAPE;
    const int64_t H = g.m / 4;
    if (g.m % 4 != 0 || H % 4 != 0 || g.r % 4 != 0) return LRBI_ERR_SHAPE;
    if ((uint64_t)g.m * (uint64_t)ldw * 2u >= ((uint64_t)1 << 32)) return LRBI_ERR_SHAPE;
    const int64_t tiles = (int64_t)g.tile_rows * g.tile_cols;
    if (tiles * g.r * g.ipw >= ((int64_t)1 << 30)) return LRBI_ERR_SHAPE;
    StreamPlan p;
    if (!plan_stream(g, B, cus, p)) return LRBI_ERR_SHAPE;
    StreamArgs &a = p.a;
    LstmFuse f;
    f.H = H;
    f.C = dC;
    f.ldc = ldc;
    f.H1 = (uint16_t *)dH1;
    f.ldh1 = ldh1;
    f.H2 = (uint16_t *)dH2;
    f.ldh2 = ldh2;
    f.fp_words = 16 * g.ipw;
    f.fp_instr = (g.tile_cols * f.fp_words + 63) / 64;
    const size_t fixed = ((size_t)16 * a.ms_pitch + (size_t)4 * a.fz_pad + (size_t)f.fp_instr * 64) * 4;
    int ns = 0;
    for (int cand : {6, 4, 3}) {
        if ((size_t)cand * (ST_WSTAGE + a.x_stage) + fixed <= 80 * 1024) {
            ns = cand;
            break;
        }
    }
    if (ns == 0) return LRBI_ERR_SHAPE;
    p.lds = (size_t)ns * (ST_WSTAGE + a.x_stage) + fixed;
    p.grid = (unsigned)(H / 4);
    a.W = (const uint16_t *)dW;
    a.ldw = ldw;
    a.Ip = dIp;
    a.Iz = dIz;
    a.X = (const uint16_t *)dXH;
    a.N = (int)B;
    a.Y = nullptr;
    a.ldy = 0;
    a.P = nullptr;
    a.ldp = 0;
    a.fz_vec = ((((uintptr_t)dIz) & 15) == 0 && (a.fz_words & 3) == 0) ? 1 : 0;
    a.mask_out = nullptr;
    a.mask_pitch32 = 0;
    a.mask_words = 0;
#define LRBI_LSTM_NS(TAG)                                                     \
    switch (ns) {                                                             \
    case 6: return launch_stream_lstm_t<TAG, 6>(g, p, f, stream);             \
    case 4: return launch_stream_lstm_t<TAG, 4>(g, p, f, stream);             \
    default: return launch_stream_lstm_t<TAG, 3>(g, p, f, stream);            \
    }
    if (dt == LRBI_F16) { LRBI_LSTM_NS(F16Tag) }
    if (dt == LRBI_BF16) { LRBI_LSTM_NS(BF16Tag) }
#undef LRBI_LSTM_NS
    return LRBI_ERR_DTYPE;
}

} // namespace lrbi
