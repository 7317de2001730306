// Fused ECF8 decode + FP8 GEMM for small batches on gfx950 (MI355X), and the
// same GEMM on uncompressed FP8 weights for comparison.
//
//   Y[m][n] = sum_k X[m][k] * W[n][k],   X: M x K FP8 E4M3 (M <= 64),
//   W: rows x K FP8 E4M3 (the compressed tensor), Y: M x rows fp32.
//
// The paper materialises a layer's weights in a buffer and lets the framework's
// GEMM read them back (Section 3.3).  At small M that GEMM is bound by reading
// W, so here the decoded weights never leave the CU: a workgroup decodes a tile
// of 16 rows of W into LDS (same stage / pair table / two-chain steps as the
// decode kernel, with ds_write_b128 in place of the global store) and feeds it
// to v_mfma_f32_16x16x32_fp8_fp8 as the B operand; X is the A operand, held in
// registers.  This is the only place the matrix cores are used.  With K = 4096 and 64
// symbols per lane a chunk is exactly one row of W.
//
// Per tile: 8 waves decode 2 rows each -> barrier -> each wave multiplies its
// 512-wide K slice (16 MFMA steps per 16-row block of X) -> partial sums meet in
// LDS -> 16 x M outputs written.  Tile rows are padded by 16 bytes so the 16
// rows of a B-operand read fall into different LDS banks.
#include "ecf8_device.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int GN = 64;                    // symbols per lane this kernel is built for
constexpr int GK = 4096;                  // K: one chunk = one row of W
constexpr int GWAVES_MAX = 16;
constexpr int GSTAGE = GN * 32 + 64;      // as in the decode kernel
constexpr int GSEGS = (GSTAGE / 16 + 63) / 64;
constexpr int GPIECES = GN / 16;
constexpr int TILE_ROWS = 16;
constexpr int TILE_STRIDE = GK + 16;
constexpr int G_OFF_TBL = 0;
constexpr int G_OFF_SYM = G_OFF_TBL + TBL_ENTRIES * 2;
constexpr int G_OFF_STAGE = G_OFF_SYM + 128;
constexpr int G_OFF_TILE = G_OFF_STAGE + GWAVES_MAX * GSTAGE;
constexpr int G_TOTAL = G_OFF_TILE + TILE_ROWS * TILE_STRIDE;
static_assert(GWAVES_MAX * GSTAGE + TILE_ROWS * TILE_STRIDE >= TBL_ENTRIES * 2, "table-build scratch");
static_assert(G_TOTAL <= 160 * 1024, "LDS of one gfx950 CU");

struct GArgs {
    uint64_t d_blob, d_w, d_x, d_y;       // d_blob: compressed W; d_w: raw W (raw kernel)
    uint64_t rows, n_elem;
    uint64_t off_cb, off_lb, off_st, off_pl, st_bytes, off_tbl;
    uint8_t code_len[16];
    uint32_t M;
};

constexpr int ksteps(int nw) { return GK / nw / 32; }  // MFMA steps of 32 over a wave's K slice

// A operands of a wave: its K slice of X for every 16-row block, loaded once per workgroup and
// kept in registers for all tiles (X is M x K <= 256 KiB: half of the CU's register file at
// M = 64, but re-reading it from L2 for each of ~900 tiles costs more than everything else).
template <int MT, int NW>
__device__ __forceinline__ void load_x_slice(const GArgs &a, int tid, long (&areg)[MT][ksteps(NW)])
{
    constexpr int KSTEPS = ksteps(NW);
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const GLOBAL uint8_t *X = (const GLOBAL uint8_t *)a.d_x;
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int s = 0; s < KSTEPS; s++) {
            const uint32_t m = 16 * mt + n;                                   // A row = lane & 15
            const uint32_t k = wave * (GK / NW) + 32 * s + 8 * g;
            areg[mt][s] = 0;
            if (m < a.M) areg[mt][s] = *(const GLOBAL long *)(X + (uint64_t)m * GK + k);
        }
}

// Multiply phase shared by both kernels: the tile in LDS times X, partial sums
// reduced over the NW waves, 16 x M results written.
template <int MT, int NW>
__device__ __forceinline__ void multiply_tile(uint8_t *smem, const GArgs &a, uint64_t tile, int tid,
                                              const long (&areg)[MT][ksteps(NW)])
{
    constexpr int KSTEPS = ksteps(NW);
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    uint8_t *tile_mem = smem + G_OFF_TILE;
    // Note on accuracy: the FP8 matrix core aligns each lane's 8 products to the largest of them and
    // truncates what lies more than about 13 bits below it, so a result can be off by up to
    // 7 * 2^-13 of sum |x w| in the worst case (typically a few 1e-5 of it on heavy-tailed weights).
    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    const uint32_t kbase = wave * (GK / NW);
#pragma unroll
    for (int s = 0; s < KSTEPS; s++) {
        const uint32_t k = kbase + 32 * s + 8 * g;
        const long b = *(const long *)(tile_mem + n * TILE_STRIDE + k);       // W[n][k .. k+8)
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(areg[mt][s], b, acc[mt], 0, 0, 0);
    }
    __syncthreads();                          // every wave is done reading the tile
    f32x4 *red = (f32x4 *)tile_mem;           // [wave][mt][lane]
#pragma unroll
    for (int mt = 0; mt < MT; mt++) red[(wave * MT + mt) * 64 + lane] = acc[mt];
    __syncthreads();
    // a lane of the accumulator holds D[4*(lane>>4) + r][lane & 15], r = 0..3
    GLOBAL float *Y = (GLOBAL float *)a.d_y;
    for (int o = tid; o < MT * 256; o += NW * 64) {
        const int mt = o >> 8, l = (o >> 2) & 63, r = o & 3;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < NW; w++) sum += ((const float *)&red[(w * MT + mt) * 64 + l])[r];
        const uint32_t m = 16 * mt + 4 * (l >> 4) + r;
        if (m < a.M) Y[(uint64_t)m * a.rows + tile * TILE_ROWS + (l & 15)] = sum;
    }
    __syncthreads();                          // the tile area is free again
}

// NW waves per workgroup, each decoding RPW = 16 / NW rows of a tile.  The tile's metadata is
// loaded two tiles ahead and its stream spans and nibble planes one tile ahead (into registers),
// so the decode of a tile never waits for HBM.  PAIRFIT as in the decode kernel.
template <int MT, int NW, bool PAIRFIT>
__global__ __launch_bounds__(NW * 64) void ecf8_gemm_kernel(GArgs a)
{
    constexpr int RPW = TILE_ROWS / NW;
    constexpr int KSTEPS = ksteps(NW);
    __shared__ __attribute__((aligned(16))) uint8_t smem[G_TOTAL];
    uint16_t *tbl = (uint16_t *)(smem + G_OFF_TBL);
    uint32_t *s_len = (uint32_t *)(smem + G_OFF_SYM);
    uint32_t *s_code = s_len + 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t stage_off = G_OFF_STAGE + wave * GSTAGE;
    uint8_t *stage = smem + stage_off;
    uint8_t *tile_mem = smem + G_OFF_TILE;

    const GLOBAL uint64_t *chunk_bit = (const GLOBAL uint64_t *)(a.d_blob + a.off_cb);
    const GLOBAL uint16_t *lane_bits = (const GLOBAL uint16_t *)(a.d_blob + a.off_lb);
    const GLOBAL uint8_t *stream = (const GLOBAL uint8_t *)(a.d_blob + a.off_st);
    const GLOBAL uint8_t *plane = (const GLOBAL uint8_t *)(a.d_blob + a.off_pl);

    struct Meta { uint64_t b0, b1; uint32_t lb; };
    struct Payload { u32x4 seg[GSEGS]; u32x2 pl[GPIECES]; };
    auto row_of = [&](uint64_t tile, int rr) -> uint64_t { return tile * TILE_ROWS + wave + NW * rr; };  // chunk = row
    auto load_meta = [&](uint64_t cl) {
        Meta m;
        m.b0 = chunk_bit[cl];
        m.b1 = chunk_bit[cl + 1];
        m.lb = lane_bits[cl * 64 + lane];
        return m;
    };
    auto span_of = [&](const Meta &m, uint64_t &byte0) {
        uint64_t byte_end = ((m.b1 + 7) >> 3) + 8;
        if (byte_end > a.st_bytes) byte_end = a.st_bytes;
        byte0 = (m.b0 >> 3) & ~15ull;
        if (byte0 > byte_end) byte0 = byte_end;
        return byte_end - byte0;
    };
    auto load_payload = [&](uint64_t cl, const Meta &m) {
        Payload p;
        uint64_t byte0;
        const uint64_t span = span_of(m, byte0);
        const GLOBAL u32x2 *plane_c = (const GLOBAL u32x2 *)(plane + cl * (32ull * GN));
#pragma unroll
        for (int j = 0; j < GPIECES; j++) p.pl[j] = __builtin_nontemporal_load(&plane_c[j * 64 + lane]);
#pragma unroll
        for (int k = 0; k < GSEGS; k++) {
            const uint32_t i = (lane + 64 * k) * 16;
            p.seg[k] = u32x4{0, 0, 0, 0};
            if (span <= (uint64_t)GSTAGE && i < (uint32_t)span)
                p.seg[k] = __builtin_nontemporal_load((const GLOBAL u32x4 *)(stream + byte0 + i));
        }
        return p;
    };

    const uint64_t n_tiles = a.rows / TILE_ROWS;
    uint64_t tile = blockIdx.x;
    // start-up: the first tile's loads are in flight while the table is set up
    Meta m_cur[RPW], m_next[RPW];
    Payload p_cur[RPW];
#pragma unroll
    for (int rr = 0; rr < RPW; rr++) {
        m_cur[rr] = Meta{0, 0, 0};
        if (tile < n_tiles) m_cur[rr] = load_meta(row_of(tile, rr));
        m_next[rr] = m_cur[rr];
        if (tile + gridDim.x < n_tiles) m_next[rr] = load_meta(row_of(tile + gridDim.x, rr));
    }
#pragma unroll
    for (int rr = 0; rr < RPW; rr++)
        if (tile < n_tiles) p_cur[rr] = load_payload(row_of(tile, rr), m_cur[rr]);

    uint64_t len_lo, len_hi;
    __builtin_memcpy(&len_lo, a.code_len, 8);
    __builtin_memcpy(&len_hi, a.code_len + 8, 8);
    if (a.off_tbl) {
        const GLOBAL u32x4 *src = (const GLOBAL u32x4 *)(a.d_blob + a.off_tbl);
        for (int i = tid; i < TBL_ENTRIES * 2 / 16; i += NW * 64) ((u32x4 *)tbl)[i] = src[i];
        build_symbol_arrays(len_lo, len_hi, s_len, s_code, tid);
        __syncthreads();
    } else {
        build_tables(len_lo, len_hi, tbl, s_len, s_code, (uint16_t *)(smem + G_OFF_STAGE), tid, NW * 64);
    }

    long areg[MT][KSTEPS];
    load_x_slice<MT, NW>(a, tid, areg);

    for (; tile < n_tiles; tile += gridDim.x) {
        const uint64_t tile1 = tile + gridDim.x, tile2 = tile1 + gridDim.x;
#pragma unroll
        for (int rr = 0; rr < RPW; rr++) {
            const Meta m = m_cur[rr];
            uint8_t *trow = tile_mem + (wave + NW * rr) * TILE_STRIDE;
            uint64_t byte0;
            const uint64_t span = span_of(m, byte0);
            const uint32_t rel = wave_incl_scan(m.lb) - m.lb;
            const uint64_t start = __builtin_amdgcn_readfirstlane((uint32_t)m.b0) |
                                   ((uint64_t)__builtin_amdgcn_readfirstlane((uint32_t)(m.b0 >> 32)) << 32);
            const bool staged = __builtin_amdgcn_readfirstlane((uint32_t)(span <= (uint64_t)GSTAGE)) != 0;
            u32x2 pl[GPIECES];
#pragma unroll
            for (int j = 0; j < GPIECES; j++) pl[j] = p_cur[rr].pl[j];
            if (staged) {
#pragma unroll
                for (int k = 0; k < GSEGS; k++) {
                    const uint32_t i = (lane + 64 * k) * 16;
                    if (i < (uint32_t)GSTAGE) *(u32x4 *)(stage + i) = p_cur[rr].seg[k];
                }
            }
            // this row's registers are free: fetch the same row of the next tile, and the
            // metadata of the tile after it
            Meta m_next2 = m_next[rr];
            if (tile1 < n_tiles) {
                p_cur[rr] = load_payload(row_of(tile1, rr), m_next[rr]);
                if (tile2 < n_tiles) m_next2 = load_meta(row_of(tile2, rr));
            }
            if (staged) {
                uint32_t bpA = stage_off * 8 + (uint32_t)(start - byte0 * 8) + rel;
                uint32_t bpB = bpA + m.lb;
#pragma unroll
                for (int Q = 0; Q < GPIECES / 2; Q++) {
                    uint32_t dwA[4], dwB[4];
#pragma unroll
                    for (int t = 0; t < 4; t++) quad_step2<PAIRFIT>(smem, tbl, s_len, s_code, bpA, bpB, dwA[t], dwB[t]);
                    *(u32x4 *)(trow + (Q * 64 + lane) * 16) = merge_piece(dwA, pl[Q]);
                    *(u32x4 *)(trow + ((Q + GPIECES / 2) * 64 + lane) * 16) = merge_piece(dwB, pl[Q + GPIECES / 2]);
                }
            } else {
                // span larger than the stage: symbol by symbol from HBM into the tile row
                const GLOBAL uint8_t *sp = stream + byte0;
                uint64_t bA = (start - byte0 * 8) + rel, bB = bA + m.lb;
                const uint64_t elem0 = row_of(tile, rr) * (uint64_t)GK;
#pragma unroll 1
                for (int Q = 0; Q < GPIECES; Q++) {
                    const uint32_t o = (Q * 64 + lane) * 16;
                    const bool fwd = Q < GPIECES / 2;
#pragma unroll 1
                    for (uint32_t i = 0; i < 16; i++) {
                        const uint32_t w = fwd ? global_window<+1>(sp, bA) : global_window<-1>(sp, bB);
                        const uint32_t r = decode_one(w, tbl, s_len, s_code);
                        if (fwd) bA += r >> 8; else bB -= r >> 8;
                        const uint64_t el = elem0 + o + i;
                        const uint32_t pb = plane[(el >> 3) * 4 + (el & 3)];
                        const uint32_t nib = (el & 4) ? pb >> 4 : pb & 15u;
                        trow[o + i] = (uint8_t)(((r & 15u) << 3) | ((nib & 8u) << 4) | (nib & 7u));
                    }
                }
            }
            m_cur[rr] = m_next[rr];
            m_next[rr] = m_next2;
        }
        __syncthreads();
        multiply_tile<MT, NW>(smem, a, tile, tid, areg);
    }
}

// The same GEMM on uncompressed W, with the fused kernel's workgroup shape and K split, so that
// the two agree bit for bit.
template <int MT, int NW>
__global__ __launch_bounds__(NW * 64) void ecf8_gemm_raw_kernel(GArgs a)
{
    constexpr int RPW = TILE_ROWS / NW, KSTEPS = ksteps(NW);
    __shared__ __attribute__((aligned(16))) uint8_t smem[G_TOTAL];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint8_t *tile_mem = smem + G_OFF_TILE;
    const GLOBAL uint8_t *W = (const GLOBAL uint8_t *)a.d_w;
    long areg[MT][KSTEPS];
    load_x_slice<MT, NW>(a, tid, areg);
    const uint64_t n_tiles = a.rows / TILE_ROWS;
    for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        u32x4 v[RPW][GK / 1024];
#pragma unroll
        for (int rr = 0; rr < RPW; rr++)
#pragma unroll
            for (int j = 0; j < GK / 1024; j++)
                v[rr][j] = *(const GLOBAL u32x4 *)(W + (tile * TILE_ROWS + wave + NW * rr) * (uint64_t)GK + (j * 64 + lane) * 16);
#pragma unroll
        for (int rr = 0; rr < RPW; rr++)
#pragma unroll
            for (int j = 0; j < GK / 1024; j++)
                *(u32x4 *)(tile_mem + (wave + NW * rr) * TILE_STRIDE + (j * 64 + lane) * 16) = v[rr][j];
        __syncthreads();
        multiply_tile<MT, NW>(smem, a, tile, tid, areg);
    }
}

int grid_for(uint64_t n_tiles)
{
    int cus = device_cus();
    if (cus <= 0) return -1;
    return (int)(n_tiles < (uint64_t)cus ? n_tiles : (uint64_t)cus);
}

int check_gemm_args(uint64_t rows, uint64_t cols, const void *d_x, uint32_t M, const void *d_y)
{
    if (!d_x || !d_y || M == 0 || M > 64) return ECF8_E_ARG;
    if (cols != GK || rows == 0 || rows % TILE_ROWS) return ECF8_E_ARG;
    if (((uintptr_t)d_x & 15) || ((uintptr_t)d_y & 3)) return ECF8_E_ALIGN;
    return ECF8_OK;
}

} // namespace

extern "C" {

int ecf8_gemm_fp8(const ecf8_header *h, const void *d_blob, const void *d_x, uint32_t M, float *d_y, void *stream)
{
    if (!h || !d_blob) return ECF8_E_ARG;
    if (h->magic != ECF8_MAGIC || h->version != ECF8_VERSION || (h->table_bits != 0 && h->table_bits != ECF8_TB))
        return ECF8_E_FORMAT;
    if (h->lane_syms != GN || h->group_chunks != 1) return ECF8_E_ARG;   // one chunk = one row of W
    int rc = check_gemm_args(h->rows, h->cols, d_x, M, d_y);
    if (rc) return rc;
    if (h->n_elem != h->rows * h->cols || h->n_chunks != h->rows) return ECF8_E_FORMAT;
    if ((uintptr_t)d_blob & 15) return ECF8_E_ALIGN;
    GArgs a{};
    a.d_blob = (uint64_t)(uintptr_t)d_blob;
    a.d_x = (uint64_t)(uintptr_t)d_x;
    a.d_y = (uint64_t)(uintptr_t)d_y;
    a.rows = h->rows;
    a.n_elem = h->n_elem;
    a.off_cb = h->off_chunk_bit;
    a.off_lb = h->off_lane_bits;
    a.off_st = h->off_stream;
    a.off_pl = h->off_plane;
    a.st_bytes = h->stream_bytes;
    a.off_tbl = h->table_bits ? 256 : 0;
    for (int i = 0; i < 16; i++) a.code_len[i] = h->code_len[i];
    a.M = M;
    const int grid = grid_for(a.rows / TILE_ROWS);
    if (grid <= 0) return ECF8_E_HIP;
    hipStream_t s = (hipStream_t)stream;
    uint32_t max_len = 0;
    for (int i = 0; i < 16; i++) max_len = h->code_len[i] > max_len ? h->code_len[i] : max_len;
    const bool pairfit = 2 * max_len <= (uint32_t)TB;
    // 16 waves (one row of the tile each) while X fits their registers, 8 waves of two rows at M > 32
#define ECF8_GEMM_LAUNCH(MT, NW)                                                                            \
    do {                                                                                                   \
        if (pairfit) hipLaunchKernelGGL((ecf8_gemm_kernel<MT, NW, true>), dim3(grid), dim3(NW * 64), 0, s, a);  \
        else hipLaunchKernelGGL((ecf8_gemm_kernel<MT, NW, false>), dim3(grid), dim3(NW * 64), 0, s, a);         \
    } while (0)
    if (M <= 16) ECF8_GEMM_LAUNCH(1, 16);
    else if (M <= 32) ECF8_GEMM_LAUNCH(2, 16);
    else ECF8_GEMM_LAUNCH(4, 8);
#undef ECF8_GEMM_LAUNCH
    return hipGetLastError() == hipSuccess ? ECF8_OK : ECF8_E_HIP;
}

int ecf8_gemm_fp8_raw(const void *d_w, uint64_t rows, uint64_t cols, const void *d_x, uint32_t M, float *d_y,
                      void *stream)
{
    if (!d_w) return ECF8_E_ARG;
    int rc = check_gemm_args(rows, cols, d_x, M, d_y);
    if (rc) return rc;
    if ((uintptr_t)d_w & 15) return ECF8_E_ALIGN;
    GArgs a{};
    a.d_w = (uint64_t)(uintptr_t)d_w;
    a.d_x = (uint64_t)(uintptr_t)d_x;
    a.d_y = (uint64_t)(uintptr_t)d_y;
    a.rows = rows;
    a.n_elem = rows * cols;
    a.M = M;
    const int grid = grid_for(rows / TILE_ROWS);
    if (grid <= 0) return ECF8_E_HIP;
    hipStream_t s = (hipStream_t)stream;
    if (M <= 16) hipLaunchKernelGGL((ecf8_gemm_raw_kernel<1, 16>), dim3(grid), dim3(16 * 64), 0, s, a);
    else if (M <= 32) hipLaunchKernelGGL((ecf8_gemm_raw_kernel<2, 16>), dim3(grid), dim3(16 * 64), 0, s, a);
    else hipLaunchKernelGGL((ecf8_gemm_raw_kernel<4, 8>), dim3(grid), dim3(8 * 64), 0, s, a);
    return hipGetLastError() == hipSuccess ? ECF8_OK : ECF8_E_HIP;
}

} // extern "C"
