// Kernels and host-side launch helpers of the fused ECF8 decode + GEMM, shared by the translation units
// that export the calls (ecf8_gemm.hip: the FP8 matrix-core calls; ecf8_gemm_exact.hip: the calls that
// multiply on the F16 matrix cores).  Everything sits in an unnamed namespace: each unit instantiates
// what it launches.
#ifndef ECF8_GEMM_KERNELS_H
#define ECF8_GEMM_KERNELS_H

#include "ecf8_device.h"

#include <cstring>

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

constexpr int GK = 4096;                        // K
constexpr int BLOCK_ROWS = 16;

// N symbols per lane: a chunk is 16 rows x 4N columns; NW waves per workgroup; MT blocks of 16 rows of X
template <int MT, int NW, int N>
struct GCfg {
    static constexpr int BLOCK_COLS = 4 * N;
    static constexpr int KCHUNKS = GK / BLOCK_COLS;        // chunks per block of rows
    static constexpr int KPW = KCHUNKS / NW;               // of which each wave takes this many
    static constexpr int PIECES = N / 16;
    static constexpr int STAGE = 64 * N * (TB / 2) / 8 + 64;   // worst-case span of a chunk under the cap
    static constexpr int SEGS = (STAGE / 16 + 63) / 64;
    static_assert(STAGE % 16 == 0, "stage rows are written with 16-byte stores");
    static_assert(KPW * NW == KCHUNKS && KPW >= 1, "waves split the chunks of a block evenly");
    static constexpr int OFF_TBL = 0;
    static constexpr int OFF_SYM = OFF_TBL + TBL_ENTRIES * 2;
    static constexpr int OFF_STAGE = OFF_SYM + 128;
    static constexpr int OFF_RED = OFF_STAGE + NW * STAGE;
    static constexpr int RED_BYTES = NW * MT * 64 * 16;            // one buffer of partial sums: one block of rows, every wave
    // Blocks per barrier.  Up to 16 columns of X with one chunk per wave and block, the workgroup's barrier per block
    // of rows is a fifth of the loop: there the waves park the partial sums of four blocks in a row in LDS and
    // meet once to add them up.  Else one block per barrier, in two buffers used in turn.
    static constexpr int BPB = (MT == 1 && KPW == 1) ? 4 : 1;
    static constexpr int RED_BUFS = BPB == 1 ? 2 : BPB;
    static constexpr int TOTAL = OFF_RED + RED_BUFS * RED_BYTES;
    static_assert(NW * STAGE + RED_BUFS * RED_BYTES >= TBL_ENTRIES * 2, "table-build scratch");
    static_assert(TOTAL <= 160 * 1024, "LDS of one gfx950 CU");
};

struct GArgs {
    uint64_t d_blob, d_w, d_x, d_y;       // d_blob: compressed W; d_w: raw W (raw kernel)
    uint64_t rows;
    uint64_t off_cb, off_lb, off_st, off_pl, st_bytes, off_tbl;
    uint8_t code_len[16];
    uint32_t M;
    uint64_t d_ws, d_xs;                  // SCALED kernels: per-128x128-block scales of W, scales of X (or 0)
    uint32_t xs_cols;                     // scales per row of X: 1, or K / 128 (one per 128 columns)
    uint64_t K;                           // columns of W (a multiple of 256; 4096 for the fixed-K kernels)
    uint32_t slices;                      // split K: workgroups that share a block of rows (divides K / 256), else 1
    uint64_t d_part, d_ctr;               // split K: partial sums [block][slice][MT * 256] fp32, arrival counters [block] u32
};

constexpr int SCALE_BLOCK = 128;                // W carries one fp32 scale per 128 x 128 block

// acc += part * s, element by element, the same operation in the fused and in the raw kernel
// acc += part * (s * x-scale), element by element, where X carries one scale per row and 128 columns: the
// scales of block kb for the accumulator rows of this lane (row m = 16 mt + 4 (lane / 16) + r) are
// fetched one tile of 16 rows at a time.
template <int MT>
__device__ __forceinline__ void add_scaled_group(f32x4 (&acc)[MT], const f32x4 (&part)[MT], float s, const GArgs &a,
                                                 int lane, uint32_t kb)
{
    const GLOBAL float *xs = (const GLOBAL float *)a.d_xs;
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const uint32_t m = 16 * mt + 4 * (lane >> 4) + r;
            v[r] = m < a.M ? xs[(uint64_t)m * a.xs_cols + kb] : 0.f;
        }
#pragma unroll
        for (int r = 0; r < 4; r++) acc[mt][r] = __builtin_fmaf(part[mt][r], s * v[r], acc[mt][r]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int MT>
__device__ __forceinline__ void add_scaled(f32x4 (&acc)[MT], const f32x4 (&part)[MT], float s)
{
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int r = 0; r < 4; r++) acc[mt][r] = __builtin_fmaf(part[mt][r], s, acc[mt][r]);
}

__device__ __forceinline__ long lo64(u32x4 v) { return (long)(((uint64_t)v.y << 32) | v.x); }
__device__ __forceinline__ long hi64(u32x4 v) { return (long)(((uint64_t)v.w << 32) | v.z); }

// A operands of a wave: for each of its chunks (K slices of 4N) and each piece q, the 16 bytes
// X[m][4N kc + 64 q + 16 g .. + 16) of lane (m = l % 16, g = l / 16), loaded once and kept for
// all blocks (X is M x K <= 256 KiB: half of the CU's register file at M = 64, but re-reading
// it for each of ~900 blocks costs more than everything else).
template <int MT, int NW, int N>
__device__ __forceinline__ void load_x_slice(const GArgs &a, int tid,
                                             u32x4 (&areg)[MT][GCfg<MT, NW, N>::KPW][GCfg<MT, NW, N>::PIECES])
{
    using C = GCfg<MT, NW, N>;
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const GLOBAL uint8_t *X = (const GLOBAL uint8_t *)a.d_x;
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int i = 0; i < C::KPW; i++)
#pragma unroll
            for (int q = 0; q < C::PIECES; q++) {
                const uint32_t m = 16 * mt + n;
                const uint32_t k = (wave + NW * i) * C::BLOCK_COLS + 64 * q + 16 * g;
                areg[mt][i][q] = u32x4{0, 0, 0, 0};
                if (m < a.M) areg[mt][i][q] = *(const GLOBAL u32x4 *)(X + (uint64_t)m * GK + k);
            }
}

// The sums of one chunk (16 rows x 256 columns).  Without scales a chunk adds straight into the block's
// accumulators.  With scales its two 128-column halves -- exactly its forward and its backward run --
// are summed by the matrix cores apart and enter the block's sum through one multiply-add each, with
// the scale of their 128 x 128 block of W (times the scale of X for that row and slice, if X has those).
template <int MT, int SC>
struct ChunkSums {
    static constexpr bool SCALED = SC != 0, XGROUPS = SC == 2;
    f32x4 partA[SCALED ? MT : 1], partB[SCALED ? MT : 1];
    float sA = 1.f, sB = 1.f;
    uint32_t kbA = 0;              // the chunk's first 128-column block of K

    __device__ __forceinline__ void begin(const GArgs &a, uint64_t block, uint32_t kc)
    {
        if constexpr (SCALED) {
            const GLOBAL float *ws = (const GLOBAL float *)a.d_ws + (block * BLOCK_ROWS / SCALE_BLOCK) * (a.K / SCALE_BLOCK) + 2 * kc;
            sA = ws[0];
            sB = ws[1];
            kbA = 2 * kc;
#pragma unroll
            for (int mt = 0; mt < MT; mt++) partA[mt] = partB[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
    // where the MFMAs of the forward / backward run accumulate
    __device__ __forceinline__ auto &first(f32x4 (&acc)[MT]) { if constexpr (SCALED) return partA; else return acc; }
    __device__ __forceinline__ auto &second(f32x4 (&acc)[MT]) { if constexpr (SCALED) return partB; else return acc; }
    __device__ __forceinline__ void end(f32x4 (&acc)[MT], const GArgs &a, int lane)
    {
        if constexpr (XGROUPS) {   // the scales of X are fetched here: held over the decode they would cost it registers
            add_scaled_group<MT>(acc, partA, sA, a, lane, kbA);
            add_scaled_group<MT>(acc, partB, sB, a, lane, kbA + 1);
        } else if constexpr (SCALED) {
            add_scaled<MT>(acc, partA, sA);
            add_scaled<MT>(acc, partB, sB);
        }
    }
};

// Eight E4M3 bytes as eight halves.  Every E4M3 value, subnormals included, is a half exactly (3 mantissa
// bits, exponents 2^-9 .. 2^8), so nothing is rounded here; NaN encodings stay NaN.
__device__ __forceinline__ f16x8 e4m3x8_to_f16(uint32_t lo, uint32_t hi)
{
    const f16x2 a = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lo, 1.0f, false);
    const f16x2 b = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lo, 1.0f, true);
    const f16x2 c = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hi, 1.0f, false);
    const f16x2 d = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hi, 1.0f, true);
    return f16x8{a.x, a.y, b.x, b.y, c.x, c.y, d.x, d.y};
}

// One piece (16 K-elements of this lane's row of W, in w) times the matching 16 columns of X (A_OF_MT:
// the piece of X for tile mt_).  Two ways to multiply, chosen by the kernels' ACC parameter:
//   ACC = 0  the FP8 matrix core (v_mfma_f32_16x16x32_fp8_fp8) on the bytes as they are.  It aligns each
//            lane's 8 products to the largest of them and drops what lies more than about 13 bits below
//            it, so an output can be off by up to 7 * 2^-13 of sum |x w| (a few 1e-5 of it on
//            heavy-tailed weights);
//   ACC = 1  both operands converted to halves in registers (exact, see above) and multiplied by the F16
//            matrix core (v_mfma_f32_16x16x32_f16), which keeps the exact products' fp32 sums: outputs
//            within fp32 rounding of the true sum.  Same lanes, same K order: a lane's 8 bytes of a step
//            become its 8 halves.
#define ECF8_MFMA_OPERANDS(acc, A_OF_MT, W_PIECE)                                                        \
    do {                                                                                                 \
        const u32x4 w_ = (W_PIECE);                                                                      \
        if constexpr (ACC == 0) {                                                                        \
            _Pragma("unroll") for (int mt_ = 0; mt_ < MT; mt_++) {                                       \
                const u32x4 a_ = A_OF_MT;                                                                \
                acc[mt_] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(lo64(a_), lo64(w_), acc[mt_], 0, 0, 0); \
                acc[mt_] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(hi64(a_), hi64(w_), acc[mt_], 0, 0, 0); \
            }                                                                                            \
        } else {                                                                                         \
            const f16x8 wl_ = e4m3x8_to_f16(w_.x, w_.y), wh_ = e4m3x8_to_f16(w_.z, w_.w);                \
            _Pragma("unroll") for (int mt_ = 0; mt_ < MT; mt_++) {                                       \
                const u32x4 a_ = A_OF_MT;                                                                \
                acc[mt_] = __builtin_amdgcn_mfma_f32_16x16x32_f16(e4m3x8_to_f16(a_.x, a_.y), wl_, acc[mt_], 0, 0, 0); \
                acc[mt_] = __builtin_amdgcn_mfma_f32_16x16x32_f16(e4m3x8_to_f16(a_.z, a_.w), wh_, acc[mt_], 0, 0, 0); \
            }                                                                                            \
        }                                                                                                \
    } while (0)
#define ECF8_MFMA_PIECE(acc, areg, i, p, W_PIECE) ECF8_MFMA_OPERANDS(acc, areg[mt_][i][p], W_PIECE)

// Partial sums of the NW waves -> 16 x M outputs of block `block`.  `red` is the buffer of this
// block's parity; the one barrier also orders its reuse two blocks later (a thread passes the
// next block's barrier only after every thread has finished summing here).
template <int MT, int NW, bool SCALED = false>
__device__ __forceinline__ void reduce_block(f32x4 *red, const GArgs &a, uint64_t block, int tid, const f32x4 (&acc)[MT])
{
    const int lane = tid & 63, wave = tid >> 6;
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
        if (m < a.M) {
            if (SCALED && a.d_xs && a.xs_cols == 1) sum *= ((const GLOBAL float *)a.d_xs)[m];
            Y[(uint64_t)m * a.rows + block * BLOCK_ROWS + (l & 15)] = sum;
        }
    }
}

// reduce_block for `count` blocks of rows at once (up to 16 columns of X): the waves have parked their partial sums of
// blocks first, first + stride, ... in buffers 0, 1, ... of `red`; the caller's barrier lies between that and this.
// Every output is summed over the waves in reduce_block's order.
template <int NW, bool SCALED>
__device__ __forceinline__ void reduce_parked(const f32x4 *red, const GArgs &a, uint64_t first, uint64_t stride, uint32_t count, int tid)
{
    GLOBAL float *Y = (GLOBAL float *)a.d_y;
    for (uint32_t o = tid; o < count * 256; o += NW * 64) {
        const uint32_t j = o >> 8, l = (o >> 2) & 63, r = o & 3;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < NW; w++) sum += ((const float *)&red[(j * NW + w) * 64 + l])[r];
        const uint32_t m = 4 * (l >> 4) + r;
        if (m < a.M) {
            if (SCALED && a.d_xs && a.xs_cols == 1) sum *= ((const GLOBAL float *)a.d_xs)[m];
            Y[(uint64_t)m * a.rows + (first + j * stride) * BLOCK_ROWS + (l & 15)] = sum;
        }
    }
}

// How the NW waves of a workgroup share the work of a unit in the any-K kernels.  Long K: a unit is one
// block of rows and its chunks are dealt round-robin to all waves.  Short K (at most NW / 2 chunks per
// block): the waves form `groups` groups of `wpb`, and each group takes a block of rows of its own --
// blocks j, j + 1, ... of the workgroup's sequence -- so that no wave is left without work (at K = 2048,
// 8 chunks, half of 16 waves would be).
struct Deal {
    uint32_t groups, wpb;       // blocks per unit; waves per block
    uint32_t gi, kw;            // this wave: its group, its place in the group
    uint32_t my_chunks;         // chunks of a block (or slice) that fall to this wave
};

template <int NW>
__device__ __forceinline__ Deal deal_chunks(uint32_t unit_chunks, bool split, int wave)
{
    Deal d;
    const uint32_t w = uniform32((uint32_t)wave);       // the same for every lane: keep all of this in scalar registers
    d.groups = (!split && 2 * unit_chunks <= (uint32_t)NW) ? (uint32_t)NW / unit_chunks : 1u;
    d.wpb = (uint32_t)NW / d.groups;
    d.gi = w / d.wpb;
    d.kw = w % d.wpb;
    d.my_chunks = (d.gi < d.groups && unit_chunks > d.kw) ? (unit_chunks - d.kw + d.wpb - 1) / d.wpb : 0u;
    return d;
}

// reduce_block for a unit of d.groups blocks: blocks j0 .. j0 + groups - 1 of the sequence first + j * stride
// (those below `count`), each summed over the waves of its group -- in the order reduce_block takes them,
// so that a block's result does not depend on how many blocks shared the unit.
template <int MT, int NW, bool SCALED>
__device__ __forceinline__ void reduce_groups(f32x4 *red, const GArgs &a, uint64_t first, uint64_t stride, uint64_t j0, uint64_t count,
                                              const Deal &d, int tid, const f32x4 (&acc)[MT])
{
    if (d.groups == 1) {
        reduce_block<MT, NW, SCALED>(red, a, first + j0 * stride, tid, acc);
        return;
    }
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int mt = 0; mt < MT; mt++) red[(wave * MT + mt) * 64 + lane] = acc[mt];
    __syncthreads();
    GLOBAL float *Y = (GLOBAL float *)a.d_y;
    for (uint32_t o = tid; o < d.groups * (MT * 256); o += NW * 64) {
        const uint32_t g = o / (MT * 256), oo = o % (MT * 256);
        const uint32_t mt = oo >> 8, l = (oo >> 2) & 63, r = oo & 3;
        if (j0 + g >= count) break;                     // the sequence ended inside this unit
        float sum = 0.f;
        for (uint32_t w = g * d.wpb; w < (g + 1) * d.wpb; w++) sum += ((const float *)&red[(w * MT + mt) * 64 + l])[r];
        const uint32_t m = 16 * mt + 4 * (l >> 4) + r;
        if (m < a.M) {
            if (SCALED && a.d_xs && a.xs_cols == 1) sum *= ((const GLOBAL float *)a.d_xs)[m];
            Y[(uint64_t)m * a.rows + (first + (j0 + g) * stride) * BLOCK_ROWS + (l & 15)] = sum;
        }
    }
}

// Split K: the partial sums of the unit (block of rows, slice of K) go to the workspace, and the
// workgroup that brings a block's last slice adds the slices up -- in slice order, so the result
// does not depend on which one that was -- and writes the outputs.  No workgroup waits for
// another; the last one leaves the counter at zero for the next call.
// Memory order.  Every thread writes its partial sums, the workgroup meets at a barrier, and ONE thread
// adds to the block's arrival counter with release and acquire order at agent scope: the barrier orders the
// other threads' stores before that add (release side) and the add before the other threads' loads in
// the workgroup that turns out to be last (acquire side), so the last workgroup's reads of the other
// slices are ordered after their writes by the memory model itself.  The agent-scope release / acquire
// writes back and invalidates caches once per workgroup (measured: about 2 us per launch).  Partial
// sums move through agent-scope atomic stores and loads, so they are never served from or left in a
// cache private to a part of the chip; each wave also waits for its own stores before the barrier.
template <int MT, int NW, bool SCALED>
__device__ __forceinline__ void reduce_split(f32x4 *red, uint32_t *s_flag, const GArgs &a, uint32_t block, uint32_t slice,
                                             int tid, const f32x4 (&acc)[MT])
{
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int mt = 0; mt < MT; mt++) red[(wave * MT + mt) * 64 + lane] = acc[mt];
    __syncthreads();
    GLOBAL uint32_t *part = (GLOBAL uint32_t *)a.d_part + (uint64_t)block * a.slices * (MT * 256);
    GLOBAL uint32_t *ctr = (GLOBAL uint32_t *)a.d_ctr + block;
    for (int o = tid; o < MT * 256; o += NW * 64) {
        const int mt = o >> 8, l = (o >> 2) & 63, r = o & 3;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < NW; w++) sum += ((const float *)&red[(w * MT + mt) * 64 + l])[r];
        __hip_atomic_store(part + (uint64_t)slice * (MT * 256) + o, __float_as_uint(sum), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this wave's stores have completed ...
    __syncthreads();                                        // ... and so have every wave's
    if (tid == 0) *s_flag = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (*s_flag != a.slices - 1) return;          // uniform: the same LDS word for every thread
    GLOBAL float *Y = (GLOBAL float *)a.d_y;
    for (int o = tid; o < MT * 256; o += NW * 64) {
        const int mt = o >> 8, l = (o >> 2) & 63, r = o & 3;
        float sum = 0.f;
        for (uint32_t sl = 0; sl < a.slices; sl++)
            sum += __uint_as_float(__hip_atomic_load(part + (uint64_t)sl * (MT * 256) + o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        const uint32_t m = 16 * mt + 4 * (l >> 4) + r;
        if (m < a.M) {
            if (SCALED && a.d_xs && a.xs_cols == 1) sum *= ((const GLOBAL float *)a.d_xs)[m];
            Y[(uint64_t)m * a.rows + (uint64_t)block * BLOCK_ROWS + (l & 15)] = sum;
        }
    }
    if (tid == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int MT, int NW, int N, int SC, int ACC = 0>       // SC: 0 no scales, 1 scales of W (and one per row of X), 2 also one per row and 128 columns of X; ACC: see ECF8_MFMA_OPERANDS
__global__ __launch_bounds__(NW * 64) void ecf8_gemm_kernel(GArgs a)
{
    constexpr bool SCALED = SC != 0;
    static_assert(!SCALED || 4 * N == 2 * SCALE_BLOCK, "a chunk spans two scale blocks of K");
    using C = GCfg<MT, NW, N>;
    constexpr int KPW = C::KPW, KCHUNKS = C::KCHUNKS, BLOCK_COLS = C::BLOCK_COLS;
    constexpr int GPIECES = C::PIECES, GSTAGE = C::STAGE, GSEGS = C::SEGS;
    __shared__ __attribute__((aligned(16))) uint8_t smem[C::TOTAL];
    uint16_t *tbl = (uint16_t *)(smem + C::OFF_TBL);
    uint32_t *s_len = (uint32_t *)(smem + C::OFF_SYM);
    uint32_t *s_code = s_len + 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t stage_off = C::OFF_STAGE + wave * GSTAGE;
    uint8_t *stage = smem + stage_off;

    const GLOBAL uint64_t *chunk_bit = (const GLOBAL uint64_t *)(a.d_blob + a.off_cb);
    const GLOBAL uint16_t *lane_bits = (const GLOBAL uint16_t *)(a.d_blob + a.off_lb);
    const GLOBAL uint8_t *stream = (const GLOBAL uint8_t *)(a.d_blob + a.off_st);
    const GLOBAL uint8_t *plane = (const GLOBAL uint8_t *)(a.d_blob + a.off_pl);
    // this lane's piece 0 inside a chunk: row l % 16, column 16 (l / 16) of the block
    const uint64_t lane_elem = (uint64_t)(lane & 15) * GK + (uint64_t)(lane >> 4) * 16;

    struct Meta { uint64_t b0, b1; uint32_t lb; };
    const uint64_t n_blocks = a.rows / BLOCK_ROWS;
    const uint32_t wave_s = uniform32((uint32_t)wave);             // the same for every lane: chunk addresses stay in scalar registers
    // the wave's chunks in the order it meets them: step s = its (s % KPW)-th chunk of its (s / KPW)-th block
    auto block_of = [&](uint64_t s) -> uint64_t { return blockIdx.x + (s / KPW) * (uint64_t)gridDim.x; };
    auto kc_of = [&](uint64_t s) -> uint32_t { return wave_s + NW * (uint32_t)(s % KPW); };
    auto load_meta = [&](uint64_t s) {
        const uint64_t c = block_of(s) * KCHUNKS + kc_of(s);
        Meta m;
        m.b0 = chunk_bit[c];
        m.b1 = chunk_bit[c + 1];
        m.lb = lane_bits[c * 64 + lane];
        return m;
    };
    // A chunk's span of the stream (16-byte aligned start, 8 bytes of look-ahead), from the chunk's two start
    // bits: values every lane holds alike, so the arithmetic is done once, in scalar registers.
    auto span_of = [&](const Meta &m, uint64_t &byte0) {
        const uint64_t b0 = uniform64(m.b0), b1 = uniform64(m.b1);
        uint64_t byte_end = ((b1 + 7) >> 3) + 8;
        if (byte_end > a.st_bytes) byte_end = a.st_bytes;
        byte0 = (b0 >> 3) & ~15ull;
        if (byte0 > byte_end) byte0 = byte_end;
        return byte_end - byte0;
    };
    // The span's 16-byte units into `seg` (unit lane + 64 k into seg[k]); units beyond the span keep what they
    // held: the lanes' codewords never reach into them.
    const uint32_t lane16 = (uint32_t)lane * 16;
    auto load_stream = [&](const Meta &m, u32x4 (&seg)[GSEGS], bool wanted = true) {
        uint64_t byte0;
        const uint32_t whole = (uint32_t)span_of(m, byte0);         // at most GSTAGE under the cap on codewords
        const uint32_t span = wanted ? whole : 0u;
        const GLOBAL uint8_t *sp = stream + byte0;
#pragma unroll
        for (int k = 0; k < GSEGS; k++) {
            const uint32_t i = lane16 + 1024 * k;
            if (i < (uint32_t)GSTAGE && i < span) seg[k] = __builtin_nontemporal_load((const GLOBAL u32x4 *)(sp + i));
        }
    };
    // nibble plane of step s: piece q of this lane at plane_of(s) + lane_plane + 32 q
    const uint32_t lane_plane = (uint32_t)(lane_elem / 2);
    auto plane_of = [&](uint64_t s) -> const GLOBAL uint8_t * {
        return plane + (block_of(s) * BLOCK_ROWS * (uint64_t)GK + kc_of(s) * (uint64_t)BLOCK_COLS) / 2;
    };

    // start-up: the first chunks' loads and those of X are in flight while the table is set up
    const uint64_t n_steps = blockIdx.x < n_blocks ? ((n_blocks - blockIdx.x + gridDim.x - 1) / gridDim.x) * KPW : 0;
    Meta m_cur{0, 0, 0}, m_next{0, 0, 0};
    u32x4 seg[GSEGS];
    u32x2 pl[GPIECES];
#pragma unroll
    for (int k = 0; k < GSEGS; k++) seg[k] = u32x4{0, 0, 0, 0};
#pragma unroll
    for (int q = 0; q < GPIECES; q++) pl[q] = u32x2{0, 0};
    if (n_steps > 0) {
        m_cur = load_meta(0);
        m_next = load_meta(n_steps > 1 ? 1 : 0);
        load_stream(m_cur, seg);
        const GLOBAL uint8_t *pp = plane_of(0);
#pragma unroll
        for (int q = 0; q < GPIECES; q++) pl[q] = __builtin_nontemporal_load((const GLOBAL u32x2 *)(pp + lane_plane + 32 * q));
    }

    u32x4 areg[MT][KPW][GPIECES];
    load_x_slice<MT, NW, N>(a, tid, areg);

    uint64_t len_lo, len_hi;
    __builtin_memcpy(&len_lo, a.code_len, 8);
    __builtin_memcpy(&len_hi, a.code_len + 8, 8);
    if (a.off_tbl) {
        const GLOBAL u32x4 *src = (const GLOBAL u32x4 *)(a.d_blob + a.off_tbl);
        for (int i = tid; i < TBL_ENTRIES * 2 / 16; i += NW * 64) ((u32x4 *)tbl)[i] = src[i];
        build_symbol_arrays(len_lo, len_hi, s_len, s_code, tid);
        __syncthreads();
    } else {
        build_tables(len_lo, len_hi, tbl, s_len, s_code, (uint16_t *)(smem + C::OFF_STAGE), tid, NW * 64);
    }

    uint32_t parity = 0;
    for (uint64_t s0 = 0; s0 < n_steps; s0 += KPW) {
        f32x4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; mt++) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < KPW; i++) {
            const uint64_t s = s0 + i;
            const Meta m = m_cur;
            uint64_t byte0;
            span_of(m, byte0);
            const uint32_t rel = wave_incl_scan(m.lb) - m.lb;
            const uint64_t start = uniform64(m.b0);
#pragma unroll
            for (int k = 0; k < GSEGS; k++) {
                const uint32_t j = lane16 + 1024 * k;
                if (j < (uint32_t)GSTAGE) *(u32x4 *)(stage + j) = seg[k];
            }
            // The stream registers are free: fetch the next chunk's span, and the metadata of the chunk after it.
            // The last steps have nothing to fetch and no branch around the loads either: the metadata of the last
            // chunk again (12 bytes), a span of no bytes, and the plane's first chunk, which every wave then asks for.
            const bool more = s + 1 < n_steps;                 // the same for every lane
            const uint64_t sn = more ? s + 1 : s, sn2 = s + 2 < n_steps ? s + 2 : sn;
            load_stream(m_next, seg, more);
            const Meta m_next2 = load_meta(sn2);
            const GLOBAL uint8_t *pp = more ? plane_of(sn) : plane;
            const uint32_t bpA = stage_off * 8 + (uint32_t)(start - byte0 * 8) + rel - 1;   // one bit off, see quad_step2
            HeldRuns runs;
            runs.begin(smem, bpA, bpA + m.lb - 30);
            ChunkSums<MT, SC> sums;
            sums.begin(a, block_of(s), kc_of(s));
            auto &dstA = sums.first(acc);
            auto &dstB = sums.second(acc);
#pragma unroll
            for (int Q = 0; Q < GPIECES / 2; Q++) {
                uint32_t dwA[4], dwB[4];
#pragma unroll
                for (int t = 0; t < 4; t++) quad_step_held(smem, tbl, runs, dwA[t], dwB[t]);
                // a piece of the nibble plane is merged, and its registers take the same piece of the next chunk
                const u32x4 wA = merge_piece(dwA, pl[Q]);
                pl[Q] = __builtin_nontemporal_load((const GLOBAL u32x2 *)(pp + lane_plane + 32 * Q));
                ECF8_MFMA_PIECE(dstA, areg, i, Q, wA);
                const u32x4 wB = merge_piece(dwB, pl[Q + GPIECES / 2]);
                pl[Q + GPIECES / 2] = __builtin_nontemporal_load((const GLOBAL u32x2 *)(pp + lane_plane + 32 * (Q + GPIECES / 2)));
                ECF8_MFMA_PIECE(dstB, areg, i, Q + GPIECES / 2, wB);
            }
            sums.end(acc, a, lane);
            m_cur = m_next;
            m_next = m_next2;
        }
        if constexpr (C::BPB == 1) {
            reduce_block<MT, NW, SCALED>((f32x4 *)(smem + C::OFF_RED + parity * C::RED_BYTES), a, block_of(s0), tid, acc);
            parity ^= 1;
        } else {
            // park this block's partial sums; the workgroup meets after every BPB-th block and after the last one
            f32x4 *red = (f32x4 *)(smem + C::OFF_RED);
            const uint32_t j = (uint32_t)((s0 / KPW) % C::BPB);
            red[(j * NW + wave_s) * 64 + lane] = acc[0];
            const bool last = s0 + KPW >= n_steps;           // the same for the whole workgroup
            if (j == C::BPB - 1 || last) {
                __syncthreads();
                reduce_parked<NW, SCALED>(red, a, block_of(s0 - j * KPW), gridDim.x, j + 1, tid);
                if (!last) __syncthreads();                  // the buffers are free again
            }
        }
    }
}

// The same GEMM on uncompressed row-major W, with the fused kernel's workgroup shape, K split
// and order of accumulation, so that the two agree bit for bit.
template <int MT, int NW, int N, int SC, int ACC = 0>
__global__ __launch_bounds__(NW * 64) void ecf8_gemm_raw_kernel(GArgs a)
{
    constexpr bool SCALED = SC != 0;
    using C = GCfg<MT, NW, N>;
    constexpr int KPW = C::KPW, BLOCK_COLS = C::BLOCK_COLS, GPIECES = C::PIECES;
    __shared__ __attribute__((aligned(16))) uint8_t smem[C::RED_BUFS * C::RED_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const GLOBAL uint8_t *W = (const GLOBAL uint8_t *)a.d_w;
    const uint64_t lane_elem = (uint64_t)(lane & 15) * GK + (uint64_t)(lane >> 4) * 16;
    const uint64_t n_blocks = a.rows / BLOCK_ROWS;
    const uint64_t n_steps = blockIdx.x < n_blocks ? ((n_blocks - blockIdx.x + gridDim.x - 1) / gridDim.x) * KPW : 0;
    auto block_of = [&](uint64_t s) -> uint64_t { return blockIdx.x + (s / KPW) * (uint64_t)gridDim.x; };
    auto load_w = [&](uint64_t s, u32x4 (&w)[GPIECES]) {
        const uint64_t e0 = block_of(s) * BLOCK_ROWS * (uint64_t)GK + (wave + NW * (uint32_t)(s % KPW)) * (uint64_t)BLOCK_COLS + lane_elem;
#pragma unroll
        for (int q = 0; q < GPIECES; q++) w[q] = __builtin_nontemporal_load((const GLOBAL u32x4 *)(W + e0 + 64 * q));
    };
    u32x4 w_cur[GPIECES], w_next[GPIECES];
    if (n_steps > 0) load_w(0, w_cur);
    u32x4 areg[MT][KPW][GPIECES];
    load_x_slice<MT, NW, N>(a, tid, areg);
    uint32_t parity = 0;
    for (uint64_t s0 = 0; s0 < n_steps; s0 += KPW) {
        f32x4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; mt++) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < KPW; i++) {
            const uint64_t s = s0 + i;
#pragma unroll
            for (int q = 0; q < GPIECES; q++) w_next[q] = w_cur[q];
            if (s + 1 < n_steps) load_w(s + 1, w_next);
            ChunkSums<MT, SC> sums;
            sums.begin(a, block_of(s), wave + NW * (uint32_t)(s % KPW));
            auto &dstA = sums.first(acc);
            auto &dstB = sums.second(acc);
#pragma unroll
            for (int Q = 0; Q < GPIECES / 2; Q++) {
                ECF8_MFMA_PIECE(dstA, areg, i, Q, w_cur[Q]);
                ECF8_MFMA_PIECE(dstB, areg, i, Q + GPIECES / 2, w_cur[Q + GPIECES / 2]);
            }
            sums.end(acc, a, lane);
#pragma unroll
            for (int q = 0; q < GPIECES; q++) w_cur[q] = w_next[q];
        }
        if constexpr (C::BPB == 1) {
            reduce_block<MT, NW, SCALED>((f32x4 *)(smem + parity * C::RED_BYTES), a, block_of(s0), tid, acc);
            parity ^= 1;
        } else {
            f32x4 *red = (f32x4 *)smem;                      // as in the fused kernel
            const uint32_t j = (uint32_t)((s0 / KPW) % C::BPB);
            red[(j * NW + wave) * 64 + lane] = acc[0];
            const bool last = s0 + KPW >= n_steps;
            if (j == C::BPB - 1 || last) {
                __syncthreads();
                reduce_parked<NW, SCALED>(red, a, block_of(s0 - j * KPW), gridDim.x, j + 1, tid);
                if (!last) __syncthreads();
            }
        }
    }
}

// ---- any K (a multiple of 256) ----
// The kernels above keep the wave's slice of X in registers, which is what makes K = 4096 fast
// and what ties them to it.  These take any K: the K / 256 chunks of a block of rows are dealt
// round-robin to the NW waves (some waves get one chunk fewer; where a block has at most NW / 2
// chunks the waves split into groups with a block each, see Deal), and
// the A operands of a chunk are fetched from X (L2-resident: M x K bytes) one chunk ahead, like
// the chunk's payload.  Same decode, same MFMA order inside a chunk, same reduction.

template <int MT, int N>
struct XPieces { u32x4 v[MT][N / 16]; };

// A operands for chunk kc: X[m][256 kc + 64 q + 16 g .. + 16) of lane (m = l % 16 (+ 16 mt), g = l / 16)
template <int MT, int N>
__device__ __forceinline__ void load_x_chunk(const GArgs &a, int lane, uint32_t kc, XPieces<MT, N> &x)
{
    const GLOBAL uint8_t *X = (const GLOBAL uint8_t *)a.d_x;
    const int n = lane & 15, g = lane >> 4;
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int q = 0; q < N / 16; q++) {
            const uint32_t m = 16 * mt + n;
            x.v[mt][q] = u32x4{0, 0, 0, 0};
            if (m < a.M) x.v[mt][q] = *(const GLOBAL u32x4 *)(X + (uint64_t)m * a.K + (uint64_t)kc * (4 * N) + 64 * q + 16 * g);
        }
}

#define ECF8_MFMA_XPIECE(acc, xp, p, W_PIECE) ECF8_MFMA_OPERANDS(acc, xp.v[mt_][p], W_PIECE)

// Position of a wave in its sequence of chunks: its i-th chunk of its workgroup's b-th unit.  A unit
// is a block of 16 rows of W, or with split K one of the `slices` equal parts of its chunks: `block`
// is the unit's block of rows, k0 its first chunk.
struct Walk {
    uint64_t b;
    uint32_t i;
    uint64_t block;
    uint32_t k0;
};

// The work of one workgroup on one matrix: its units first_unit, first_unit + unit_stride, ... (my_units
// of them), table set-up included.  `parity` says which of the two reduction buffers comes next and is
// carried on to the caller's next matrix.
template <int MT, int NW, int N, int SC, bool SPLIT, int ACC = 0>
__device__ __forceinline__ void anyk_walk(const GArgs &a, uint8_t *smem, uint32_t *s_flag, uint64_t first_unit, uint64_t unit_stride,
                                          uint64_t my_units, uint32_t &parity)
{
    constexpr bool SCALED = SC != 0;
    using C = GCfg<MT, NW, N>;
    constexpr int BLOCK_COLS = C::BLOCK_COLS, GPIECES = C::PIECES, GSTAGE = C::STAGE, GSEGS = C::SEGS;
    static_assert(!SCALED || 4 * N == 2 * SCALE_BLOCK, "a chunk spans two scale blocks of K");
    uint16_t *tbl = (uint16_t *)(smem + C::OFF_TBL);
    uint32_t *s_len = (uint32_t *)(smem + C::OFF_SYM);
    uint32_t *s_code = s_len + 16;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = (int)uniform32((uint32_t)tid >> 6);           // the same for every lane: what follows from it stays in scalar registers
    const uint32_t stage_off = C::OFF_STAGE + wave * GSTAGE;
    uint8_t *stage = smem + stage_off;

    const GLOBAL uint64_t *chunk_bit = (const GLOBAL uint64_t *)(a.d_blob + a.off_cb);
    const GLOBAL uint16_t *lane_bits = (const GLOBAL uint16_t *)(a.d_blob + a.off_lb);
    const GLOBAL uint8_t *stream = (const GLOBAL uint8_t *)(a.d_blob + a.off_st);
    const GLOBAL uint8_t *plane = (const GLOBAL uint8_t *)(a.d_blob + a.off_pl);
    const uint64_t lane_elem = (uint64_t)(lane & 15) * a.K + (uint64_t)(lane >> 4) * 16;
    const uint32_t kchunks = (uint32_t)(a.K / BLOCK_COLS);
    const uint32_t unit_chunks = SPLIT ? kchunks / a.slices : kchunks;                                     // chunks of K per unit
    const Deal deal = deal_chunks<NW>(unit_chunks, SPLIT, wave);
    const uint32_t my_chunks = deal.my_chunks;                                                             // wave-uniform
    const uint64_t my_blocks = (my_units + deal.groups - 1) / deal.groups;                                 // units of `groups` blocks

    struct Meta { uint64_t b0, b1; uint32_t lb; };
    auto at_unit = [&](uint64_t b) {
        Walk w{b, 0, first_unit + (b * deal.groups + deal.gi) * unit_stride, 0};
        if constexpr (SPLIT) {
            const uint32_t u = (uint32_t)w.block;            // units < 2^31, checked on the host
            w.block = u / a.slices;
            w.k0 = (u % a.slices) * unit_chunks;
        }
        return w;
    };
    auto block_of = [&](const Walk &w) -> uint64_t { return w.block; };
    auto kc_of = [&](const Walk &w) -> uint32_t { return w.k0 + deal.kw + deal.wpb * w.i; };
    auto valid = [&](const Walk &w) { return my_chunks != 0 && w.b * deal.groups + deal.gi < my_units; };
    auto next_of = [&](Walk w) { if (++w.i == my_chunks) w = at_unit(w.b + 1); return w; };
    auto load_meta = [&](const Walk &w) {
        const uint64_t c = block_of(w) * kchunks + kc_of(w);
        Meta m;
        m.b0 = chunk_bit[c];
        m.b1 = chunk_bit[c + 1];
        m.lb = lane_bits[c * 64 + lane];
        return m;
    };
    // A chunk's span of the stream (16-byte aligned start, 8 bytes of look-ahead), from the chunk's two start
    // bits: values every lane holds alike, so the arithmetic is done once, in scalar registers.
    auto span_of = [&](const Meta &m, uint64_t &byte0) {
        const uint64_t b0 = uniform64(m.b0), b1 = uniform64(m.b1);
        uint64_t byte_end = ((b1 + 7) >> 3) + 8;
        if (byte_end > a.st_bytes) byte_end = a.st_bytes;
        byte0 = (b0 >> 3) & ~15ull;
        if (byte0 > byte_end) byte0 = byte_end;
        return byte_end - byte0;
    };
    // The span's 16-byte units into `seg` (unit lane + 64 k into seg[k]); units beyond the span keep what they
    // held: the lanes' codewords never reach into them.
    const uint32_t lane16 = (uint32_t)lane * 16;
    auto load_stream = [&](const Meta &m, u32x4 (&seg)[GSEGS], bool wanted = true) {
        uint64_t byte0;
        const uint32_t whole = (uint32_t)span_of(m, byte0);         // at most GSTAGE under the cap on codewords
        const uint32_t span = wanted ? whole : 0u;
        const GLOBAL uint8_t *sp = stream + byte0;
#pragma unroll
        for (int k = 0; k < GSEGS; k++) {
            const uint32_t i = lane16 + 1024 * k;
            if (i < (uint32_t)GSTAGE && i < span) seg[k] = __builtin_nontemporal_load((const GLOBAL u32x4 *)(sp + i));
        }
    };
    // nibble plane of a chunk: piece q of this lane at plane_of(w) + lane_plane + 32 q
    const uint64_t lane_plane = lane_elem / 2;
    auto plane_of = [&](const Walk &w) -> const GLOBAL uint8_t * {
        return plane + (block_of(w) * BLOCK_ROWS * a.K + kc_of(w) * (uint64_t)BLOCK_COLS) / 2;
    };

    Walk cur = at_unit(0);
    Meta m_cur{0, 0, 0}, m_next{0, 0, 0};
    u32x4 seg[GSEGS];
    u32x2 pl[GPIECES];
#pragma unroll
    for (int k = 0; k < GSEGS; k++) seg[k] = u32x4{0, 0, 0, 0};
#pragma unroll
    for (int q = 0; q < GPIECES; q++) pl[q] = u32x2{0, 0};
    XPieces<MT, N> x_cur;
    if (valid(cur)) {
        m_cur = load_meta(cur);
        m_next = m_cur;
        if (valid(next_of(cur))) m_next = load_meta(next_of(cur));
        load_stream(m_cur, seg);
        const GLOBAL uint8_t *pp = plane_of(cur) + lane_plane;
#pragma unroll
        for (int q = 0; q < GPIECES; q++) pl[q] = __builtin_nontemporal_load((const GLOBAL u32x2 *)(pp + 32 * q));
        load_x_chunk<MT, N>(a, lane, kc_of(cur), x_cur);
    }

    uint64_t len_lo, len_hi;
    __builtin_memcpy(&len_lo, a.code_len, 8);
    __builtin_memcpy(&len_hi, a.code_len + 8, 8);
    if (a.off_tbl) {
        const GLOBAL u32x4 *src = (const GLOBAL u32x4 *)(a.d_blob + a.off_tbl);
        for (int i = tid; i < TBL_ENTRIES * 2 / 16; i += NW * 64) ((u32x4 *)tbl)[i] = src[i];
        build_symbol_arrays(len_lo, len_hi, s_len, s_code, tid);
        __syncthreads();
    } else {
        build_tables(len_lo, len_hi, tbl, s_len, s_code, (uint16_t *)(smem + C::OFF_STAGE), tid, NW * 64);
    }

    for (uint64_t b = 0; b < my_blocks; b++) {            // uniform for the workgroup: one barrier per block
        f32x4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; mt++) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        const uint32_t n_mine = valid(at_unit(b)) ? my_chunks : 0;       // the sequence may end inside the last unit
#pragma unroll 1
        for (uint32_t i = 0; i < n_mine; i++) {
            const Meta m = m_cur;
            uint64_t byte0;
            span_of(m, byte0);
            const uint32_t rel = wave_incl_scan(m.lb) - m.lb;
            const uint64_t start = uniform64(m.b0);
#pragma unroll
            for (int k = 0; k < GSEGS; k++) {
                const uint32_t j = lane16 + 1024 * k;
                if (j < (uint32_t)GSTAGE) *(u32x4 *)(stage + j) = seg[k];
            }
            const XPieces<MT, N> x = x_cur;
            ChunkSums<MT, SC> sums;
            sums.begin(a, block_of(cur), kc_of(cur));
            // The stream registers are free: fetch the next chunk's span and its share of X, and the metadata of the
            // chunk after it.
            const Walk nxt = next_of(cur);
            const bool more = valid(nxt);
            Meta m_next2 = m_next;
            if (more) {
                load_stream(m_next, seg);
                load_x_chunk<MT, N>(a, lane, kc_of(nxt), x_cur);
                if (valid(next_of(nxt))) m_next2 = load_meta(next_of(nxt));
            }
            // after the last chunk the plane pieces are fetched from the plane's first chunk (every wave's last fetch: cached)
            const GLOBAL uint8_t *pp = (more ? plane_of(nxt) : plane) + lane_plane;
            const uint32_t bpA = stage_off * 8 + (uint32_t)(start - byte0 * 8) + rel - 1;   // one bit off, see quad_step2
            HeldRuns runs;
            runs.begin(smem, bpA, bpA + m.lb - 30);
            auto &dstA = sums.first(acc);
            auto &dstB = sums.second(acc);
#pragma unroll
            for (int Q = 0; Q < GPIECES / 2; Q++) {
                uint32_t dwA[4], dwB[4];
#pragma unroll
                for (int t = 0; t < 4; t++) quad_step_held(smem, tbl, runs, dwA[t], dwB[t]);
                // a piece of the nibble plane is merged, and its registers take the same piece of the next chunk
                const u32x4 wA = merge_piece(dwA, pl[Q]);
                pl[Q] = __builtin_nontemporal_load((const GLOBAL u32x2 *)(pp + 32 * Q));
                ECF8_MFMA_XPIECE(dstA, x, Q, wA);
                const u32x4 wB = merge_piece(dwB, pl[Q + GPIECES / 2]);
                pl[Q + GPIECES / 2] = __builtin_nontemporal_load((const GLOBAL u32x2 *)(pp + 32 * (Q + GPIECES / 2)));
                ECF8_MFMA_XPIECE(dstB, x, Q + GPIECES / 2, wB);
            }
            sums.end(acc, a, lane);
            cur = nxt;
            m_cur = m_next;
            m_next = m_next2;
        }
        f32x4 *red = (f32x4 *)(smem + C::OFF_RED + parity * C::RED_BYTES);
        const Walk unit = at_unit(b);
        if constexpr (SPLIT) reduce_split<MT, NW, SCALED>(red, s_flag, a, (uint32_t)unit.block, unit.k0 / unit_chunks, tid, acc);
        else reduce_groups<MT, NW, SCALED>(red, a, first_unit, unit_stride, b * deal.groups, my_units, deal, tid, acc);
        parity ^= 1;
    }
}

// units of workgroup blockIdx.x when n_units are dealt round-robin to the grid
__device__ __forceinline__ uint64_t units_of_workgroup(uint64_t n_units)
{
    return blockIdx.x < n_units ? (n_units - blockIdx.x + gridDim.x - 1) / gridDim.x : 0;
}

template <int MT, int NW, int N, int SC, bool SPLIT = false, int ACC = 0>
__global__ __launch_bounds__(NW * 64) void ecf8_gemm_anyk_kernel(GArgs a)
{
    __shared__ __attribute__((aligned(16))) uint8_t smem[GCfg<MT, NW, N>::TOTAL];
    __shared__ uint32_t s_flag;                   // split K: the arrival count this workgroup drew
    uint32_t parity = 0;
    anyk_walk<MT, NW, N, SC, SPLIT, ACC>(a, smem, &s_flag, blockIdx.x, gridDim.x,
                                    units_of_workgroup(a.rows / BLOCK_ROWS * (SPLIT ? a.slices : 1u)), parity);
}

// The any-K GEMM on uncompressed W: same deal of chunks, same order of accumulation.
template <int MT, int NW, int N, int SC, bool SPLIT, int ACC = 0>
__device__ __forceinline__ void raw_anyk_walk(const GArgs &a, uint8_t *smem, uint32_t *s_flag, uint64_t first_unit, uint64_t unit_stride,
                                              uint64_t my_units, uint32_t &parity)
{
    constexpr bool SCALED = SC != 0;
    using C = GCfg<MT, NW, N>;
    constexpr int BLOCK_COLS = C::BLOCK_COLS, GPIECES = C::PIECES;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const GLOBAL uint8_t *W = (const GLOBAL uint8_t *)a.d_w;
    const uint64_t lane_elem = (uint64_t)(lane & 15) * a.K + (uint64_t)(lane >> 4) * 16;
    const uint32_t kchunks = (uint32_t)(a.K / BLOCK_COLS);
    const uint32_t unit_chunks = SPLIT ? kchunks / a.slices : kchunks;
    const Deal deal = deal_chunks<NW>(unit_chunks, SPLIT, wave);
    const uint32_t my_chunks = deal.my_chunks;
    const uint64_t my_blocks = (my_units + deal.groups - 1) / deal.groups;
    auto at_unit = [&](uint64_t b) {
        Walk w{b, 0, first_unit + (b * deal.groups + deal.gi) * unit_stride, 0};
        if constexpr (SPLIT) {
            const uint32_t u = (uint32_t)w.block;
            w.block = u / a.slices;
            w.k0 = (u % a.slices) * unit_chunks;
        }
        return w;
    };
    auto block_of = [&](const Walk &w) -> uint64_t { return w.block; };
    auto kc_of = [&](const Walk &w) -> uint32_t { return w.k0 + deal.kw + deal.wpb * w.i; };
    auto valid = [&](const Walk &w) { return my_chunks != 0 && w.b * deal.groups + deal.gi < my_units; };
    auto next_of = [&](Walk w) { if (++w.i == my_chunks) w = at_unit(w.b + 1); return w; };
    auto load_w = [&](const Walk &w, u32x4 (&v)[GPIECES]) {
        const uint64_t e0 = block_of(w) * BLOCK_ROWS * a.K + kc_of(w) * (uint64_t)BLOCK_COLS + lane_elem;
#pragma unroll
        for (int q = 0; q < GPIECES; q++) v[q] = __builtin_nontemporal_load((const GLOBAL u32x4 *)(W + e0 + 64 * q));
    };
    Walk cur = at_unit(0);
    u32x4 w_cur[GPIECES], w_next[GPIECES];
    XPieces<MT, N> x_cur;
    if (valid(cur)) {
        load_w(cur, w_cur);
        load_x_chunk<MT, N>(a, lane, kc_of(cur), x_cur);
    }
    for (uint64_t b = 0; b < my_blocks; b++) {
        f32x4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; mt++) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        const uint32_t n_mine = valid(at_unit(b)) ? my_chunks : 0;
#pragma unroll 1
        for (uint32_t i = 0; i < n_mine; i++) {
            const XPieces<MT, N> x = x_cur;
            ChunkSums<MT, SC> sums;
            sums.begin(a, block_of(cur), kc_of(cur));
            const Walk nxt = next_of(cur);
#pragma unroll
            for (int q = 0; q < GPIECES; q++) w_next[q] = w_cur[q];
            if (valid(nxt)) {
                load_w(nxt, w_next);
                load_x_chunk<MT, N>(a, lane, kc_of(nxt), x_cur);
            }
            auto &dstA = sums.first(acc);
            auto &dstB = sums.second(acc);
#pragma unroll
            for (int Q = 0; Q < GPIECES / 2; Q++) {
                ECF8_MFMA_XPIECE(dstA, x, Q, w_cur[Q]);
                ECF8_MFMA_XPIECE(dstB, x, Q + GPIECES / 2, w_cur[Q + GPIECES / 2]);
            }
            sums.end(acc, a, lane);
#pragma unroll
            for (int q = 0; q < GPIECES; q++) w_cur[q] = w_next[q];
            cur = nxt;
        }
        f32x4 *red = (f32x4 *)(smem + parity * C::RED_BYTES);
        const Walk unit = at_unit(b);
        if constexpr (SPLIT) reduce_split<MT, NW, SCALED>(red, s_flag, a, (uint32_t)unit.block, unit.k0 / unit_chunks, tid, acc);
        else reduce_groups<MT, NW, SCALED>(red, a, first_unit, unit_stride, b * deal.groups, my_units, deal, tid, acc);
        parity ^= 1;
    }
}

template <int MT, int NW, int N, int SC, bool SPLIT = false, int ACC = 0>
__global__ __launch_bounds__(NW * 64) void ecf8_gemm_raw_anyk_kernel(GArgs a)
{
    __shared__ __attribute__((aligned(16))) uint8_t smem[2 * GCfg<MT, NW, N>::RED_BYTES];
    __shared__ uint32_t s_flag;
    uint32_t parity = 0;
    raw_anyk_walk<MT, NW, N, SC, SPLIT, ACC>(a, smem, &s_flag, blockIdx.x, gridDim.x,
                                        units_of_workgroup(a.rows / BLOCK_ROWS * (SPLIT ? a.slices : 1u)), parity);
}

// ---- a group of matrices in one launch ----
// Many small products at once, each with its own W, X, M and Y (the experts a batch of tokens is
// routed to): a launch per matrix would be bound by launches and would leave the chip half empty
// (a 2048 x 7168 expert has 128 blocks of rows).  The blocks of all matrices form one sequence,
// weighted by their K / 256 chunks; every workgroup takes an equal share of it, a contiguous run
// of blocks that may cross from one matrix into the next, and works through it with the any-K loop,
// setting up the code again where the matrix changes.  Inside a block nothing differs from the
// single call with the same number of waves, so the results are the same bit for bit.
struct GItem {
    uint64_t first_work;        // chunks of the matrices before this one
    GArgs a;
};
static_assert(sizeof(GItem) % 8 == 0 && sizeof(GItem) <= sizeof(ecf8_gemm_group_item), "item fits its public slot");

struct GGArgs {
    uint64_t d_items;           // device array of ecf8_gemm_group_item
    uint32_t n_items;
    uint64_t total_work;
};

template <int MT, int NW, int N, int SC, bool RAW>
__global__ __launch_bounds__(NW * 64) void ecf8_gemm_grouped_kernel(GGArgs g)
{
    using C = GCfg<MT, NW, N>;
    __shared__ __attribute__((aligned(16))) uint8_t smem[RAW ? 2 * C::RED_BYTES : C::TOTAL];
    __shared__ uint32_t s_flag;
    constexpr uint32_t WORDS = sizeof(ecf8_gemm_group_item) / 8;
    const GLOBAL uint64_t *items = (const GLOBAL uint64_t *)g.d_items;
    // this workgroup takes the blocks whose first chunk lies in [pos, end) of the sequence
    uint64_t pos = g.total_work * blockIdx.x / gridDim.x;
    const uint64_t end = g.total_work * (blockIdx.x + 1) / gridDim.x;
    uint32_t parity = 0;
    while (pos < end) {                                 // one round per matrix the share touches (uniform)
        uint32_t lo = 0, hi = g.n_items - 1;
        while (lo < hi) {
            const uint32_t mid = (lo + hi + 1) >> 1;
            if (uniform64(items[(uint64_t)mid * WORDS]) <= pos) lo = mid; else hi = mid - 1;
        }
        GItem it;
        {
            uint64_t *dst = (uint64_t *)&it;
#pragma unroll
            for (int i = 0; i < (int)(sizeof(GItem) / 8); i++) dst[i] = uniform64(items[(uint64_t)lo * WORDS + i]);
        }
        const uint64_t kchunks = it.a.K / C::BLOCK_COLS, n_blocks = it.a.rows / BLOCK_ROWS;
        const uint64_t b0 = (pos - it.first_work + kchunks - 1) / kchunks;
        uint64_t b1 = (end - it.first_work + kchunks - 1) / kchunks;
        if (b1 > n_blocks) b1 = n_blocks;
        __syncthreads();                                // the last matrix's table and reduction buffers are out of use
        if (b0 < b1) {
            if constexpr (RAW) raw_anyk_walk<MT, NW, N, SC, false>(it.a, smem, &s_flag, b0, 1, b1 - b0, parity);
            else anyk_walk<MT, NW, N, SC, false>(it.a, smem, &s_flag, b0, 1, b1 - b0, parity);
        }
        pos = it.first_work + n_blocks * kchunks;       // on to the next matrix (or past `end`)
    }
}

inline int grid_for(uint64_t n_blocks)
{
    int cus = device_cus();
    if (cus <= 0) return -1;
    return (int)(n_blocks < (uint64_t)cus ? n_blocks : (uint64_t)cus);
}

inline int check_gemm_args(uint64_t rows, uint64_t cols, const void *d_x, uint32_t M, const void *d_y)
{
    if (!d_x || !d_y || M == 0 || M > 64) return ECF8_E_ARG;
    if (cols == 0 || cols % 256 || cols > (1u << 20) || rows == 0 || rows % BLOCK_ROWS) return ECF8_E_ARG;
    if (((uintptr_t)d_x & 15) || ((uintptr_t)d_y & 3)) return ECF8_E_ALIGN;
    return ECF8_OK;
}

// Checks of the fused call's blob; fills the kernel arguments.
inline int fused_args(const ecf8_header *h, const void *d_blob, const void *d_x, uint32_t M, float *d_y, GArgs *out)
{
    if (!h || !d_blob) return ECF8_E_ARG;
    if (h->magic != ECF8_MAGIC || h->version != ECF8_VERSION || (h->table_bits != 0 && h->table_bits != ECF8_TB))
        return ECF8_E_FORMAT;
    uint32_t max_len = 0;
    for (int i = 0; i < 16; i++) max_len = h->code_len[i] > max_len ? h->code_len[i] : max_len;
    // row-tiled blob of 16 x 256 chunks, every pair of codewords one table hit
    if (h->lane_syms != 64 || h->tile_rows != BLOCK_ROWS || h->group_chunks != 1 || max_len == 0 ||
        2 * max_len > (uint32_t)TB)
        return ECF8_E_ARG;
    int rc = check_gemm_args(h->rows, h->cols, d_x, M, d_y);
    if (rc) return rc;
    if (h->n_elem != h->rows * h->cols || h->n_chunks != h->n_elem / (64ull * h->lane_syms)) return ECF8_E_FORMAT;
    if (h->off_plane + h->plane_bytes > h->total_size || h->off_stream + h->stream_bytes > h->off_plane ||
        h->plane_bytes != h->n_elem / 2)
        return ECF8_E_FORMAT;
    if ((uintptr_t)d_blob & 15) return ECF8_E_ALIGN;
    GArgs a{};
    a.d_blob = (uint64_t)(uintptr_t)d_blob;
    a.d_x = (uint64_t)(uintptr_t)d_x;
    a.d_y = (uint64_t)(uintptr_t)d_y;
    a.rows = h->rows;
    a.off_cb = h->off_chunk_bit;
    a.off_lb = h->off_lane_bits;
    a.off_st = h->off_stream;
    a.off_pl = h->off_plane;
    a.st_bytes = h->stream_bytes;
    a.off_tbl = h->table_bits ? 256 : 0;
    for (int i = 0; i < 16; i++) a.code_len[i] = h->code_len[i];
    a.M = M;
    a.K = h->cols;
    *out = a;
    return ECF8_OK;
}

inline int raw_args(const void *d_w, uint64_t rows, uint64_t cols, const void *d_x, uint32_t M, float *d_y, GArgs *out)
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
    a.M = M;
    a.K = cols;
    *out = a;
    return ECF8_OK;
}

inline int scale_args(const float *d_w_scale, const float *d_x_scale, uint32_t x_scale_cols, GArgs *a)
{
    if (!d_w_scale) return ECF8_E_ARG;
    if (d_x_scale ? (x_scale_cols != 1 && x_scale_cols != a->K / SCALE_BLOCK) : x_scale_cols != 0) return ECF8_E_ARG;
    a->xs_cols = x_scale_cols;
    if (((uintptr_t)d_w_scale & 3) || ((uintptr_t)d_x_scale & 3)) return ECF8_E_ALIGN;
    a->d_ws = (uint64_t)(uintptr_t)d_w_scale;
    a->d_xs = (uint64_t)(uintptr_t)d_x_scale;
    return ECF8_OK;
}

// 16 waves (one K chunk of the block each) while X fits their registers, 8 waves of two chunks
// at M > 32.  (16 x 512 chunks with 8 waves were measured too: slower, 37.7 us against 25.5.)
template <int SCALED, int ACC = 0>
int launch_fused(const GArgs &a, void *stream)
{
    const int grid = grid_for(a.rows / BLOCK_ROWS);
    if (grid <= 0) return ECF8_E_HIP;
    hipStream_t s = (hipStream_t)stream;
    // any K: X does not stay in registers, fetched chunk by chunk.  Also with a scale per row and 128 columns of X
    // at M > 32: beside four tiles of X in registers the scales do not fit (93 us against 83 at M = 64)
    // ... and on the F16 matrix cores at M > 16, where X in registers and the converted operands do not fit together
    if (a.K != GK || (SCALED == 2 && a.M > 32) || (ACC == 1 && a.M > 16)) {
        if (a.M <= 16) hipLaunchKernelGGL((ecf8_gemm_anyk_kernel<1, 16, 64, SCALED, false, ACC>), dim3(grid), dim3(16 * 64), 0, s, a);
        else if (a.M <= 32) hipLaunchKernelGGL((ecf8_gemm_anyk_kernel<2, 8, 64, SCALED, false, ACC>), dim3(grid), dim3(8 * 64), 0, s, a);   // X pieces of two chunks: 8 waves' worth of registers
        else hipLaunchKernelGGL((ecf8_gemm_anyk_kernel<4, 8, 64, SCALED, false, ACC>), dim3(grid), dim3(8 * 64), 0, s, a);
        return hipGetLastError() == hipSuccess ? ECF8_OK : ECF8_E_HIP;
    }
    if (a.M <= 16) hipLaunchKernelGGL((ecf8_gemm_kernel<1, 16, 64, SCALED, ACC>), dim3(grid), dim3(16 * 64), 0, s, a);
    else if constexpr (ACC == 0) {
        if (a.M <= 32) hipLaunchKernelGGL((ecf8_gemm_kernel<2, 16, 64, SCALED, ACC>), dim3(grid), dim3(16 * 64), 0, s, a);
        else if constexpr (SCALED != 2) hipLaunchKernelGGL((ecf8_gemm_kernel<4, 8, 64, SCALED, ACC>), dim3(grid), dim3(8 * 64), 0, s, a);
    }
    return hipGetLastError() == hipSuccess ? ECF8_OK : ECF8_E_HIP;
}

template <int SCALED, int ACC = 0>
int launch_raw(const GArgs &a, void *stream)
{
    const int grid = grid_for(a.rows / BLOCK_ROWS);
    if (grid <= 0) return ECF8_E_HIP;
    hipStream_t s = (hipStream_t)stream;
    if (a.K != GK || (SCALED == 2 && a.M > 32) || (ACC == 1 && a.M > 16)) {      // the same routes as the fused call: same order of accumulation
        if (a.M <= 16) hipLaunchKernelGGL((ecf8_gemm_raw_anyk_kernel<1, 16, 64, SCALED, false, ACC>), dim3(grid), dim3(16 * 64), 0, s, a);
        else if (a.M <= 32) hipLaunchKernelGGL((ecf8_gemm_raw_anyk_kernel<2, 8, 64, SCALED, false, ACC>), dim3(grid), dim3(8 * 64), 0, s, a);
        else hipLaunchKernelGGL((ecf8_gemm_raw_anyk_kernel<4, 8, 64, SCALED, false, ACC>), dim3(grid), dim3(8 * 64), 0, s, a);
        return hipGetLastError() == hipSuccess ? ECF8_OK : ECF8_E_HIP;
    }
    if (a.M <= 16) hipLaunchKernelGGL((ecf8_gemm_raw_kernel<1, 16, 64, SCALED, ACC>), dim3(grid), dim3(16 * 64), 0, s, a);
    else if constexpr (ACC == 0) {
        if (a.M <= 32) hipLaunchKernelGGL((ecf8_gemm_raw_kernel<2, 16, 64, SCALED, ACC>), dim3(grid), dim3(16 * 64), 0, s, a);
        else if constexpr (SCALED != 2) hipLaunchKernelGGL((ecf8_gemm_raw_kernel<4, 8, 64, SCALED, ACC>), dim3(grid), dim3(8 * 64), 0, s, a);
    }
    return hipGetLastError() == hipSuccess ? ECF8_OK : ECF8_E_HIP;
}

// The counters (one per block of rows; a split matrix has at most compute units / 2 blocks) take a fixed
// area at the start of the workspace whatever the shape, so that the partial sums of one call never
// land where another shape's call keeps its counters.
constexpr uint64_t CTR_BYTES = 4096;

// Split K.  Workgroups that share a block of rows: the largest divisor of the K / 256 chunks that
// still gives every workgroup a compute unit of its own (1 = the matrix has blocks enough).
inline uint32_t pick_slices(uint64_t rows, uint64_t cols, int cus)
{
    const uint64_t n_blocks = rows / BLOCK_ROWS, kchunks = cols / 256;
    uint32_t best = 1;
    if (n_blocks * 4 > CTR_BYTES) return 1;
    for (uint64_t sl = 2; sl <= kchunks && n_blocks * sl <= (uint64_t)cus; sl++)
        if (kchunks % sl == 0) best = (uint32_t)sl;
    return best;
}

inline int tiles_of(uint32_t M) { return M <= 16 ? 1 : M <= 32 ? 2 : 4; }
inline uint64_t workspace_bytes(uint64_t rows, uint32_t M, uint32_t slices)
{
    return slices <= 1 ? 0 : CTR_BYTES + rows / BLOCK_ROWS * slices * tiles_of(M) * 256 * 4;
}

inline int split_args(GArgs *a, void *d_workspace, uint64_t bytes, uint32_t *slices)
{
    const int cus = device_cus();
    if (cus <= 0) return ECF8_E_HIP;
    *slices = pick_slices(a->rows, a->K, cus);
    if (*slices <= 1) return ECF8_OK;
    if (!d_workspace) return ECF8_E_ARG;
    if ((uintptr_t)d_workspace & 15) return ECF8_E_ALIGN;
    if (bytes < workspace_bytes(a->rows, a->M, *slices)) return ECF8_E_CAPACITY;
    a->slices = *slices;
    a->d_ctr = (uint64_t)(uintptr_t)d_workspace;
    a->d_part = a->d_ctr + CTR_BYTES;
    return ECF8_OK;
}

template <int SCALED, bool RAW>
int launch_split(const GArgs &a, void *stream)
{
    const int grid = grid_for(a.rows / BLOCK_ROWS * a.slices);      // <= the compute units by the choice of slices
    if (grid <= 0) return ECF8_E_HIP;
    hipStream_t s = (hipStream_t)stream;
    if constexpr (RAW) {
        if (a.M <= 16) hipLaunchKernelGGL((ecf8_gemm_raw_anyk_kernel<1, 16, 64, SCALED, true>), dim3(grid), dim3(16 * 64), 0, s, a);
        else if (a.M <= 32) hipLaunchKernelGGL((ecf8_gemm_raw_anyk_kernel<2, 8, 64, SCALED, true>), dim3(grid), dim3(8 * 64), 0, s, a);
        else hipLaunchKernelGGL((ecf8_gemm_raw_anyk_kernel<4, 8, 64, SCALED, true>), dim3(grid), dim3(8 * 64), 0, s, a);
    } else {
        if (a.M <= 16) hipLaunchKernelGGL((ecf8_gemm_anyk_kernel<1, 16, 64, SCALED, true>), dim3(grid), dim3(16 * 64), 0, s, a);
        else if (a.M <= 32) hipLaunchKernelGGL((ecf8_gemm_anyk_kernel<2, 8, 64, SCALED, true>), dim3(grid), dim3(8 * 64), 0, s, a);
        else hipLaunchKernelGGL((ecf8_gemm_anyk_kernel<4, 8, 64, SCALED, true>), dim3(grid), dim3(8 * 64), 0, s, a);
    }
    return hipGetLastError() == hipSuccess ? ECF8_OK : ECF8_E_HIP;
}

// the common tail of the two split-K calls: scales (or none), workspace, route
template <bool RAW>
int run_split(GArgs &a, const float *d_w_scale, const float *d_x_scale, uint32_t x_scale_cols, void *d_workspace,
              uint64_t bytes, void *stream)
{
    int sc = 0;
    if (d_w_scale || d_x_scale || x_scale_cols) {
        const int rc = scale_args(d_w_scale, d_x_scale, x_scale_cols, &a);
        if (rc) return rc;
        sc = a.xs_cols > 1 ? 2 : 1;
    }
    uint32_t slices;
    const int rc = split_args(&a, d_workspace, bytes, &slices);
    if (rc) return rc;
    if (slices <= 1) {      // blocks enough: the plain kernels
        if constexpr (RAW) return sc == 0 ? launch_raw<0>(a, stream) : sc == 1 ? launch_raw<1>(a, stream) : launch_raw<2>(a, stream);
        else return sc == 0 ? launch_fused<0>(a, stream) : sc == 1 ? launch_fused<1>(a, stream) : launch_fused<2>(a, stream);
    }
    return sc == 0 ? launch_split<0, RAW>(a, stream) : sc == 1 ? launch_split<1, RAW>(a, stream) : launch_split<2, RAW>(a, stream);
}

template <int SCALED, bool RAW>
int launch_grouped(const GGArgs &g, uint32_t max_M, void *stream)
{
    const int cus = device_cus();
    if (cus <= 0) return ECF8_E_HIP;
    // no more workgroups than blocks of 16 chunks: below that a share is less than a block's worth of the waves' work
    uint64_t grid = (g.total_work + 15) / 16;
    if (grid > (uint64_t)cus) grid = (uint64_t)cus;
    if (grid == 0) grid = 1;
    hipStream_t s = (hipStream_t)stream;
    if (max_M <= 16) hipLaunchKernelGGL((ecf8_gemm_grouped_kernel<1, 16, 64, SCALED, RAW>), dim3((unsigned)grid), dim3(16 * 64), 0, s, g);
    else if (max_M <= 32) hipLaunchKernelGGL((ecf8_gemm_grouped_kernel<2, 8, 64, SCALED, RAW>), dim3((unsigned)grid), dim3(8 * 64), 0, s, g);
    else hipLaunchKernelGGL((ecf8_gemm_grouped_kernel<4, 8, 64, SCALED, RAW>), dim3((unsigned)grid), dim3(8 * 64), 0, s, g);
    return hipGetLastError() == hipSuccess ? ECF8_OK : ECF8_E_HIP;
}

__global__ __attribute__((unused)) void gemm_fill_zero_kernel(uint64_t p, uint64_t n_dwords)
{
    const uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    if (i < n_dwords) ((GLOBAL uint32_t *)p)[i] = 0u;
}

} // namespace

#endif
