// Wide-alphabet decode kernels (E5M2, BF16) for gfx950, wave64: Algorithm 1 of
// the paper for exponent fields of 5 and 8 bits, organised like the ECF8 decoder
// (ecf8_decode.hip): one wavefront per chunk of 64 lanes x N symbols, the lanes'
// start bits from a prefix scan over the recorded lane lengths, the chunk's span
// of the stream staged in LDS, two independent runs per lane (one read forward,
// one backward), finished 16-byte pieces held in registers and stored in one
// burst, persistent workgroups over contiguous chunk ranges with an LDS ticket
// counter among their waves.  What differs:
//  * the lookup table has 2^12 16-bit entries and resolves ONE codeword per
//    lookup (with up to 256 symbols a pair table would not fit LDS); an entry is
//    the exponent field already shifted to its place in the output element, plus
//    the codeword's length.  One 32-bit window serves two lookups;
//  * under the encoder's default cap of 12 bits every codeword is a table hit
//    (FAST kernels: straight-line code); longer codes (cap 13..16) fall to a
//    canonical first-code comparison per length, in a rarely taken branch;
//  * the remaining bits come from planes laid out so that whole output words are
//    merged with a few bit selects (BF16: a byte per element in the order
//    0 2 1 3; E5M2: mantissas sliced by output word, signs as a bit mask);
//  * these kernels are bound by the LDS, not by HBM, unless the window reads are
//    kept off each other's banks: the FAST kernels move every lane's bits from
//    the linear image of the span into a column of its own before decoding
//    (dword r of lane l at row r, column l), see WCfg;
//  * one launch may cover many tensors (ecfw_decode_batched): a workgroup's
//    range of chunks runs through the batch and the code is set up again where
//    it crosses into another tensor.
#include "ecfw.h"

#include "ecf8_device.h"

#include <cstring>

#include <cstdlib>

namespace {

constexpr int WTB = ECFW_TABLE_BITS;
constexpr uint32_t WMASK2 = ((1u << WTB) - 1) << 1;   // byte offset mask of a 16-bit entry

typedef ecfw_batch_item WArgs;          // one tensor, as the kernel sees it

struct BArgs {
    WArgs single;                        // used when items == nullptr
    const GLOBAL WArgs *items;           // device array for the batched call
    uint32_t n_items;
    uint64_t total_chunks;
};

template <int FMT> struct Fmt;
template <> struct Fmt<ECFW_FMT_E5M2> {
    static constexpr int P = 16, ELEM = 1, A = 32;
    static constexpr int SYM_SHIFT = 2, LEN_SHIFT = 8;     // entry = exponent << 2 | length << 8
};
template <> struct Fmt<ECFW_FMT_BF16> {
    static constexpr int P = 8, ELEM = 2, A = 256;
    static constexpr int SYM_SHIFT = 7, LEN_SHIFT = 0;     // entry = exponent << 7 | length
};

// COLS: after the chunk's span has landed in LDS, every lane copies the dwords of its own bits into a
// column of its own (dword r of lane l at row r, column l: bank l % 32), so that the two window
// reads of every decode step are free of bank conflicts; the copy reads each dword once instead.
template <int FMT, int N, int WAVES, bool COLS>
struct WCfg {
    using F = Fmt<FMT>;
    static constexpr int PIECES = N / F::P;                 // 16-byte pieces per lane
    // span of a chunk whose codewords average AVG bits: uniformly random exponent fields still fit
    static constexpr int AVG = COLS ? (FMT == ECFW_FMT_BF16 ? 8 : 5) : 8;
    static constexpr int STAGE = 8 * AVG * N + 64;
    static constexpr int SEGS = (STAGE / 16 + 63) / 64;
    // rows of a lane's column: its bits at up to AVG + 1/2 bits per codeword, the dword before, the
    // dword after, and the misalignment of its first bit
    static constexpr int ROWS = COLS ? ((2 * AVG + 1) * N / 64 + 3) : 0;
    static constexpr int OFF_TBL = 0;
    static constexpr int OFF_WCNT = OFF_TBL + (2 << WTB);   // symbols per (wavefront, length) while the code is set up
    static constexpr int OFF_SORTED = OFF_WCNT + 320;       // symbols ordered by (length, symbol)
    static constexpr int OFF_CNT = OFF_SORTED + 256;        // per length 0..16: count, first code, offset into sorted
    static constexpr int OFF_FIRST = OFF_CNT + 80;
    static constexpr int OFF_OFFS = OFF_FIRST + 80;
    static constexpr int OFF_TICKET = OFF_OFFS + 80;
    static constexpr int OFF_STAGE = OFF_TICKET + 16 + 16;  // one spare slot below: a column's first row is the dword
                                                            // before the lane's first one
    static constexpr int OFF_COLS = OFF_STAGE + WAVES * STAGE;
    static constexpr int TOTAL = OFF_COLS + WAVES * ROWS * 256;
    static_assert(STAGE % 16 == 0 && OFF_STAGE % 16 == 0, "16-byte LDS stores");
    static_assert(PIECES % 2 == 0, "two runs of whole pieces");
    static_assert(TOTAL <= 160 * 1024, "LDS of one gfx950 CU");
};

struct CodeArrays {
    const uint16_t *tbl;
    const uint8_t *sorted;
    const uint32_t *cnt, *first, *offs;
};

// Sets up, from the code lengths in the blob: the per-length canonical arrays
// (count, first code, offset into the list of symbols sorted by (length, symbol))
// and the lookup table.  All threads of the workgroup call it; it needs at least
// four wavefronts.  Symbols are ranked with wave ballots (wavefront w holds symbols
// 64w..64w+63), so nothing here loops over the alphabet.
template <int FMT>
__device__ void build_code(const GLOBAL uint8_t *code_len, uint32_t *wavecnt, uint8_t *sorted, uint32_t *cnt,
                           uint32_t *first, uint32_t *offs, uint16_t *tbl, int tid, int nthreads)
{
    using F = Fmt<FMT>;
    constexpr int L = (int)ECFW_MAX_CODE_LEN;
    const int lane = tid & 63, wave = tid >> 6;
    uint32_t my_len = 0, my_rank = 0;
    if (tid < 256) {
        my_len = tid < F::A ? code_len[tid] : 0;
        if (my_len > (uint32_t)L) my_len = 0;
        const uint64_t below = ((uint64_t)1 << lane) - 1;
#pragma unroll
        for (int l = 1; l <= L; l++) {
            const uint64_t m = __ballot(my_len == (uint32_t)l);
            if (my_len == (uint32_t)l) my_rank = (uint32_t)__popcll(m & below);
            if (lane == 0) wavecnt[wave * 20 + l] = (uint32_t)__popcll(m);
        }
    }
    __syncthreads();
    // every thread keeps the canonical arrays of the lengths the table covers in registers
    uint32_t r_first[WTB + 1], r_offs[WTB + 1], r_limit[WTB + 1];   // limit: first code of the next length, left-aligned
    {
        uint32_t code = 0, off = 0, prev = 0;
#pragma unroll
        for (int l = 1; l <= L; l++) {
            const uint32_t c = wavecnt[l] + wavecnt[20 + l] + wavecnt[40 + l] + wavecnt[60 + l];
            code = (code + prev) << 1;
            if (l <= WTB) {
                r_first[l] = code;
                r_offs[l] = off;
                r_limit[l] = (code + c) << (WTB - l);
            }
            if (tid == 0) { cnt[l] = c; first[l] = code; offs[l] = off; }
            if (my_len == (uint32_t)l) {
                uint32_t before = 0;
#pragma unroll
                for (int w = 0; w < 4; w++) before += w < wave ? wavecnt[w * 20 + l] : 0;
                my_rank += off + before;
            }
            off += c;
            prev = c;
        }
    }
    if (tid < 256 && my_len) sorted[my_rank] = (uint8_t)tid;
    __syncthreads();
    // entry i: the codeword spelled by the bits of i, bit 0 first
    for (int i = tid; i < (1 << WTB); i += nthreads) {
        const uint32_t v = __brev((uint32_t)i) >> (32 - WTB);       // the 12 bits, first bit most significant
        uint32_t e = 0;
#pragma unroll
        for (int l = WTB; l >= 1; l--)                              // the smallest length whose codes reach past v
            if (v < r_limit[l]) e = ((uint32_t)l << 16) | (r_offs[l] + (v >> (WTB - l)) - r_first[l]);
        if (e) e = ((uint32_t)sorted[e & 0xffffu] << F::SYM_SHIFT) | ((e >> 16) << F::LEN_SHIFT);
        tbl[i] = (uint16_t)e;
    }
    __syncthreads();
}

template <int FMT>
__device__ __forceinline__ uint32_t entry_len(uint32_t e)
{
    return (e >> Fmt<FMT>::LEN_SHIFT) & 31u;
}

// A codeword longer than the table index: compare the next bits with the first
// code of every longer length.  `bits`: >= 16 valid stream bits, next bit = bit 0.
template <int FMT>
__device__ __noinline__ uint32_t long_code(uint32_t bits, const uint8_t *sorted, const uint32_t *cnt,
                                           const uint32_t *first, const uint32_t *offs)
{
    using F = Fmt<FMT>;
    const uint32_t r = __brev(bits);
    uint32_t e = (uint32_t)ECFW_MAX_CODE_LEN << F::LEN_SHIFT;     // no match (corrupt stream): skip 16 bits
#pragma unroll 1
    for (int l = WTB + 1; l <= (int)ECFW_MAX_CODE_LEN; l++) {
        const uint32_t d = (r >> (32 - l)) - first[l];
        if (d < cnt[l]) e = ((uint32_t)sorted[offs[l] + d] << F::SYM_SHIFT) | ((uint32_t)l << F::LEN_SHIFT);
    }
    return e;
}

template <int FMT, bool FAST>
__device__ __forceinline__ uint32_t decode_entry(uint32_t bits, const CodeArrays &ca)
{
    uint32_t e = ca.tbl[bits & ((1u << WTB) - 1)];
    if (!FAST && __builtin_expect(e == 0, 0)) e = long_code<FMT>(bits, ca.sorted, ca.cnt, ca.first, ca.offs);
    return e;
}

// Two codewords of each run.  pa = (next bit of the forward run) - 1 and
// pb = (one past the next bit of the backward run) - 31 as absolute LDS bit
// addresses: the windows read there are the stream bits shifted left by one,
// which masked is the byte offset of a table entry.
// COLS: pa and pb count bits inside the lane's column (row = bit / 32), `smem` points at the lane's
// slot of row 0, and consecutive dwords of the lane lie 256 bytes apart.
template <int FMT, bool FAST, bool COLS>
__device__ __forceinline__ void pair_step(const uint8_t *smem, const CodeArrays &ca, uint32_t &pa, uint32_t &pb,
                                          uint32_t &eA0, uint32_t &eA1, uint32_t &eB0, uint32_t &eB1)
{
    static_assert(!COLS || FAST, "the long-code branch reads windows from the linear stage");
    const uint8_t *tb = (const uint8_t *)ca.tbl;
    constexpr uint32_t NEXT = COLS ? 256 : 4;
    const uint32_t aA = COLS ? (pa >> 5) << 8 : (pa >> 3) & ~3u, aB = COLS ? (pb >> 5) << 8 : (pb >> 3) & ~3u;
    const uint32_t wA = __builtin_amdgcn_alignbit(*(const uint32_t *)(smem + aA + NEXT), *(const uint32_t *)(smem + aA), pa);
    const uint32_t wB = __brev(__builtin_amdgcn_alignbit(*(const uint32_t *)(smem + aB + NEXT), *(const uint32_t *)(smem + aB), pb));
    eA0 = *(const uint16_t *)(tb + (wA & WMASK2));
    eB0 = *(const uint16_t *)(tb + (wB & WMASK2));
    uint32_t lA0 = entry_len<FMT>(eA0), lB0 = entry_len<FMT>(eB0);
    eA1 = *(const uint16_t *)(tb + ((wA >> lA0) & WMASK2));      // 31 - 12 >= 12 bits left
    eB1 = *(const uint16_t *)(tb + ((wB >> lB0) & WMASK2));
    uint32_t lA1 = entry_len<FMT>(eA1), lB1 = entry_len<FMT>(eB1);
    // a miss leaves the length 0, so the second lookup repeats the first: testing the second covers both
    if (!FAST && __builtin_expect(eA1 == 0 || eB1 == 0, 0)) {
        if (eA1 == 0) {
            if (eA0 == 0) { eA0 = long_code<FMT>(wA >> 1, ca.sorted, ca.cnt, ca.first, ca.offs); lA0 = entry_len<FMT>(eA0); }
            eA1 = decode_entry<FMT, false>(lds_window<+1>(smem, pa + 1 + lA0), ca);
            lA1 = entry_len<FMT>(eA1);
        }
        if (eB1 == 0) {
            if (eB0 == 0) { eB0 = long_code<FMT>(wB >> 1, ca.sorted, ca.cnt, ca.first, ca.offs); lB0 = entry_len<FMT>(eB0); }
            eB1 = decode_entry<FMT, false>(lds_window<-1>(smem, pb + 31 - lB0), ca);
            lB1 = entry_len<FMT>(eB1);
        }
    }
    pa += lA0 + lA1;
    pb -= lB0 + lB1;
}

__device__ __forceinline__ uint32_t bit_sel(uint32_t mask, uint32_t a, uint32_t b)   // (a & mask) | (b & ~mask)
{
    return __builtin_amdgcn_bitop3_b32(a, b, mask, 0xE4);
}

// One 16-byte piece from its table entries and plane words.
// BF16: e[0..7]; pl.x / pl.y hold the remainder bytes of elements 0 2 1 3 / 4 6 5 7.
__device__ __forceinline__ u32x4 merge_bf16(const uint32_t e[8], u32x2 pl)
{
    u32x4 d;
    const uint32_t x0 = __builtin_amdgcn_perm(e[1], e[0], 0x05040100u), x1 = __builtin_amdgcn_perm(e[3], e[2], 0x05040100u);
    const uint32_t x2 = __builtin_amdgcn_perm(e[5], e[4], 0x05040100u), x3 = __builtin_amdgcn_perm(e[7], e[6], 0x05040100u);
    // per 16-bit half: bit 15 sign, bits 14..7 exponent (from the entry), bits 6..0 mantissa
    d.x = bit_sel(0x7f807f80u, x0, bit_sel(0x80008000u, pl.x << 8, pl.x));
    d.y = bit_sel(0x7f807f80u, x1, bit_sel(0x80008000u, pl.x, pl.x >> 8));
    d.z = bit_sel(0x7f807f80u, x2, bit_sel(0x80008000u, pl.y << 8, pl.y));
    d.w = bit_sel(0x7f807f80u, x3, bit_sel(0x80008000u, pl.y, pl.y >> 8));
    return d;
}

// E5M2: e[0..15]; mant = the piece's mantissa word, sign = its 16 sign bits.
__device__ __forceinline__ u32x4 merge_e5m2(const uint32_t e[16], uint32_t mant, uint32_t sign)
{
    uint32_t out[4];
#pragma unroll
    for (int d = 0; d < 4; d++) {
        const uint32_t lo = __builtin_amdgcn_perm(e[4 * d + 1], e[4 * d], 0x0c0c0400u);       // bytes 0, 1
        const uint32_t hi = __builtin_amdgcn_perm(e[4 * d + 3], e[4 * d + 2], 0x04000c0cu);   // bytes 2, 3
        // four sign bits -> bit 0 of each byte (the partial products do not overlap), then up to bit 7
        const uint32_t s4 = __builtin_amdgcn_ubfe(sign, 4 * d, 4);
        const uint32_t sp = __umul24(s4, 0x204081u) << 7;
        out[d] = bit_sel(0x7c7c7c7cu, lo | hi, bit_sel(0x80808080u, sp, mant >> (2 * d)));
    }
    return u32x4{out[0], out[1], out[2], out[3]};
}

template <int FMT, int N, int WAVES, bool FAST>
__global__ __launch_bounds__(WAVES * 64) void ecfw_decode_kernel(BArgs b)
{
    constexpr bool COLS = FAST;
    using C = WCfg<FMT, N, WAVES, COLS>;
    using F = Fmt<FMT>;
    constexpr int PIECES = C::PIECES, SEGS = C::SEGS, STAGE = C::STAGE, P = F::P, ROWS = C::ROWS;
    __shared__ __attribute__((aligned(16))) uint8_t smem[C::TOTAL];
    uint16_t *tbl = (uint16_t *)(smem + C::OFF_TBL);
    uint32_t *s_ticket = (uint32_t *)(smem + C::OFF_TICKET);
    const CodeArrays ca{tbl, smem + C::OFF_SORTED, (const uint32_t *)(smem + C::OFF_CNT),
                        (const uint32_t *)(smem + C::OFF_FIRST), (const uint32_t *)(smem + C::OFF_OFFS)};

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t stage_off = C::OFF_STAGE + wave * STAGE;
    uint8_t *stage = smem + stage_off;
    uint8_t *column = smem + C::OFF_COLS + wave * (ROWS * 256) + lane * 4;      // this lane's slot of row 0

    // contiguous range of chunks for this workgroup, cut at multiples of 64 chunks when there is
    // enough work so that the waves of a workgroup share the interleaved groups of the layout
    const uint64_t NWG = gridDim.x, wg = blockIdx.x;
    const uint64_t unit = b.total_chunks >= NWG * 1024 ? 64 : b.total_chunks >= NWG * 128 ? 8 : 1;   // >= 16 units each: shares differ by 1/16 at most
    const uint64_t units = (b.total_chunks + unit - 1) / unit;
    uint64_t g = units * wg / NWG * unit;              // chunk numbers run through the whole batch
    uint64_t g_end = units * (wg + 1) / NWG * unit;
    if (g_end > b.total_chunks) g_end = b.total_chunks;

    while (g < g_end) {                                // one round per tensor the range touches (uniform)
    WArgs a;
    if (b.items) {
        uint32_t lo = 0, hi = b.n_items - 1;
        while (lo < hi) {
            const uint32_t mid = (lo + hi + 1) >> 1;
            if (uniform64(b.items[mid].first_chunk) <= g) lo = mid; else hi = mid - 1;
        }
        // the item is the same for every lane: say so, or its fields (and all the address arithmetic
        // on them) would live in vector registers
        const GLOBAL uint64_t *src = (const GLOBAL uint64_t *)(b.items + lo);
        uint64_t *dst = (uint64_t *)&a;
#pragma unroll
        for (int i = 0; i < (int)(sizeof(WArgs) / 8); i++) dst[i] = uniform64(src[i]);
    } else {
        a = b.single;
    }
    const uint64_t c_begin = g - a.first_chunk;        // chunk numbers inside the tensor
    const uint64_t c_end = g_end - a.first_chunk < a.n_chunks ? g_end - a.first_chunk : a.n_chunks;
    const GLOBAL uint8_t *blob = (const GLOBAL uint8_t *)a.d_blob;
    const GLOBAL uint64_t *chunk_bit = (const GLOBAL uint64_t *)(blob + a.off_chunk_bit);
    const GLOBAL uint16_t *lane_bits = (const GLOBAL uint16_t *)(blob + a.off_lane_bits);
    const GLOBAL uint8_t *stream = blob + a.off_stream;
    const GLOBAL uint8_t *plane = blob + a.off_plane;
    const GLOBAL uint8_t *signs = blob + a.off_sign;
    GLOBAL uint8_t *out = (GLOBAL uint8_t *)a.d_out;


    if (tid == 0) *s_ticket = 0;
    static_assert(WAVES >= 4, "the code set-up ranks 256 symbols with four wavefronts");
    build_code<FMT>(blob + a.off_code_len, (uint32_t *)(smem + C::OFF_WCNT), smem + C::OFF_SORTED, (uint32_t *)(smem + C::OFF_CNT),
                    (uint32_t *)(smem + C::OFF_FIRST), (uint32_t *)(smem + C::OFF_OFFS), tbl, tid, WAVES * 64);

    const uint64_t E = 64ull * N;
    const uint64_t whole = a.n_elem / (a.group_chunks * E) * a.group_chunks;     // chunks inside complete groups
    auto chunk_base = [&](uint64_t c) -> uint64_t {
        return c < whole ? (c - c % a.group_chunks) * E + (c % a.group_chunks) * (64 * P) : c * E;
    };
    auto chunk_stride = [&](uint64_t c) -> uint64_t { return c < whole ? (uint64_t)a.group_chunks * (64 * P) : 64ull * P; };

    struct Meta { uint64_t b0, b1; uint32_t lb; };
    struct Payload {
        u32x4 seg[SEGS];
        u32x2 pl[FMT == ECFW_FMT_BF16 ? PIECES : 1];
        uint32_t mant[FMT == ECFW_FMT_E5M2 ? PIECES : 1];
        uint32_t sign[FMT == ECFW_FMT_E5M2 ? PIECES : 1];
    };
    auto draw = [&]() -> uint64_t {
        uint32_t t = 0;
        if (lane == 0) t = atomicAdd(s_ticket, 1u);
        return c_begin + uniform32(t);
    };
    auto load_meta = [&](uint64_t c) {
        Meta m;
        m.b0 = chunk_bit[c];
        m.b1 = chunk_bit[c + 1];
        m.lb = lane_bits[c * 64 + lane];
        return m;
    };
    auto span_of = [&](const Meta &m, uint64_t &byte0) -> uint64_t {
        uint64_t byte_end = ((m.b1 + 7) >> 3) + 8;
        if (byte_end > a.stream_bytes) byte_end = a.stream_bytes;
        byte0 = (m.b0 >> 3) & ~15ull;
        if (byte0 > byte_end) byte0 = byte_end;
        return byte_end - byte0;
    };
    auto load_payload = [&](uint64_t c, const Meta &m, Payload &p) {
        uint64_t byte0;
        const uint64_t span = span_of(m, byte0);
        const uint64_t e0 = chunk_base(c) + (uint64_t)lane * P, stride = chunk_stride(c);
#pragma unroll
        for (int q = 0; q < PIECES; q++) {
            const uint64_t e = e0 + q * stride;
            if (FMT == ECFW_FMT_BF16) {
                p.pl[q] = __builtin_nontemporal_load((const GLOBAL u32x2 *)(plane + e));
            } else {
                p.mant[q] = __builtin_nontemporal_load((const GLOBAL uint32_t *)(plane + e / 4));
                p.sign[q] = __builtin_nontemporal_load((const GLOBAL uint16_t *)(signs + e / 8));
            }
        }
#pragma unroll
        for (int k = 0; k < SEGS; k++) {
            const uint32_t i = (lane + 64 * k) * 16;
            p.seg[k] = u32x4{0, 0, 0, 0};
            if (i < (uint32_t)STAGE && i < span)
                p.seg[k] = __builtin_nontemporal_load((const GLOBAL u32x4 *)(stream + byte0 + i));
        }
    };

    // The careful way, one symbol at a time with windows straight from HBM: the ragged last
    // chunk, and chunks whose span does not fit the stage (codewords averaging over 8 bits).
    auto symbol_pass = [&](uint64_t c, const Meta &m) {
        const uint32_t rel = wave_incl_scan(m.lb) - m.lb;
        const uint64_t limit = a.stream_bytes * 8 - 64;
        uint64_t posA = m.b0 + rel, posB = posA + m.lb;
        const uint64_t e0 = chunk_base(c) + (uint64_t)lane * P, stride = chunk_stride(c);
#pragma unroll 1
        for (int k = 0; k < N; k++) {
            const uint64_t e = e0 + (uint64_t)(k / P) * stride + (uint32_t)(k % P);
            if (e >= a.n_elem) continue;
            uint32_t en;
            if (k < N / 2) {
                if (posA > limit) posA = limit;
                en = decode_entry<FMT, false>(global_window<+1>(stream, posA), ca);
                posA += entry_len<FMT>(en);
            } else {
                if (posB > limit) posB = limit;
                en = decode_entry<FMT, false>(global_window<-1>(stream, posB), ca);
                const uint32_t l = entry_len<FMT>(en);
                posB = posB >= l ? posB - l : 0;
            }
            if (FMT == ECFW_FMT_BF16) {
                const uint32_t swap = (0x3120u >> (4 * (uint32_t)(e & 3))) & 3u;      // 0 2 1 3
                const uint32_t r = plane[(e & ~3ull) + swap];
                ((GLOBAL uint16_t *)out)[e] = (uint16_t)(((r & 0x80u) << 8) | (en & 0x7f80u) | (r & 0x7fu));
            } else {
                const uint32_t j = (uint32_t)(e & 3), d = (uint32_t)(e >> 2) & 3;
                const uint32_t mw = ((const GLOBAL uint32_t *)plane)[e / 16];
                const uint32_t sw = ((const GLOBAL uint16_t *)signs)[e / 16];
                out[e] = (uint8_t)((((sw >> (e & 15)) & 1u) << 7) | (en & 0x7cu) | ((mw >> (8 * j + 2 * d)) & 3u));
            }
        }
    };

    uint64_t cur = draw();
    Meta m_cur{0, 0, 0}, m_next{0, 0, 0};
    Payload p_cur;
    if (cur < c_end) {
        m_cur = load_meta(cur);
        load_payload(cur, m_cur, p_cur);
    }
    uint64_t nxt = draw();
    if (nxt < c_end) m_next = load_meta(nxt);

    while (cur < c_end) {
        const Meta m = m_cur;
        uint64_t byte0;
        const uint64_t span = span_of(m, byte0);
        const uint32_t rel = wave_incl_scan(m.lb) - m.lb;
        const uint64_t start = uniform64(m.b0);
        const uint32_t first_bit = (uint32_t)(start - byte0 * 8) + rel;           // this lane's first bit, counted from byte0
        // COLS: rows this lane's bits take (with the dword before and the one after), and the most any lane takes
        const uint32_t rows_used = COLS ? wave_max(((32 + (first_bit & 31) + m.lb) >> 5) + 2) : 0;
        const bool careful = span > (uint64_t)STAGE || (cur + 1) * E > a.n_elem || rows_used > (uint32_t)ROWS;    // uniform
        if (!careful) {
#pragma unroll
            for (int k = 0; k < SEGS; k++) {
                const uint32_t j = (lane + 64 * k) * 16;
                if (j < (uint32_t)STAGE) *(u32x4 *)(stage + j) = p_cur.seg[k];
            }
        }
        u32x2 pl[FMT == ECFW_FMT_BF16 ? PIECES : 1];
        uint32_t mant[FMT == ECFW_FMT_E5M2 ? PIECES : 1], sign[FMT == ECFW_FMT_E5M2 ? PIECES : 1];
#pragma unroll
        for (int q = 0; q < PIECES; q++) {
            if (FMT == ECFW_FMT_BF16) pl[q] = p_cur.pl[q];
            else { mant[q] = p_cur.mant[q]; sign[q] = p_cur.sign[q]; }
        }
        // the payload registers are free: fetch the next chunk, draw the one after and fetch its metadata
        uint64_t nn = c_end;
        Meta m_next2{0, 0, 0};
        if (nxt < c_end) {
            load_payload(nxt, m_next, p_cur);
            nn = draw();
            if (nn < c_end) m_next2 = load_meta(nn);
        }
        if (careful) {
            symbol_pass(cur, m);
        } else {
            uint32_t pa = stage_off * 8 + first_bit - 1;    // one bit off, see pair_step
            if constexpr (COLS) {
                // row r of the column = dword (first_bit / 32) - 1 + r of the stage (row 0 of a lane that starts in the
                // stage's first dword is the spare slot below the stage)
                const uint8_t *src = stage + ((first_bit >> 5) << 2) - 4;
#pragma unroll
                for (int r = 0; r < ROWS; r++)
                    if ((uint32_t)r < rows_used) *(uint32_t *)(column + r * 256) = *(const uint32_t *)(src + r * 4);
                pa = 32 + (first_bit & 31) - 1;
            }
            uint32_t pb = pa + m.lb - 30;
            const uint8_t *bits = COLS ? column : smem;
            GLOBAL uint8_t *dst = out + (chunk_base(cur) + (uint64_t)lane * P) * F::ELEM;
            const uint64_t stride_bytes = chunk_stride(cur) * F::ELEM;
            // finished pieces wait in registers and leave in bursts of eight (8 KiB per wavefront)
            constexpr int BURST = PIECES / 2 < 4 ? PIECES / 2 : 4;
            static_assert((PIECES / 2) % BURST == 0, "whole bursts");
#pragma unroll
            for (int q0 = 0; q0 < PIECES / 2; q0 += BURST) {
                u32x4 pieceA[BURST], pieceB[BURST];
#pragma unroll
                for (int i = 0; i < BURST; i++) {
                    const int q = q0 + i;
                    uint32_t eA[P], eB[P];
#pragma unroll
                    for (int t = 0; t < P / 2; t++)
                        pair_step<FMT, FAST, COLS>(bits, ca, pa, pb, eA[2 * t], eA[2 * t + 1], eB[2 * t], eB[2 * t + 1]);
                    if constexpr (FMT == ECFW_FMT_BF16) {
                        pieceA[i] = merge_bf16(eA, pl[q]);
                        pieceB[i] = merge_bf16(eB, pl[q + PIECES / 2]);
                    } else {
                        pieceA[i] = merge_e5m2(eA, mant[q], sign[q]);
                        pieceB[i] = merge_e5m2(eB, mant[q + PIECES / 2], sign[q + PIECES / 2]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < BURST; i++) __builtin_nontemporal_store(pieceA[i], (GLOBAL u32x4 *)(dst + (q0 + i) * stride_bytes));
#pragma unroll
                for (int i = 0; i < BURST; i++)
                    __builtin_nontemporal_store(pieceB[i], (GLOBAL u32x4 *)(dst + (q0 + i + PIECES / 2) * stride_bytes));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        cur = nxt;
        nxt = nn;
        m_cur = m_next;
        m_next = m_next2;
    }
    g = a.first_chunk + c_end;
    __syncthreads();                                   // every wave is done with this tensor's table and tickets
    }
}

template <int FMT, int N, int WAVES, bool FAST>
int launch_as(const BArgs &a, uint32_t max_workgroups, hipStream_t stream)
{
    int cus = device_cus();
    if (cus <= 0) return ECF8_E_HIP;
    uint64_t grid = (uint64_t)cus;
    if (max_workgroups && max_workgroups < grid) grid = max_workgroups;
    if (grid > a.total_chunks) grid = a.total_chunks;
    hipLaunchKernelGGL((ecfw_decode_kernel<FMT, N, WAVES, FAST>), dim3((unsigned)grid), dim3(WAVES * 64), 0, stream, a);
    return hipGetLastError() == hipSuccess ? ECF8_OK : ECF8_E_HIP;
}

template <int FMT>
int launch_fmt(const BArgs &a, uint32_t N, bool fast, uint32_t max_workgroups, hipStream_t stream)
{
    // the branch-free kernels at N = 64 need under 128 registers: 16 wavefronts hide more of the LDS latency
    if (N == 64 && fast) return launch_as<FMT, 64, 16, true>(a, max_workgroups, stream);
    if (N == 64) return launch_as<FMT, 64, 8, false>(a, max_workgroups, stream);
    // E5M2 at N = 128 needs under 170 registers: three wavefronts per SIMD
    if constexpr (FMT == ECFW_FMT_E5M2)
        if (fast) return launch_as<FMT, 128, 12, true>(a, max_workgroups, stream);
    return fast ? launch_as<FMT, 128, 8, true>(a, max_workgroups, stream) : launch_as<FMT, 128, 8, false>(a, max_workgroups, stream);
}

int launch(const BArgs &a, uint32_t fmt, uint32_t N, uint32_t max_code_len, uint32_t max_workgroups, void *stream)
{
    const bool fast = max_code_len <= ECFW_TABLE_BITS;
    hipStream_t s = (hipStream_t)stream;
    return fmt == ECFW_FMT_BF16 ? launch_fmt<ECFW_FMT_BF16>(a, N, fast, max_workgroups, s)
                                : launch_fmt<ECFW_FMT_E5M2>(a, N, fast, max_workgroups, s);
}

// Checks of one tensor's header and buffers; fills the kernel's view of it.
int make_item(const ecfw_header *h, const void *d_blob, void *d_out, uint64_t out_capacity, WArgs *it)
{
    if (!d_blob || !h || !d_out) return ECF8_E_ARG;
    if (h->magic != ECFW_MAGIC || h->version != ECFW_VERSION) return ECF8_E_FORMAT;
    if (h->fmt != ECFW_FMT_E5M2 && h->fmt != ECFW_FMT_BF16) return ECF8_E_FORMAT;
    if (h->lane_syms != 64 && h->lane_syms != 128) return ECF8_E_FORMAT;
    const uint32_t g = h->group_chunks;
    if (g < 1 || g > 64 || (g & (g - 1))) return ECF8_E_FORMAT;
    if (h->n_elem == 0 || h->n_chunks != (h->n_elem + 64ull * h->lane_syms - 1) / (64ull * h->lane_syms)) return ECF8_E_FORMAT;
    if (h->max_code_len < 1 || h->max_code_len > ECFW_MAX_CODE_LEN || h->stream_bytes < 16 || h->stream_bytes % 16)
        return ECF8_E_FORMAT;
    const uint64_t elem = h->fmt == ECFW_FMT_BF16 ? 2 : 1;
    if (out_capacity / elem < h->n_elem) return ECF8_E_CAPACITY;
    if (((uintptr_t)d_blob & 255) || ((uintptr_t)d_out & 15)) return ECF8_E_ALIGN;
    if ((h->off_code_len | h->off_chunk_bit | h->off_lane_bits | h->off_stream | h->off_plane | h->off_sign) & 255)
        return ECF8_E_FORMAT;
    std::memset(it, 0, sizeof(*it));
    it->d_blob = (uint64_t)(uintptr_t)d_blob;
    it->d_out = (uint64_t)(uintptr_t)d_out;
    it->n_elem = h->n_elem;
    it->n_chunks = h->n_chunks;
    it->first_chunk = 0;
    it->stream_bytes = h->stream_bytes;
    it->off_code_len = h->off_code_len;
    it->off_chunk_bit = h->off_chunk_bit;
    it->off_lane_bits = h->off_lane_bits;
    it->off_stream = h->off_stream;
    it->off_plane = h->off_plane;
    it->off_sign = h->off_sign;
    it->group_chunks = g;
    return ECF8_OK;
}

} // namespace

extern "C" int ecfw_decode(const void *d_blob, const ecfw_header *h, void *d_out, uint64_t out_capacity,
                           uint32_t max_workgroups, void *stream)
{
    BArgs a;
    int rc = make_item(h, d_blob, d_out, out_capacity, &a.single);
    if (rc) return rc;
    a.items = nullptr;
    a.n_items = 1;
    a.total_chunks = h->n_chunks;
    return launch(a, h->fmt, h->lane_syms, h->max_code_len, max_workgroups, stream);
}

extern "C" int ecfw_batch_prepare(const ecfw_header *hdrs, const void *const *d_blobs, void *const *d_outs,
                                  const uint64_t *out_capacities, uint32_t n, ecfw_batch_item *items_host,
                                  ecfw_batch_info *info)
{
    if (!hdrs || !d_blobs || !d_outs || !out_capacities || !items_host || !info || n == 0) return ECF8_E_ARG;
    std::memset(info, 0, sizeof(*info));
    uint64_t chunks = 0;
    for (uint32_t i = 0; i < n; i++) {
        int rc = make_item(&hdrs[i], d_blobs[i], d_outs[i], out_capacities[i], &items_host[i]);
        if (rc) return rc;
        if (hdrs[i].fmt != hdrs[0].fmt || hdrs[i].lane_syms != hdrs[0].lane_syms) return ECF8_E_ARG;
        items_host[i].first_chunk = chunks;
        chunks += hdrs[i].n_chunks;
        if (hdrs[i].max_code_len > info->max_code_len) info->max_code_len = hdrs[i].max_code_len;
    }
    info->total_chunks = chunks;
    info->fmt = hdrs[0].fmt;
    info->lane_syms = hdrs[0].lane_syms;
    return ECF8_OK;
}

extern "C" int ecfw_decode_batched(const void *d_items, uint32_t n, const ecfw_batch_info *info, void *stream)
{
    if (!d_items || !info || n == 0 || info->total_chunks == 0) return ECF8_E_ARG;
    if (info->fmt != ECFW_FMT_E5M2 && info->fmt != ECFW_FMT_BF16) return ECF8_E_ARG;
    if (info->lane_syms != 64 && info->lane_syms != 128) return ECF8_E_ARG;
    if (info->max_code_len < 1 || info->max_code_len > ECFW_MAX_CODE_LEN) return ECF8_E_ARG;
    if ((uintptr_t)d_items & 7) return ECF8_E_ALIGN;
    BArgs a;
    std::memset(&a.single, 0, sizeof(a.single));
    a.items = (const GLOBAL WArgs *)d_items;
    a.n_items = n;
    a.total_chunks = info->total_chunks;
    return launch(a, info->fmt, info->lane_syms, info->max_code_len, info->max_workgroups, stream);
}
