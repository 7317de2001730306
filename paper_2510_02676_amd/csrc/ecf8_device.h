// Device-side building blocks of the ECF8 decoder for gfx950, shared by the
// decode kernels and the fused decode + GEMM kernel: pair-table set-up in LDS,
// aligned LDS / HBM bit windows, the two-chain decode step, the nibble merge.
// See ecf8_decode.hip for how they fit together.
#ifndef ECF8_DEVICE_H
#define ECF8_DEVICE_H

#include "ecf8.h"
#include "ecf8_table.h"

#include <hip/hip_runtime.h>

#include <mutex>

namespace {

constexpr int TB = ECF8_TB;            // table index bits
constexpr int TBL_ENTRIES = 1 << TB;
constexpr uint32_t TBL_MASK = TBL_ENTRIES - 1;

// Table entry (16 bits) for index bits b0 b1 ... (b0 = next stream bit):
//   bits 3..6   : exponent field of the first symbol  (output position of byte 0)
//   bits 11..14 : exponent field of the second symbol (output position of byte 1)
//   bits 7..10  : stream bits consumed by both symbols; 0 = the pair does not
//                 fit in TB bits (second level decides)
//   bits 0..2,15: code length of the first symbol alone (low 3 bits, high bit);
//                 0 = the first codeword is longer than TB bits
// Control fields sit in bits the merge masks off (0x78 per byte keeps the
// exponent field only).
constexpr uint32_t EXP_MASK = 0x78787878u;

#define GLOBAL __attribute__((address_space(1))) // HBM pointers: global_load/store, not flat
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// code_len[16] travels as two 64-bit words (one byte per symbol)
__device__ __forceinline__ uint32_t len_of(uint64_t lo, uint64_t hi, int s)
{
    return (uint32_t)((s < 8 ? lo >> (8 * s) : hi >> (8 * (s - 8))) & 0xff);
}

// The first active lane's value, in scalar registers.  The builtin returns a signed int: widened
// as it is, a low word with bit 31 set would smear ones over the high word.
__device__ __forceinline__ uint32_t uniform32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint64_t uniform64(uint64_t v)
{
    return (uint64_t)uniform32((uint32_t)v) | ((uint64_t)uniform32((uint32_t)(v >> 32)) << 32);
}

// Inclusive wave64 prefix sum with DPP row shifts and row broadcasts.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x)
{
    uint32_t v = x;
    v += __builtin_amdgcn_update_dpp(0u, v, 0x111, 0xf, 0xf, false); // row_shr:1
    v += __builtin_amdgcn_update_dpp(0u, v, 0x112, 0xf, 0xf, false); // row_shr:2
    v += __builtin_amdgcn_update_dpp(0u, v, 0x114, 0xf, 0xf, false); // row_shr:4
    v += __builtin_amdgcn_update_dpp(0u, v, 0x118, 0xf, 0xf, false); // row_shr:8
    v += __builtin_amdgcn_update_dpp(0u, v, 0x142, 0xa, 0xf, false); // row_bcast:15 -> rows 1,3
    v += __builtin_amdgcn_update_dpp(0u, v, 0x143, 0xc, 0xf, false); // row_bcast:31 -> rows 2,3
    return v;
}

// Largest value of x over the wavefront (every lane gets it).
__device__ __forceinline__ uint32_t wave_max(uint32_t x)
{
    uint32_t v = x;
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, 0x111, 0xf, 0xf, false));   // row_shr:1
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, 0x112, 0xf, 0xf, false));   // row_shr:2
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, 0x114, 0xf, 0xf, false));   // row_shr:4
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, 0x118, 0xf, 0xf, false));   // row_shr:8
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, 0x142, 0xa, 0xf, false));   // row_bcast:15
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, 0x143, 0xc, 0xf, false));   // row_bcast:31
    return (uint32_t)__builtin_amdgcn_readlane(v, 63);
}

// A codeword longer than TB bits (rarer than 2^-TB): match the next 15 stream
// bits against the long canonical codes.  Returns exponent | length << 8.
__device__ __noinline__ __attribute__((unused)) uint32_t decode_long(uint32_t bits, const uint32_t *s_len, const uint32_t *s_code)
{
    uint32_t v = __brev(bits) >> 17;          // next 15 bits, first bit most significant
    uint32_t r = 15u << 8;                    // no match (corrupt stream): skip 15 bits, exponent 0
#pragma unroll 1
    for (int s = 0; s < 16; s++) {
        uint32_t ls = s_len[s];
        if (ls > TB && (v >> (15 - ls)) == s_code[s]) r = (uint32_t)s | (ls << 8);
    }
    return r;
}

// One symbol the careful way.  `bits`: stream bits from the current position
// (>= 15 valid).  Returns exponent | length << 8.
// LONG = false: the launch has no codeword longer than TB bits, so the table always answers (a blob that
// breaks the promise decodes to wrong bytes, in bounds) and the out-of-line matcher is compiled out.
template <bool LONG = true>
__device__ __forceinline__ uint32_t decode_one(uint32_t bits, const uint16_t *tbl, const uint32_t *s_len,
                                               const uint32_t *s_code)
{
    uint32_t e = tbl[bits & TBL_MASK];
    uint32_t l = (e & 7u) | ((e >> 12) & 8u);
    if constexpr (!LONG) return ((e >> 3) & 15u) | ((l ? l : 15u) << 8);
    if (__builtin_expect(l != 0, 1)) return ((e >> 3) & 15u) | (l << 8);
    return decode_long(bits, s_len, s_code);
}

// Second level for one pair: the table entry `e` at the bottom of `bits` (32
// valid stream bits) has no pair (the two codewords need more than TB bits, or
// the first one alone does).  Decodes the two symbols one at a time and returns
// them in `e` in pair-entry layout, their total length (up to 30) in `n`.
template <bool LONG = true>
__device__ __forceinline__ void pair_second_level(uint32_t bits, uint32_t &e, uint32_t &n, const uint16_t *tbl,
                                                  const uint32_t *s_len, const uint32_t *s_code)
{
    const uint32_t r1 = decode_one<LONG>(bits, tbl, s_len, s_code);
    const uint32_t l1 = r1 >> 8;
    const uint32_t r2 = decode_one<LONG>(bits >> l1, tbl, s_len, s_code);
    e = ((r1 & 15u) << 3) | ((r2 & 15u) << 11);
    n = l1 + (r2 >> 8);
}

// Builds the pair table and the per-symbol (length, code) arrays in LDS from
// the 16 code lengths.  `tmp` is TBL_ENTRIES u16 of scratch LDS.
__device__ __forceinline__ void build_symbol_arrays(uint64_t len_lo, uint64_t len_hi, uint32_t *s_len,
                                                    uint32_t *s_code, int tid)
{
    if (tid < 16) {
        uint32_t l = len_of(len_lo, len_hi, tid);
        uint32_t code = 0;
#pragma unroll
        for (int j = 0; j < 16; j++) {
            uint32_t lj = len_of(len_lo, len_hi, j);
            if (lj != 0 && lj < l) code += 1u << (l - lj);     // all shorter codes precede
            else if (lj == l && j < tid) code += 1;            // same length: by symbol value
        }
        s_len[tid] = l;
        s_code[tid] = code;
    }
}

__device__ __attribute__((unused)) void build_tables(uint64_t len_lo, uint64_t len_hi, uint16_t *tbl, uint32_t *s_len,
                                                     uint32_t *s_code, uint16_t *tmp, int tid, int nthreads)
{
    build_symbol_arrays(len_lo, len_hi, s_len, s_code, tid);
    for (int i = tid; i < TBL_ENTRIES; i += nthreads) tmp[i] = 0;
    __syncthreads();
    // single-symbol table: every index whose low bits spell the codeword (first bit = bit 0)
    for (int s = 0; s < 16; s++) {
        uint32_t l = s_len[s];
        if (l == 0 || l > TB) continue;
        uint32_t r = __brev(s_code[s]) >> (32 - l);
        uint32_t reps = 1u << (TB - l);
        for (uint32_t j = tid; j < reps; j += nthreads) tmp[r | (j << l)] = (uint16_t)(s | (l << 4));
    }
    __syncthreads();
    for (int idx = tid; idx < TBL_ENTRIES; idx += nthreads) {
        const uint32_t t1 = tmp[idx];
        const uint32_t l1 = t1 >> 4;
        const uint32_t t2 = l1 ? tmp[idx >> l1] : 0u;
        tbl[idx] = ecf8_pair_entry(t1 & 15u, l1, t2 & 15u, t2 >> 4);
    }
    __syncthreads();
}

// 32 stream bits in reading order (bit 0 = next bit to read) from LDS.
// DIR = +1: the bits [bp, bp+32);  DIR = -1: the bits bp-1, bp-2, ..., bp-32.
template <int DIR>
__device__ __forceinline__ uint32_t lds_window(const uint8_t *smem, uint32_t bp)
{
    const uint32_t p = DIR > 0 ? bp : bp - 32;
    const uint32_t aw = (p >> 3) & ~3u;
    const uint32_t d0 = *(const uint32_t *)(smem + aw);
    const uint32_t d1 = *(const uint32_t *)(smem + aw + 4);
    const uint32_t w = __builtin_amdgcn_alignbit(d1, d0, p);
    return DIR > 0 ? w : __brev(w);
}

// Second level of a decode step: some lane of the wave has a pair that needs more than TB bits.  wA, wB: the runs'
// 32-bit windows at pa, pb (one bit off, as in quad_step2), WA, WB: the same windows 64 bits long; e and n: the two
// entries of each run as looked up and their pair lengths, replaced by entries in pair layout and the lengths used.
// An entry without a pair still names its first symbol and that symbol's length (unless that codeword alone is
// longer than TB bits), and the pair's other symbol is the first symbol of the entry that many bits on.  The whole
// wave redoes both runs branch-free (a wave takes this path far more often than a lane needs it): three rounds of
// lookups, both runs side by side.
template <bool LONG>
__device__ __forceinline__ void second_level(const uint8_t *smem, const uint16_t *tbl, const uint32_t *s_len, const uint32_t *s_code,
                                             uint32_t pa, uint32_t pb, uint32_t wA, uint32_t wB, uint64_t WA, uint64_t WB,
                                             uint32_t &eA1, uint32_t &nA1, uint32_t &eA2, uint32_t &nA2,
                                             uint32_t &eB1, uint32_t &nB1, uint32_t &eB2, uint32_t &nB2)
{
    constexpr uint32_t OFF_MASK = TBL_MASK << 1;
    const uint8_t *tb = (const uint8_t *)tbl;
    {
        const uint32_t oA1 = eA1, oB1 = eB1, mA1 = nA1, mB1 = nB1;      // as looked up, for the lanes that start over below
        auto first_len = [](uint32_t e) { return (e & 7u) | ((e >> 12) & 8u); };
        auto two_firsts = [](uint32_t e, uint32_t x) { return (e & 0x78u) | ((x & 0x78u) << 8); };   // as a pair entry
        auto entry_at = [&](uint64_t W, uint32_t bits) { return (uint32_t) * (const uint16_t *)(tb + ((uint32_t)(W >> bits) & OFF_MASK)); };
        bool beyond = false;                  // LONG: a codeword longer than TB bits is in the way
        // first pairs (at most 28 bits, inside the 31 of the short windows)
        const uint32_t lA1 = first_len(eA1), lB1 = first_len(eB1);
        const uint32_t xA1 = *(const uint16_t *)(tb + ((wA >> lA1) & OFF_MASK));
        const uint32_t xB1 = *(const uint16_t *)(tb + ((wB >> lB1) & OFF_MASK));
        if (nA1 == 0) { eA1 = two_firsts(eA1, xA1); nA1 = lA1 + first_len(xA1); beyond |= lA1 == 0 || first_len(xA1) == 0; }
        if (nB1 == 0) { eB1 = two_firsts(eB1, xB1); nB1 = lB1 + first_len(xB1); beyond |= lB1 == 0 || first_len(xB1) == 0; }
        // second pairs, from where the first ones now end (at most 28 + 28 + TB bits from the windows' start)
        eA2 = entry_at(WA, nA1);
        eB2 = entry_at(WB, nB1);
        nA2 = (eA2 >> 7) & 15u;
        nB2 = (eB2 >> 7) & 15u;
        const uint32_t lA2 = first_len(eA2), lB2 = first_len(eB2);
        const uint32_t xA2 = entry_at(WA, nA1 + lA2);
        const uint32_t xB2 = entry_at(WB, nB1 + lB2);
        if (nA2 == 0) { eA2 = two_firsts(eA2, xA2); nA2 = lA2 + first_len(xA2); beyond |= lA2 == 0 || first_len(xA2) == 0; }
        if (nB2 == 0) { eB2 = two_firsts(eB2, xB2); nB2 = lB2 + first_len(xB2); beyond |= lB2 == 0 || first_len(xB2) == 0; }
        if constexpr (LONG) {
            // rarer than 2^-TB per symbol: such a lane starts over, symbol by symbol, with the matcher for long codewords
            if (__builtin_expect(beyond, 0)) {
                eA1 = oA1; nA1 = mA1;
                if (nA1 == 0) pair_second_level<true>(wA >> 1, eA1, nA1, tbl, s_len, s_code);   // 31 valid bits, 30 needed
                uint32_t w2 = lds_window<+1>(smem, pa + 1 + nA1);                                // fresh window after the first pair
                eA2 = tbl[w2 & TBL_MASK];
                nA2 = (eA2 >> 7) & 15u;
                if (nA2 == 0) pair_second_level<true>(w2, eA2, nA2, tbl, s_len, s_code);
                eB1 = oB1; nB1 = mB1;
                if (nB1 == 0) pair_second_level<true>(wB >> 1, eB1, nB1, tbl, s_len, s_code);
                w2 = lds_window<-1>(smem, pb + 31 - nB1);
                eB2 = tbl[w2 & TBL_MASK];
                nB2 = (eB2 >> 7) & 15u;
                if (nB2 == 0) pair_second_level<true>(w2, eB2, nB2, tbl, s_len, s_code);
            }
        }
    }
}

// One decode step of both runs of a lane: four symbols each = two table
// lookups each.  The two runs are independent, and the common path is one
// straight line, so their LDS round trips overlap; the second level for pairs
// that do not fit TB bits is one shared, rarely taken branch.  Returns the four
// exponent fields of each run in their output byte positions (other bits are
// noise the merge masks off) and moves the runs past the codewords.
// The runs' positions are kept one bit off, pa = (next bit of the forward run) - 1
// and pb = (one past the next bit of the backward run) - 31: the windows read at
// those positions are the stream bits shifted left by one, i.e. already the byte
// offset of a 16-bit table entry once masked.
// PAIRFIT: no codeword is longer than TB/2 bits, so every pair is in the table and
// the second level is compiled out (a blob that breaks the promise decodes to wrong
// bytes, in bounds).
template <bool PAIRFIT, bool LONG = true>
__device__ __forceinline__ void quad_step2(const uint8_t *smem, const uint16_t *tbl, const uint32_t *s_len,
                                           const uint32_t *s_code, uint32_t &pa, uint32_t &pb,
                                           uint32_t &outA, uint32_t &outB)
{
    constexpr uint32_t OFF_MASK = TBL_MASK << 1;
    const uint8_t *tb = (const uint8_t *)tbl;
    const uint32_t aA = (pa >> 3) & ~3u, aB = (pb >> 3) & ~3u;
    const uint32_t dA0 = *(const uint32_t *)(smem + aA), dA1 = *(const uint32_t *)(smem + aA + 4);
    const uint32_t dB0 = *(const uint32_t *)(smem + aB), dB1 = *(const uint32_t *)(smem + aB + 4);
    const uint32_t wA = __builtin_amdgcn_alignbit(dA1, dA0, pa);
    const uint32_t wB = __brev(__builtin_amdgcn_alignbit(dB1, dB0, pb));
    uint32_t eA1 = *(const uint16_t *)(tb + (wA & OFF_MASK));
    uint32_t eB1 = *(const uint16_t *)(tb + (wB & OFF_MASK));
    uint32_t nA1 = (eA1 >> 7) & 15u;
    uint32_t nB1 = (eB1 >> 7) & 15u;
    uint32_t eA2 = *(const uint16_t *)(tb + ((wA >> nA1) & OFF_MASK));    // >= 17 valid bits left in the window
    uint32_t eB2 = *(const uint16_t *)(tb + ((wB >> nB1) & OFF_MASK));
    uint32_t nA2 = (eA2 >> 7) & 15u;
    uint32_t nB2 = (eB2 >> 7) & 15u;
    // n1 == 0 makes the second lookup repeat the first, so n2 == 0 covers both pairs of a run
    if (!PAIRFIT && __builtin_expect(nA2 == 0 || nB2 == 0, 0)) {
        const uint32_t dA2 = *(const uint32_t *)(smem + aA + 8), dBm = *(const uint32_t *)(smem + aB - 4);
        second_level<LONG>(smem, tbl, s_len, s_code, pa, pb, wA, wB, wA | ((uint64_t)__builtin_amdgcn_alignbit(dA2, dA1, pa) << 32),
                           wB | ((uint64_t)__brev(__builtin_amdgcn_alignbit(dB0, dBm, pb)) << 32), eA1, nA1, eA2, nA2, eB1, nB1, eB2, nB2);
    }
    pa += nA1 + nA2;
    pb = pb - nB1 - nB2;
    // bytes 0,1 of the first entry and bytes 0,1 of the second
    outA = __builtin_amdgcn_perm(eA2, eA1, 0x05040100u);
    outB = __builtin_amdgcn_perm(eB2, eB1, 0x05040100u);
}

// The two runs of a lane with their windows held in registers: three consecutive dwords of the LDS image per run
// (the two a window is made of and the one the run moves into next).  A step then has two LDS round trips on
// its critical path, the two table lookups, instead of three: the dword that refills the spare is fetched at the
// end of a step and first needed at the end of the next one.  Positions are kept one bit off as in quad_step2.
struct HeldRuns {
    uint32_t pa, pb;           // forward run: next bit - 1; backward run: one past its next bit - 31
    uint32_t a0, a1, a2;       // dwords at A, A + 4, A + 8 with A = (pa / 8) & ~3
    uint32_t bm, b0, b1;       // dwords at B - 4, B, B + 4 with B = (pb / 8) & ~3

    __device__ __forceinline__ void begin(const uint8_t *smem, uint32_t pa_, uint32_t pb_)
    {
        pa = pa_;
        pb = pb_;
        const uint32_t A = (pa >> 3) & ~3u, B = (pb >> 3) & ~3u;
        a0 = *(const uint32_t *)(smem + A);
        a1 = *(const uint32_t *)(smem + A + 4);
        a2 = *(const uint32_t *)(smem + A + 8);
        bm = *(const uint32_t *)(smem + B - 4);
        b0 = *(const uint32_t *)(smem + B);
        b1 = *(const uint32_t *)(smem + B + 4);
    }
};

// quad_step2 over held windows, for launches whose pairs always fit the table (PAIRFIT; with a second level in
// the way the general kernels measured faster on windows fetched per step).  A step moves a run by at most 28 bits,
// so by at most one dword: bit 5 of the position tells.  The refill reads past the stage of the last wave by up to
// 8 bytes and before the first one by up to 4: the caller's LDS map has something there.
__device__ __forceinline__ void quad_step_held(const uint8_t *smem, const uint16_t *tbl, HeldRuns &r, uint32_t &outA, uint32_t &outB)
{
    constexpr uint32_t OFF_MASK = TBL_MASK << 1;
    const uint8_t *tb = (const uint8_t *)tbl;
    const uint32_t wA = __builtin_amdgcn_alignbit(r.a1, r.a0, r.pa);
    const uint32_t wB = __brev(__builtin_amdgcn_alignbit(r.b1, r.b0, r.pb));
    const uint32_t eA1 = *(const uint16_t *)(tb + (wA & OFF_MASK));
    const uint32_t eB1 = *(const uint16_t *)(tb + (wB & OFF_MASK));
    const uint32_t nA1 = (eA1 >> 7) & 15u;
    const uint32_t nB1 = (eB1 >> 7) & 15u;
    const uint32_t eA2 = *(const uint16_t *)(tb + ((wA >> nA1) & OFF_MASK));    // >= 17 valid bits left in the window
    const uint32_t eB2 = *(const uint16_t *)(tb + ((wB >> nB1) & OFF_MASK));
    const uint32_t pa = r.pa + nA1 + ((eA2 >> 7) & 15u);
    const uint32_t pb = r.pb - nB1 - ((eB2 >> 7) & 15u);
    const uint32_t ldA = *(const uint32_t *)(smem + ((pa >> 3) & ~3u) + 8);
    const uint32_t ldB = *(const uint32_t *)(smem + ((pb >> 3) & ~3u) - 4);
    const bool upA = ((pa ^ r.pa) & 32u) != 0, downB = ((pb ^ r.pb) & 32u) != 0;
    r.a0 = upA ? r.a1 : r.a0;
    r.a1 = upA ? r.a2 : r.a1;
    r.a2 = ldA;                     // the dword at the new A + 8 either way
    r.b1 = downB ? r.b0 : r.b1;
    r.b0 = downB ? r.bm : r.b0;
    r.bm = ldB;
    r.pa = pa;
    r.pb = pb;
    outA = __builtin_amdgcn_perm(eA2, eA1, 0x05040100u);
    outB = __builtin_amdgcn_perm(eB2, eB1, 0x05040100u);
}

// byte = exponent<<3 | sign<<7 | mantissa  (Algorithm 1, byte assembly) for one
// 16-byte piece: dw = four dwords of exponent fields, pl = the piece's 8 bytes
// of the nibble plane (byte j of a dword: low nibble element j, high nibble
// element j + 4 of that 8-element group).
// (a & mask) | (b & ~mask) in one v_bitop3_b32 (truth table over a = 0xF0, b = 0xCC, mask = 0xAA);
// written as plain C the compiler expands the nested selects below into five operations per dword
__device__ __forceinline__ uint32_t bit_select(uint32_t mask, uint32_t a, uint32_t b)
{
    return __builtin_amdgcn_bitop3_b32(a, b, mask, 0xE4);
}

__device__ __forceinline__ u32x4 merge_piece(const uint32_t dw[4], u32x2 pl)
{
    const uint32_t p0 = pl.x, p1 = pl.y;
    // per byte: bits 0..2 mantissa, bit 7 sign (bits 3..6 of the inner select are overwritten)
    u32x4 d;
    d.x = bit_select(EXP_MASK, dw[0], bit_select(0x07070707u, p0, p0 << 4));
    d.y = bit_select(EXP_MASK, dw[1], bit_select(0x07070707u, p0 >> 4, p0));
    d.z = bit_select(EXP_MASK, dw[2], bit_select(0x07070707u, p1, p1 << 4));
    d.w = bit_select(EXP_MASK, dw[3], bit_select(0x07070707u, p1 >> 4, p1));
    return d;
}

// 32 stream bits in reading order straight from HBM (generic pass).  `bit` is
// relative to the 4-byte aligned pointer sp; DIR as in lds_window.
template <int DIR>
__device__ __forceinline__ uint32_t global_window(const GLOBAL uint8_t *sp, uint64_t bit)
{
    if (DIR > 0) {
        const GLOBAL uint32_t *q = (const GLOBAL uint32_t *)(sp + ((bit >> 3) & ~3ull));
        return __builtin_amdgcn_alignbit(q[1], q[0], (uint32_t)bit);
    }
    if (bit < 32) {   // fewer than 32 bits below: the missing ones are never consumed
        const uint32_t d0 = *(const GLOBAL uint32_t *)sp;
        return __brev(bit ? d0 << (32 - (uint32_t)bit) : 0u);
    }
    const uint64_t p = bit - 32;
    const GLOBAL uint32_t *q = (const GLOBAL uint32_t *)(sp + ((p >> 3) & ~3ull));
    return __brev(__builtin_amdgcn_alignbit(q[1], q[0], (uint32_t)p));
}

int device_cus()
{
    static std::mutex m;
    static int cus[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return -1;
    std::lock_guard<std::mutex> lk(m);
    if (cus[dev] == 0) {
        hipDeviceProp_t p;
        if (hipGetDeviceProperties(&p, dev) != hipSuccess) return -1;
        cus[dev] = p.multiProcessorCount > 0 ? p.multiProcessorCount : 1;
    }
    return cus[dev];
}

} // namespace

#endif
