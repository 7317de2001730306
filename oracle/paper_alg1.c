/*
 * ECF8 CPU oracle, part 3 -- TEST INFRASTRUCTURE ONLY.
 *
 * The paper's own container and block decoder on the CPU, the threads of a
 * block run one after another: cascaded 8-bit lookup tables (Section 3.1,
 * "Hierarchical lookup table construction"), per-thread 4-bit gaps and
 * per-block output positions (Section 3.1, "Encoding and synchronization
 * metadata generation"; Table 4), and the two-phase block decoder
 * (Algorithm 1) with B = 8 bytes per thread, stated through the meaning of
 * the metadata and run on the oracle's bit-serial tree walk; the cascaded
 * table is checked against that walk on every prefix on its own.  Its only
 * job is to show that the readings this build takes of the garbled passages
 * are mutually consistent: gaps land on codeword starts, per-thread counts
 * add up to the block's share, and the decoder gives back the input bytes.
 *
 * Readings (each stated again where it is used):
 *  - a table entry holds a symbol when some codeword is a PREFIX of the
 *    path-so-far followed by the entry's byte (short codes are replicated);
 *  - pointer entries hold 256 - (sub-table index), sub-tables are numbered
 *    from 1, the length table is the last row;
 *  - thread t's gap is the distance from the start of its 8B-bit window to the
 *    first codeword that STARTS inside or after it (0..15), zero for windows
 *    past the end of the stream;
 *  - outpos[b] counts the codewords that start before block b's first bit;
 *  - the stream is zero padded past the last block's windows, and symbols
 *    decoded from padding are clipped by n_elem.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_NSYM 16
#define ORC_MSB_FIRST 0
#define ORC_OK 0
#define ORC_E_ARG (-1)
#define ORC_E_FORMAT (-2)
#define ORC_E_CAPACITY (-3)
#define ORC_E_CODE (-4)
#define ORC_E_META (-5)

#define PB 8 /* B: bytes of the stream per thread (Algorithm 1 loads B + 2 of them, ten) */

void orc_split(uint8_t v, uint8_t *s, uint8_t *e, uint8_t *m);
void orc_histogram(const uint8_t *x, uint64_t n, uint64_t freq[ORC_NSYM]);
int orc_huffman_lengths(const uint64_t freq[ORC_NSYM], uint8_t len[ORC_NSYM]);
int orc_canonical_codes(const uint8_t len[ORC_NSYM], uint16_t code[ORC_NSYM]);
uint64_t orc_stream_bits(const uint64_t freq[ORC_NSYM], const uint8_t len[ORC_NSYM]);
int orc_encode_exponents(const uint8_t *x, uint64_t n, const uint8_t len[ORC_NSYM],
                         const uint16_t code[ORC_NSYM], int order, uint8_t *stream,
                         uint64_t stream_cap_bytes, uint64_t *nbits_out,
                         uint64_t mark_every, uint64_t *marks);
void orc_pack_nibbles_paper(const uint8_t *x, uint64_t n, uint8_t *packed);
uint8_t orc_join(uint8_t s, uint8_t e, uint8_t m);
int orc_decode_symbols_dir(const uint8_t *stream, int64_t start, int dir, int64_t lo, int64_t hi,
                           int order, const uint8_t len[ORC_NSYM], uint64_t n, uint8_t *sym_out,
                           int64_t *next);

/* Cascaded decode table + length table with W-bit sub-tables (the paper uses
 * W = 8; Figure 2 illustrates the construction with W = 2).  Row 0 is the
 * root; rows 1..k the sub-tables, one per distinct first W bits of a codeword
 * longer than W bits; row k+1 the length table L[x].  Rows have 2^W entries.
 * Two levels only, i.e. code lengths up to 2W.  lut must hold 18 rows. */
int orc_paper_build_lut_w(const uint8_t len[ORC_NSYM], const uint16_t code[ORC_NSYM],
                          uint32_t W, uint8_t *lut, uint32_t *n_luts_out)
{
    uint32_t n_sub = 0;
    uint32_t R = 1u << W; /* entries per row */
    if (W < 1 || W > 8) return ORC_E_ARG;
    memset(lut, 0, 18 * R);
    for (int s = 0; s < ORC_NSYM; s++) {
        uint32_t l = len[s];
        if (l == 0) continue;
        if (l > 2 * W) return ORC_E_ARG;
        if (l <= W) {
            /* every W-bit pattern that starts with this codeword resolves to s */
            uint32_t lo = (uint32_t)code[s] << (W - l);
            for (uint32_t j = 0; j < (1u << (W - l)); j++) lut[lo + j] = (uint8_t)s;
        } else {
            uint32_t p = (uint32_t)code[s] >> (l - W);
            uint32_t idx;
            if (lut[p] >= 240) idx = 256u - lut[p];
            else {
                idx = ++n_sub;
                if (idx > 16) return ORC_E_CODE;
                lut[p] = (uint8_t)(256u - idx); /* pointer value 256 - index */
            }
            uint32_t rest = (uint32_t)code[s] & ((1u << (l - W)) - 1);
            uint32_t lo = rest << (2 * W - l);
            for (uint32_t j = 0; j < (1u << (2 * W - l)); j++) lut[R * idx + lo + j] = (uint8_t)s;
        }
    }
    uint32_t n_luts = n_sub + 2;
    for (int s = 0; s < ORC_NSYM && s < (int)R; s++) lut[R * (n_luts - 1) + s] = len[s];
    *n_luts_out = n_luts;
    return ORC_OK;
}

int orc_paper_build_lut(const uint8_t len[ORC_NSYM], const uint16_t code[ORC_NSYM],
                        uint8_t *lut, uint32_t *n_luts_out)
{
    return orc_paper_build_lut_w(len, code, 8, lut, n_luts_out);
}

/* Sizes the caller must provide for orc_paper_encode. */
void orc_paper_sizes(uint64_t stream_bits, uint32_t T, uint64_t *n_bytes, uint64_t *n_blocks,
                     uint64_t *encoded_alloc, uint64_t *gaps_bytes)
{
    *n_bytes = (stream_bits + 7) / 8;
    *n_blocks = (*n_bytes + (uint64_t)T * PB - 1) / ((uint64_t)T * PB);
    if (*n_blocks == 0) *n_blocks = 1;
    *encoded_alloc = *n_blocks * T * PB + 2;
    *gaps_bytes = (*n_blocks * T + 1) / 2;
}

/* Encoder side of the paper's container. */
int orc_paper_encode(const uint8_t *x, uint64_t n, uint32_t T,
                     uint8_t len[ORC_NSYM], uint8_t *lut, uint32_t *n_luts,
                     uint8_t *encoded, uint64_t encoded_alloc, uint64_t *n_bytes_out,
                     uint8_t *packed, int64_t *outpos, uint8_t *gaps, uint64_t *n_blocks_out)
{
    uint64_t freq[ORC_NSYM];
    uint16_t code[ORC_NSYM];
    if (n == 0 || T == 0) return ORC_E_ARG;
    orc_histogram(x, n, freq);
    int rc = orc_huffman_lengths(freq, len);
    if (rc < 0) return rc;
    rc = orc_canonical_codes(len, code);
    if (rc) return rc;
    rc = orc_paper_build_lut(len, code, lut, n_luts);
    if (rc) return rc;

    uint64_t bits = orc_stream_bits(freq, len);
    uint64_t n_bytes, n_blocks, need, gbytes;
    orc_paper_sizes(bits, T, &n_bytes, &n_blocks, &need, &gbytes);
    if (need > encoded_alloc) return ORC_E_CAPACITY;
    memset(encoded, 0, need);
    uint64_t *start = (uint64_t *)malloc((n + 1) * sizeof(uint64_t));
    if (!start) return ORC_E_CAPACITY;
    uint64_t got = 0;
    rc = orc_encode_exponents(x, n, len, code, ORC_MSB_FIRST, encoded, need, &got, 1, start);
    if (rc == ORC_OK && got != bits) rc = ORC_E_FORMAT;
    if (rc) { free(start); return rc; }
    start[n] = bits;
    orc_pack_nibbles_paper(x, n, packed);

    /* gaps: thread t_g owns bits [64 t_g, 64 t_g + 64) */
    memset(gaps, 0, gbytes);
    uint64_t j = 0; /* first symbol whose start >= window start */
    for (uint64_t tg = 0; tg < n_blocks * T; tg++) {
        uint64_t w0 = tg * PB * 8;
        while (j < n && start[j] < w0) j++;
        uint32_t g = 0;
        if (j < n) {
            uint64_t d = start[j] - w0;
            if (d > 15) { free(start); return ORC_E_META; } /* cannot happen: lengths <= 16 */
            g = (uint32_t)d;
        } else if (bits > w0) {
            /* the last codeword reaches into this window: decoding resumes after it */
            uint64_t d = bits - w0;
            g = d > 15 ? 15 : (uint32_t)d; /* d <= 15 for the same reason */
        }
        if ((tg & 1) == 0) gaps[tg / 2] |= (uint8_t)(g << 4);
        else gaps[tg / 2] |= (uint8_t)g;
    }
    /* outpos: codewords starting before each block's first bit */
    j = 0;
    for (uint64_t b = 0; b < n_blocks; b++) {
        uint64_t w0 = b * T * PB * 8;
        while (j < n && start[j] < w0) j++;
        outpos[b] = (int64_t)j;
    }
    outpos[n_blocks] = (int64_t)n;
    free(start);
    *n_bytes_out = n_bytes;
    *n_blocks_out = n_blocks;
    return ORC_OK;
}

/* One codeword through the cascaded table (Section 3.1, hierarchical lookup table construction): the root
 * row is indexed by the next W stream bits; an entry of 240 or more stands for sub-table 256 - entry,
 * indexed by the W bits after those; the last row holds the length of every symbol.  `bits` holds the
 * next 2W stream bits, first bit most significant. */
int orc_paper_lut_lookup(const uint8_t *lut, uint32_t n_luts, uint32_t W, uint32_t bits, uint32_t *sym,
                         uint32_t *length)
{
    uint32_t R = 1u << W;
    uint32_t x = lut[(bits >> W) & (R - 1)];
    if (x >= 240) {
        uint32_t sub = 256u - x;
        if (sub + 1 >= n_luts) return ORC_E_CODE;
        x = lut[R * sub + (bits & (R - 1))];
    }
    if (x >= ORC_NSYM) return ORC_E_CODE;
    *sym = x;
    *length = lut[R * (n_luts - 1) + x];
    return *length ? ORC_OK : ORC_E_CODE;
}

/* The cascaded table against the code itself: every 16-bit prefix is sent through the table and through
 * the bit-serial tree walk; returns the number of prefixes on which symbol or length differ (prefixes
 * no codeword matches, possible only for an incomplete code, are skipped). */
int64_t orc_paper_lut_mismatches(const uint8_t len[ORC_NSYM], const uint8_t *lut, uint32_t n_luts)
{
    int64_t bad = 0;
    for (uint32_t v = 0; v < 65536; v++) {
        uint8_t two[2] = {(uint8_t)(v >> 8), (uint8_t)v};
        uint8_t s_walk;
        int64_t next = 0;
        if (orc_decode_symbols_dir(two, 0, +1, 0, 16, ORC_MSB_FIRST, len, 1, &s_walk, &next) != ORC_OK) continue;
        uint32_t s_lut = 0, l_lut = 0;
        if (orc_paper_lut_lookup(lut, n_luts, 8, v, &s_lut, &l_lut) != ORC_OK || s_lut != s_walk ||
            l_lut != (uint32_t)next)
            bad++;
    }
    return bad;
}

static uint32_t gap_of(const uint8_t *gaps, uint64_t tg) { return (tg % 2 == 0) ? gaps[tg / 2] >> 4 : gaps[tg / 2] & 15u; }

/* Block decoder over the paper's container (Algorithm 1), stated through what the metadata means rather
 * than through the listing's window arithmetic.  Thread tg owns the codewords whose first bit lies in
 * its window [64 tg, 64 tg + 64): the first of them starts `gap` bits into the window, and the walk goes
 * on codeword by codeword (bit-serial, through the code tree) until a codeword would start at or past
 * the window's end.  Phase 1 only counts; the block's exclusive prefix sum of the counts on top of
 * outpos[b] gives each thread its first output; phase 2 walks again and writes byte = exponent<<3 |
 * sign<<7 | mantissa for outputs below n_elem.  Checked on the way (ORC_E_META when violated):
 *   - a thread's walk ends exactly where the next thread's gap says its first codeword starts, so
 *     every gap lands on a codeword start;
 *   - a block's counts add up to outpos[b+1] - outpos[b] (once clipped at n_elem: the zero padding
 *     behind the stream decodes to codewords of its own). */
int orc_paper_window_decode(const uint8_t len[ORC_NSYM], const uint8_t *encoded, uint64_t encoded_alloc,
                            const uint8_t *packed, const int64_t *outpos, const uint8_t *gaps,
                            uint64_t n_blocks, uint32_t T, uint64_t n_elem, uint8_t *outputs)
{
    const int64_t limit = (int64_t)encoded_alloc * 8;
    uint32_t *cnt = (uint32_t *)malloc((uint64_t)T * sizeof(uint32_t));
    if (!cnt) return ORC_E_CAPACITY;
    int rc = ORC_OK;
    for (uint64_t b = 0; b < n_blocks && rc == ORC_OK; b++) {
        /* phase 1 */
        uint64_t total = 0;
        for (uint32_t t = 0; t < T && rc == ORC_OK; t++) {
            const uint64_t tg = b * T + t;
            const int64_t w0 = (int64_t)tg * PB * 8, w1 = w0 + PB * 8;
            int64_t pos = w0 + gap_of(gaps, tg);
            uint32_t c = 0;
            while (pos < w1) {
                uint8_t sym;
                if (orc_decode_symbols_dir(encoded, pos, +1, 0, limit, ORC_MSB_FIRST, len, 1, &sym, &pos)) { rc = ORC_E_CODE; break; }
                c++;
            }
            cnt[t] = c;
            total += c;
            if (rc == ORC_OK && tg + 1 < n_blocks * T && pos != w1 + (int64_t)gap_of(gaps, tg + 1) &&
                (uint64_t)outpos[b] + total < n_elem)      /* (inside the padding the gaps are zero) */
                rc = ORC_E_META;
        }
        if (rc) break;
        uint64_t end = (uint64_t)outpos[b] + total;
        if (end > n_elem) end = n_elem;
        if (end != (uint64_t)outpos[b + 1]) { rc = ORC_E_META; break; }
        /* phase 2 */
        uint64_t o = (uint64_t)outpos[b];
        for (uint32_t t = 0; t < T && rc == ORC_OK; t++) {
            const uint64_t tg = b * T + t;
            int64_t pos = (int64_t)tg * PB * 8 + gap_of(gaps, tg);
            uint64_t o_end = o + cnt[t];
            for (uint64_t i = o; i < o_end; i++) {
                uint8_t sym;
                if (orc_decode_symbols_dir(encoded, pos, +1, 0, limit, ORC_MSB_FIRST, len, 1, &sym, &pos)) { rc = ORC_E_CODE; break; }
                if (i >= n_elem) continue;
                const uint8_t pk = packed[i / 2];
                const uint8_t q = (i % 2 == 0) ? (uint8_t)(pk >> 4) : (uint8_t)(pk & 15);
                outputs[i] = orc_join((uint8_t)(q >> 3), sym, (uint8_t)(q & 7));
            }
            o = o_end;
        }
    }
    free(cnt);
    return rc;
}
