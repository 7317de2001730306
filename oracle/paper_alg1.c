/*
 * ECF8 CPU oracle, part 3 -- TEST INFRASTRUCTURE ONLY.
 *
 * The paper's own container and decoder, emulated on the CPU with the threads
 * of a block run one after another: cascaded 8-bit lookup tables (Section 3.1,
 * "Hierarchical lookup table construction"), per-thread 4-bit gaps and
 * per-block output positions (Section 3.1, "Encoding and synchronization
 * metadata generation"; Table 4), and the two-phase block decoder
 * (Algorithm 1) with B = 8 bytes per thread.  Its only job is to show that the
 * readings this build takes of the garbled passages are mutually consistent:
 * the emulator must give back the input bytes.
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
 *  - the stream is zero padded so the 10-byte loads of the last block stay
 *    in bounds, and symbols decoded from padding are clipped by n_elem.
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

#define PB 8 /* B: bytes per thread window, from "B + 2 = 10" in Algorithm 1 */

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

typedef struct {
    uint64_t L; /* 64-bit sliding window, oldest bit most significant */
    uint32_t S; /* 16-bit tail */
    uint32_t f; /* bits consumed from the head */
} tstate;

static void t_init(tstate *st, const uint8_t *encoded, uint64_t tg, uint32_t g)
{
    const uint8_t *lb = encoded + tg * PB; /* localbf: B + 2 bytes */
    st->L = 0;
    for (int i = 0; i < 8; i++) st->L = (st->L << 8) | lb[i];
    st->S = ((uint32_t)lb[8] << 8) | lb[9];
    st->L <<= g;
    st->f = g;
}

/* one symbol through the cascaded table; returns its length, 0 on a bad table */
static uint32_t t_step(tstate *st, const uint8_t *lut, uint32_t n_luts, uint32_t *x_out)
{
    uint32_t x = lut[st->L >> 56];
    if (x >= 240) x = lut[256 * (256 - x) + ((st->L >> 48) & 255)];
    uint32_t bl = lut[256 * (n_luts - 1) + x];
    st->L <<= bl;
    st->f += bl;
    *x_out = x;
    return bl;
}

/* Algorithm 1, all blocks, threads of a block in sequence. */
int orc_paper_alg1_decode(const uint8_t *lut, uint32_t n_luts, const uint8_t *encoded,
                          uint64_t n_bytes, const uint8_t *packed, const int64_t *outpos,
                          const uint8_t *gaps, uint64_t n_blocks, uint32_t T,
                          uint64_t n_elem, uint8_t *outputs)
{
    (void)n_bytes;
    uint64_t *accum = (uint64_t *)malloc(((uint64_t)T + 1) * sizeof(uint64_t));
    uint32_t *cnt = (uint32_t *)malloc((uint64_t)T * sizeof(uint32_t));
    if (!accum || !cnt) { free(accum); free(cnt); return ORC_E_CAPACITY; }
    int rc = ORC_OK;
    for (uint64_t b = 0; b < n_blocks && rc == ORC_OK; b++) {
        /* phase 1: count the codewords that start inside each thread's window */
        for (uint32_t t = 0; t < T && rc == ORC_OK; t++) {
            uint64_t tg = b * T + t;
            uint32_t g = (gaps[tg / 2] >> (4 - (tg % 2) * 4)) & 0x0f;
            tstate st;
            uint32_t x, c = 0;
            t_init(&st, encoded, tg, g);
            while (st.f < 16) {
                if (t_step(&st, lut, n_luts, &x) == 0) { rc = ORC_E_CODE; break; }
                c++;
            }
            if (rc) break;
            st.L |= (uint64_t)st.S << (st.f - 16);
            st.f -= 16;
            while (2 + st.f / 8 < PB) {
                if (t_step(&st, lut, n_luts, &x) == 0) { rc = ORC_E_CODE; break; }
                c++;
            }
            cnt[t] = c;
        }
        if (rc) break;
        /* block prefix sum: exclusive starts offset by outpos[b] */
        accum[0] = (uint64_t)outpos[b];
        for (uint32_t t = 0; t < T; t++) accum[t + 1] = accum[t] + cnt[t];
        uint64_t obase = accum[0];
        uint64_t wb_len = (uint64_t)outpos[b + 1] - (uint64_t)outpos[b];
        uint8_t *writebf = (uint8_t *)malloc(wb_len ? wb_len : 1);
        if (!writebf) { rc = ORC_E_CAPACITY; break; }
        /* phase 2: decode again, merge sign/mantissa, stage in writebf */
        for (uint32_t t = 0; t < T && rc == ORC_OK; t++) {
            uint64_t tg = b * T + t;
            uint32_t g = (gaps[tg / 2] >> (4 - (tg % 2) * 4)) & 0x0f;
            uint64_t ostart = accum[t];
            uint64_t oend = ostart + cnt[t];
            if (oend > n_elem) oend = n_elem;
            tstate st;
            uint32_t x;
            int stitched = 0;
            t_init(&st, encoded, tg, g);
            while (ostart < oend) {
                if (!stitched && st.f >= 16) {
                    st.L |= (uint64_t)st.S << (st.f - 16);
                    st.f -= 16;
                    stitched = 1;
                }
                if (t_step(&st, lut, n_luts, &x) == 0) { rc = ORC_E_CODE; break; }
                uint32_t q = (uint32_t)packed[ostart / 2] << ((ostart % 2) * 4);
                uint8_t byte = (uint8_t)((x << 3) | (q & 0x80) | ((q >> 4) & 0x07));
                if (ostart - obase >= wb_len) { rc = ORC_E_META; break; }
                writebf[ostart - obase] = byte;
                ostart++;
            }
        }
        /* write-back */
        if (rc == ORC_OK) memcpy(outputs + obase, writebf, wb_len);
        free(writebf);
    }
    free(accum);
    free(cnt);
    return rc;
}
