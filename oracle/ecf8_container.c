/*
 * ECF8 CPU oracle, part 2 -- TEST INFRASTRUCTURE ONLY.
 *
 * Slow reader and writer of the chunked ECF8 container, written from the
 * container's format description alone (byte offsets below), sharing no code
 * or header with the product.  The container replaces the paper's
 * synchronisation metadata (Section 3.1: per-thread gaps and per-block output
 * positions, Table 4 "gaps"/"outpos") by a sampling of codeword start
 * positions, and orders the codewords inside a chunk lane by lane so that the
 * 64 lanes of a wavefront produce adjacent output in the same step; the stream
 * is still one continuous concatenation of codewords (Section 3.1).
 *
 * Container (all integers little-endian):
 *   header, 256 bytes:
 *     0   u32 magic 0x38464345 ("ECF8")     4   u32 version (1)
 *     8   u64 total_size                    16  u64 n_elem
 *     24  u64 rows                          32  u64 cols
 *     40  u32 lane_syms N                   44  u16 table_bits (0 or 14)
 *     46  u8  group_chunks G (power of two, 1..64)
 *     47  u8  tile_rows (0: linear layout; 16: row-tiled layout, needs G = 1,
 *             rows % 16 = 0, cols % 4N = 0)
 *     48  u64 n_chunks = ceil(n_elem/(64N)) 56  u64 stream_bits
 *     64  u8  code_len[16]
 *     80  u64 off_chunk_bit   88 u64 off_lane_bits
 *     96  u64 off_stream      104 u64 off_plane
 *     112 u64 stream_bytes    120 u64 plane_bytes
 *     128 u64 freq[16]
 *   table     : only when table_bits = 14: u16[2^14] directly after the header, a
 *               decoder lookup table the reader only verifies.  Entry i
 *               describes the codewords spelled by the bits of i, bit 0 first:
 *               (s1, l1) the first codeword's symbol and length, (s2, l2) the
 *               next one's; bits 3..6 = s1, bits 0..2 = l1 & 7, bit 15 = l1 >> 3,
 *               and if l1 + l2 <= 14: bits 11..14 = s2, bits 7..10 = l1 + l2,
 *               else those are 0; 0 if the first codeword needs more than 14 bits
 *   chunk_bit : u64[n_chunks+1]   start bit of the first codeword of chunk c;
 *                                 last entry = stream_bits
 *   lane_bits : u16[n_chunks*64]  total code bits of lane l of chunk c
 *   stream    : stream_bytes bytes; stream bit i = bit (i&7) of byte (i>>3);
 *               lanes follow each other chunk by chunk, lane by lane; lane l
 *               of chunk c owns bits [S, S + lane_bits) where S = chunk_bit[c]
 *               + the lane_bits of the chunk's earlier lanes.  The k-th
 *               symbol (k = 0..N-1) of the lane is element
 *               base(c) + (k/16)*stride(c) + l*16 + k%16, where, with
 *               F = n_elem / (G*64N) whole groups of G chunks,
 *                 c <  G*F: base = (c - c%G)*64N + (c%G)*1024, stride = G*1024
 *                 c >= G*F: base = c*64N,                      stride = 1024
 *               (inside a whole group the 1024-element blocks of its G chunks
 *               alternate; the rest of the tensor is chunk after chunk);
 *               elements >= n_elem do not exist and are skipped.
 *               Row-tiled layout: the matrix is cut into blocks of 16 rows x
 *               4N columns, numbered along a row of blocks first; chunk c is
 *               block c.  Lane l works on row l%16 of the block; its k-th
 *               symbol is column 64*(k/16) + 16*(l/16) + k%16 of the block
 *               (element index = row*cols + column of the whole matrix).  Symbols k < N/2 are coded FORWARD from
 *               bit S upwards (a codeword's first = most significant bit at
 *               the lowest position); symbols k >= N/2 are coded BACKWARD from
 *               bit S + lane_bits - 1 downwards (first bit at the highest
 *               position); the two runs meet exactly.  Codes are canonical
 *               from code_len, ordered by (length, symbol); zero padded,
 *               stream_bytes = roundup16(ceil(stream_bits/8) + 8)
 *   plane     : sign/mantissa nibbles q = sign<<3 | mantissa (Table 4,
 *               "packed"), regrouped: element i sits in byte
 *               (i/8)*4 + (i%4), low nibble when (i%8) < 4, else high
 *               nibble; plane_bytes = n_chunks*32N, zero padded
 *   every section starts at a multiple of 256 bytes.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_NSYM 16
#define ORC_LSB_FIRST 1
#define ORC_OK 0
#define ORC_E_ARG (-1)
#define ORC_E_FORMAT (-2)
#define ORC_E_CAPACITY (-3)
#define ORC_E_CODE (-4)
#define ORC_E_META (-5)

/* from ecf8_oracle.c */
void orc_split(uint8_t v, uint8_t *s, uint8_t *e, uint8_t *m);
uint8_t orc_join(uint8_t s, uint8_t e, uint8_t m);
void orc_histogram(const uint8_t *x, uint64_t n, uint64_t freq[ORC_NSYM]);
int orc_huffman_lengths(const uint64_t freq[ORC_NSYM], uint8_t len[ORC_NSYM]);
int orc_huffman_lengths_limited(const uint64_t freq[ORC_NSYM], int lmax, uint8_t len[ORC_NSYM]);
int orc_canonical_codes(const uint8_t len[ORC_NSYM], uint16_t code[ORC_NSYM]);
uint64_t orc_stream_bits(const uint64_t freq[ORC_NSYM], const uint8_t len[ORC_NSYM]);
int orc_decode_symbols_dir(const uint8_t *stream, int64_t start, int dir, int64_t lo, int64_t hi,
                           int order, const uint8_t len[ORC_NSYM], uint64_t n, uint8_t *sym_out,
                           int64_t *next);

static uint64_t rd64(const uint8_t *p)
{
    uint64_t v = 0;
    for (int i = 7; i >= 0; i--) v = (v << 8) | p[i];
    return v;
}
static uint32_t rd32(const uint8_t *p)
{
    return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24);
}
static uint32_t rd16(const uint8_t *p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8); }
static void wr64(uint8_t *p, uint64_t v) { for (int i = 0; i < 8; i++) p[i] = (uint8_t)(v >> (8 * i)); }
static void wr32(uint8_t *p, uint32_t v) { for (int i = 0; i < 4; i++) p[i] = (uint8_t)(v >> (8 * i)); }
static void wr16(uint8_t *p, uint32_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); }
static uint64_t up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

/* element coded by the k-th symbol of lane l of chunk c */
typedef struct { uint32_t N, G, tile_rows; uint64_t n, cols; } orc_layout;

static uint64_t lane_element(const orc_layout *L, uint64_t c, uint64_t l, uint64_t k)
{
    uint64_t chunk = 64ull * L->N;
    if (L->tile_rows) {
        uint64_t block_cols = 4ull * L->N;
        uint64_t blocks_per_row = L->cols / block_cols;
        uint64_t block_row = c / blocks_per_row, block_col = c % blocks_per_row;
        uint64_t row = block_row * 16 + l % 16;
        uint64_t col = block_col * block_cols + 64 * (k / 16) + 16 * (l / 16) + k % 16;
        return row * L->cols + col;
    }
    uint64_t whole_groups = L->n / (L->G * chunk);
    uint64_t base, stride;
    if (c < L->G * whole_groups) {
        uint64_t slot = c % L->G;
        base = (c - slot) * chunk + slot * 1024;
        stride = (uint64_t)L->G * 1024;
    } else {
        base = c * chunk;
        stride = 1024;
    }
    return base + (k / 16) * stride + l * 16 + (k % 16);
}

static int layout_ok(const orc_layout *L, uint64_t rows)
{
    if (L->G == 0 || L->G > 64 || (L->G & (L->G - 1))) return 0;
    if (L->tile_rows == 0) return 1;
    return L->tile_rows == 16 && L->G == 1 && rows % 16 == 0 && L->cols % (4ull * L->N) == 0;
}

static uint64_t plane_byte_index(uint64_t i) { return (i / 8) * 4 + (i % 4); }
static int plane_is_high(uint64_t i) { return (i % 8) >= 4; }

/* Size in bytes the container of an n-element tensor takes when the stream
 * has `stream_bits` bits and lanes hold N symbols. */
uint64_t orc_container_size(uint64_t n, uint64_t stream_bits, uint32_t N)
{
    uint64_t chunk = 64ull * N;
    uint64_t n_chunks = (n + chunk - 1) / chunk;
    uint64_t sz = 256;
    sz = up(sz, 256) + 8 * (n_chunks + 1);
    sz = up(sz, 256) + 2 * n_chunks * 64;
    sz = up(sz, 256) + up((stream_bits + 7) / 8 + 8, 16);
    sz = up(sz, 256) + n_chunks * 32ull * N;
    return up(sz, 256);
}

/* Writer: encodes x (rows*cols raw E4M3 bytes) into blob (capacity cap).
 * Follows Section 3.1 for histogram, optimal code and in-order stream. */
int orc_container_encode(const uint8_t *x, uint64_t rows, uint64_t cols, uint32_t N, uint32_t G,
                         uint32_t max_code_len, uint32_t tile_rows, uint8_t *blob, uint64_t cap, uint64_t *size_out)
{
    uint64_t n = rows * cols;
    if (n == 0 || N == 0 || (N % 16) != 0 || N > 256) return ORC_E_ARG;
    orc_layout lay = {N, G, tile_rows, n, cols};
    if (!layout_ok(&lay, rows)) return ORC_E_ARG;
    uint64_t freq[ORC_NSYM];
    uint8_t len[ORC_NSYM];
    uint16_t code[ORC_NSYM];
    orc_histogram(x, n, freq);
    /* max_code_len >= 15 never binds with 16 symbols: plain Huffman (Section 3.1) */
    int rc = max_code_len >= 15 ? orc_huffman_lengths(freq, len)
                                : orc_huffman_lengths_limited(freq, (int)max_code_len, len);
    if (rc < 0) return rc;
    rc = orc_canonical_codes(len, code);
    if (rc) return rc;
    uint64_t bits = orc_stream_bits(freq, len);
    uint64_t total = orc_container_size(n, bits, N);
    if (total > cap) return ORC_E_CAPACITY;
    memset(blob, 0, total);

    uint64_t chunk = 64ull * N;
    uint64_t n_chunks = (n + chunk - 1) / chunk;
    uint64_t off_cb = 256;
    uint64_t off_lb = up(off_cb + 8 * (n_chunks + 1), 256);
    uint64_t off_st = up(off_lb + 2 * n_chunks * 64, 256);
    uint64_t st_bytes = up((bits + 7) / 8 + 8, 16);
    uint64_t off_pl = up(off_st + st_bytes, 256);
    uint64_t pl_bytes = n_chunks * 32ull * N;

    wr32(blob + 0, 0x38464345u);
    wr32(blob + 4, 1);
    wr64(blob + 8, total);
    wr64(blob + 16, n);
    wr64(blob + 24, rows);
    wr64(blob + 32, cols);
    wr32(blob + 40, N);
    wr16(blob + 44, 0); /* this writer embeds no decoder table */
    blob[46] = (uint8_t)G;
    blob[47] = (uint8_t)tile_rows;
    wr64(blob + 48, n_chunks);
    wr64(blob + 56, bits);
    for (int i = 0; i < ORC_NSYM; i++) blob[64 + i] = len[i];
    wr64(blob + 80, off_cb);
    wr64(blob + 88, off_lb);
    wr64(blob + 96, off_st);
    wr64(blob + 104, off_pl);
    wr64(blob + 112, st_bytes);
    wr64(blob + 120, pl_bytes);
    for (int i = 0; i < ORC_NSYM; i++) wr64(blob + 128 + 8 * i, freq[i]);

    /* lane by lane: first half of the lane's symbols forward from its first bit,
     * second half backward from its last bit */
    uint8_t *stream = blob + off_st;
    uint64_t pos = 0;
    for (uint64_t c = 0; c < n_chunks; c++) {
        wr64(blob + off_cb + 8 * c, pos);
        for (uint64_t l = 0; l < 64; l++) {
            uint64_t lb = 0;
            for (uint64_t k = 0; k < N; k++) {
                uint64_t e = lane_element(&lay, c, l, k);
                if (e >= n) continue;
                uint8_t sg, ex, mn;
                orc_split(x[e], &sg, &ex, &mn);
                lb += len[ex];
            }
            uint64_t fwd = pos, bwd = pos + lb; /* bwd: one past the next bit to write */
            for (uint64_t k = 0; k < N; k++) {
                uint64_t e = lane_element(&lay, c, l, k);
                if (e >= n) continue;
                uint8_t sg, ex, mn;
                orc_split(x[e], &sg, &ex, &mn);
                for (int bit = len[ex] - 1; bit >= 0; bit--) { /* first bit of the codeword = its MSB */
                    uint64_t at = (k < N / 2) ? fwd++ : --bwd;
                    if ((code[ex] >> bit) & 1) stream[at >> 3] |= (uint8_t)(1u << (at & 7));
                }
            }
            if (fwd != bwd) return ORC_E_FORMAT;
            wr16(blob + off_lb + 2 * (c * 64 + l), (uint32_t)lb);
            pos += lb;
        }
    }
    wr64(blob + off_cb + 8 * n_chunks, pos);
    if (pos != bits) return ORC_E_FORMAT;

    /* regrouped nibble plane */
    for (uint64_t i = 0; i < n; i++) {
        uint8_t s, e, m;
        orc_split(x[i], &s, &e, &m);
        uint8_t q = (uint8_t)((s << 3) | m);
        uint8_t *b = blob + off_pl + plane_byte_index(i);
        if (plane_is_high(i)) *b |= (uint8_t)(q << 4);
        else *b |= q;
    }
    *size_out = total;
    return ORC_OK;
}

/* Reader: decodes a container to out[n_elem], lane by lane through the metadata.
 * Every lane starts at chunk_bit[c] + the lane_bits of the chunk's earlier lanes;
 * its forward run is walked bit by bit from its first bit upwards, its backward
 * run from its last bit downwards, and the two must meet exactly; chunk starts
 * must equal the running sums; the decoded exponents must reproduce the header's
 * histogram, whose weighted lengths must give stream_bits; an embedded table is
 * rebuilt entry by entry with bit-serial walks.  ORC_E_META / ORC_E_FORMAT
 * otherwise.  stream_bits_out is returned for the size checks. */
int orc_container_decode(const uint8_t *blob, uint64_t size, uint8_t *out, uint64_t out_cap,
                         uint64_t *n_out, uint64_t *stream_bits_out)
{
    if (size < 256) return ORC_E_FORMAT;
    if (rd32(blob) != 0x38464345u || rd32(blob + 4) != 1) return ORC_E_FORMAT;
    uint64_t total = rd64(blob + 8), n = rd64(blob + 16);
    uint64_t rows = rd64(blob + 24), cols = rd64(blob + 32);
    uint32_t N = rd32(blob + 40), TBITS = rd16(blob + 44), G = blob[46], TR = blob[47];
    uint64_t n_chunks = rd64(blob + 48), bits = rd64(blob + 56);
    uint8_t len[ORC_NSYM];
    for (int i = 0; i < ORC_NSYM; i++) len[i] = blob[64 + i];
    uint64_t off_cb = rd64(blob + 80), off_lb = rd64(blob + 88);
    uint64_t off_st = rd64(blob + 96), off_pl = rd64(blob + 104);
    uint64_t st_bytes = rd64(blob + 112), pl_bytes = rd64(blob + 120);
    if (total != size || n == 0 || rows * cols != n) return ORC_E_FORMAT;
    if ((TBITS != 0 && TBITS != 14) || N == 0 || (N % 16) != 0 || N > 256) return ORC_E_FORMAT;
    orc_layout lay = {N, G, TR, n, cols};
    if (!layout_ok(&lay, rows)) return ORC_E_FORMAT;
    uint64_t tbytes = TBITS ? (2ull << TBITS) : 0;
    uint64_t chunk = 64ull * N;
    if (n_chunks != (n + chunk - 1) / chunk) return ORC_E_FORMAT;
    if ((off_cb | off_lb | off_st | off_pl) % 256) return ORC_E_FORMAT;
    if (off_cb != 256 + tbytes || off_cb + 8 * (n_chunks + 1) > off_lb) return ORC_E_FORMAT;
    if (off_lb + 2 * n_chunks * 64 > off_st) return ORC_E_FORMAT;
    if (st_bytes != up((bits + 7) / 8 + 8, 16) || off_st + st_bytes > off_pl) return ORC_E_FORMAT;
    if (pl_bytes != n_chunks * 32ull * N || off_pl + pl_bytes > total) return ORC_E_FORMAT;
    if (out_cap < n) return ORC_E_CAPACITY;

    const uint8_t *stream = blob + off_st;
    /* padding after the last stream bit must be zero */
    for (uint64_t b = bits; b < st_bytes * 8; b++)
        if ((stream[b >> 3] >> (b & 7)) & 1) return ORC_E_FORMAT;

    /* histogram in the header must reproduce stream_bits with these lengths */
    uint64_t fsum = 0, wsum = 0;
    for (int i = 0; i < ORC_NSYM; i++) {
        uint64_t f = rd64(blob + 128 + 8 * i);
        fsum += f;
        wsum += f * len[i];
        if (f > 0 && len[i] == 0) return ORC_E_FORMAT;
    }
    if (fsum != n || wsum != bits) return ORC_E_FORMAT;

    /* an embedded decoder table must say what the code says: walk the bits of every
     * index through the code, one codeword, then the next */
    if (TBITS) {
        for (uint32_t idx = 0; idx < (1u << TBITS); idx++) {
            uint8_t ib[4] = {(uint8_t)idx, (uint8_t)(idx >> 8), 0, 0};
            uint8_t two[2];
            int64_t nx = 0;
            uint32_t s1 = 0, l1 = 0, s2 = 0, l2 = 0;
            if (orc_decode_symbols_dir(ib, 0, +1, 0, TBITS, ORC_LSB_FIRST, len, 1, two, &nx) == ORC_OK) {
                s1 = two[0]; l1 = (uint32_t)nx;
                if (orc_decode_symbols_dir(ib, nx, +1, 0, TBITS, ORC_LSB_FIRST, len, 1, two + 1, &nx) == ORC_OK) {
                    s2 = two[1]; l2 = (uint32_t)nx - l1;
                }
            }
            uint32_t want = 0;
            if (l1) {
                want = (s1 << 3) | (l1 & 7) | ((l1 >> 3) << 15);
                if (l2) want |= (s2 << 11) | ((l1 + l2) << 7);
            }
            if (rd16(blob + 256 + 2 * idx) != want) return ORC_E_FORMAT;
        }
    }

    /* lane by lane through the metadata: forward run, backward run, and the two
     * must meet exactly; chunk starts must agree with the running sum */
    uint8_t *sym = (uint8_t *)malloc(n);       /* decoded exponent of every element */
    uint8_t *lane_sym = (uint8_t *)malloc(N);
    if (!sym || !lane_sym) { free(sym); free(lane_sym); return ORC_E_CAPACITY; }
    int rc = ORC_OK;
    if (rd64(blob + off_cb) != 0 || rd64(blob + off_cb + 8 * n_chunks) != bits) rc = ORC_E_META;
    uint64_t done = 0;
    for (uint64_t c = 0; c < n_chunks && rc == ORC_OK; c++) {
        uint64_t pos = rd64(blob + off_cb + 8 * c);
        for (uint64_t l = 0; l < 64 && rc == ORC_OK; l++) {
            uint64_t cntA = 0, cntB = 0;
            for (uint64_t k = 0; k < N; k++)
                if (lane_element(&lay, c, l, k) < n) { if (k < N / 2) cntA++; else cntB++; }
            uint64_t lb = rd16(blob + off_lb + 2 * (c * 64 + l));
            if (cntA + cntB == 0) { if (lb != 0) rc = ORC_E_META; continue; }
            if (pos + lb > bits) { rc = ORC_E_META; break; }
            int64_t endA = (int64_t)pos, endB = (int64_t)(pos + lb) - 1;
            int r2 = orc_decode_symbols_dir(stream, (int64_t)pos, +1, (int64_t)pos, (int64_t)(pos + lb),
                                            ORC_LSB_FIRST, len, cntA, lane_sym, &endA);
            if (r2 == ORC_OK)
                r2 = orc_decode_symbols_dir(stream, (int64_t)(pos + lb) - 1, -1, (int64_t)pos, (int64_t)(pos + lb),
                                            ORC_LSB_FIRST, len, cntB, lane_sym + cntA, &endB);
            if (r2 || endA != endB + 1) { rc = ORC_E_META; break; }
            uint64_t j = 0;
            for (uint64_t k = 0; k < N; k++) {
                uint64_t e = lane_element(&lay, c, l, k);
                if (e < n) { sym[e] = lane_sym[j++]; done++; }
            }
            pos += lb;
        }
        if (rc == ORC_OK && pos != rd64(blob + off_cb + 8 * (c + 1))) rc = ORC_E_META;
    }
    if (rc == ORC_OK && done != n) rc = ORC_E_META;
    /* the decoded exponents must reproduce the header's histogram */
    if (rc == ORC_OK) {
        uint64_t cnt[ORC_NSYM] = {0};
        for (uint64_t i = 0; i < n; i++) cnt[sym[i]]++;
        for (int i = 0; i < ORC_NSYM; i++)
            if (cnt[i] != rd64(blob + 128 + 8 * i)) rc = ORC_E_META;
    }

    if (rc == ORC_OK) {
        const uint8_t *plane = blob + off_pl;
        for (uint64_t i = 0; i < n; i++) {
            uint8_t b = plane[plane_byte_index(i)];
            uint8_t q = plane_is_high(i) ? (uint8_t)(b >> 4) : (uint8_t)(b & 15);
            out[i] = orc_join((uint8_t)(q >> 3), sym[i], (uint8_t)(q & 7));
        }
        /* padding nibbles beyond n must be zero */
        for (uint64_t i = n; i < n_chunks * chunk; i++) {
            uint8_t b = plane[plane_byte_index(i)];
            uint8_t q = plane_is_high(i) ? (uint8_t)(b >> 4) : (uint8_t)(b & 15);
            if (q) { rc = ORC_E_FORMAT; break; }
        }
    }
    free(sym);
    free(lane_sym);
    if (rc == ORC_OK) { *n_out = n; *stream_bits_out = bits; }
    return rc;
}
