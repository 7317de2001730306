/*
 * ECF8 CPU oracle, wide alphabets -- TEST INFRASTRUCTURE ONLY.
 *
 * The paper's method (Section 3.1: histogram of the exponent field, prefix code
 * under a length cap, one stream of codewords plus the raw remaining bits;
 * Section 3.2: table-free here, bit-serial decoding) applied to formats whose
 * exponent field is wider than E4M3's four bits, which the paper leaves as an
 * open direction (Section 1, the question of going beyond one format; Section
 * 3.1 caps codewords at 16 bits, a cap that only binds for such alphabets):
 *   fmt 1  E5M2  1 byte / element : sign(1) exponent(5) mantissa(2)
 *   fmt 2  BF16  2 bytes / element, little-endian : sign(1) exponent(8) mantissa(7)
 * Slow and plain on purpose; shares no code or header with the product.
 *
 * Code lengths: the cheapest prefix code with no codeword longer than L is
 * written out from its definition.  By the Kraft-McMillan inequality a prefix
 * code with lengths l_i exists iff sum 2^-l_i <= 1, so the optimum is the
 * assignment l_i in 1..L minimising sum f_i l_i under sum 2^(L-l_i) <= 2^L: a
 * knapsack over the 2^L units of code space, solved exhaustively by dynamic
 * programming (orw_lengths_limited).
 *
 * Container "ECFW" (all integers little-endian, every section at a multiple of
 * 256 bytes, in this order):
 *   header, 256 bytes:
 *     0   u32 magic 0x57464345 ("ECFW")     4   u32 version (1)
 *     8   u64 total_size                    16  u64 n_elem
 *     24  u64 rows                          32  u64 cols
 *     40  u32 fmt (1 or 2)                  44  u32 lane_syms N (64 or 128)
 *     48  u32 group_chunks G (power of two, 1..64)
 *     52  u32 max_code_len (longest codeword in use)
 *     56  u32 n_alphabet A (32 or 256)      60  u32 n_symbols (distinct present)
 *     64  u64 n_chunks = ceil(n_elem/(64N)) 72  u64 stream_bits
 *     80  u64 off_code_len   88  u64 off_freq      96  u64 off_chunk_bit
 *     104 u64 off_lane_bits  112 u64 off_stream    120 u64 off_plane
 *     128 u64 off_sign (0 for BF16)
 *     136 u64 stream_bytes   144 u64 plane_bytes   152 u64 sign_bytes
 *     160..255 zero
 *   code_len  : u8[A]   length of the codeword of exponent field x, 0 = absent
 *   freq      : u64[A]  histogram of the exponent field
 *   chunk_bit : u64[n_chunks+1]  start bit of chunk c's first codeword; last = stream_bits
 *   lane_bits : u16[n_chunks*64] code bits of lane l of chunk c
 *   stream    : stream bit i = bit (i&7) of byte (i>>3); lanes follow each other
 *               chunk by chunk, lane by lane.  A piece is P = 16 / (bytes per
 *               element) consecutive elements (16 bytes of output); the k-th
 *               symbol (k = 0..N-1) of lane l of chunk c is element
 *                   base(c) + (k/P)*stride(c) + l*P + k%P
 *               with E = 64N and F = n_elem/(G*E) whole groups:
 *                 c <  G*F: base = (c - c%G)*E + (c%G)*64P, stride = G*64P
 *                 c >= G*F: base = c*E,                     stride = 64P
 *               elements >= n_elem do not exist and are skipped.  Symbols
 *               k < N/2 are coded FORWARD from the lane's first bit upwards (a
 *               codeword's first = most significant bit lowest), symbols
 *               k >= N/2 BACKWARD from the lane's last bit downwards (first bit
 *               highest), k = N/2 at the top; the runs meet exactly.  Codes are
 *               canonical from code_len, ordered by (length, symbol).
 *               stream_bytes = roundup16(ceil(stream_bits/8) + 8), zero padded
 *   plane     : BF16: one byte sign<<7 | mantissa per element; element i sits
 *               in byte (i/4)*4 + {0,2,1,3}[i%4]; plane_bytes = n_chunks*64N.
 *               E5M2: one u32 per piece g = i/16 holding the mantissas: element
 *               i = 16g + 4d + j (d, j in 0..3) in bits 8j+2d, 8j+2d+1;
 *               plane_bytes = n_chunks*16N
 *   sign      : E5M2 only: one u16 per piece, bit i%16 = sign of element i;
 *               sign_bytes = n_chunks*8N.  Both zero padded.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORW_OK 0
#define ORW_E_ARG (-1)
#define ORW_E_FORMAT (-2)
#define ORW_E_CAPACITY (-3)
#define ORW_E_CODE (-4)
#define ORW_E_META (-5)

#define ORW_FMT_E5M2 1
#define ORW_FMT_BF16 2
#define ORW_MAX_ALPHABET 256
#define ORW_MAX_LEN 16

/* ---- the formats ---- */

int orw_alphabet(int fmt) { return fmt == ORW_FMT_E5M2 ? 32 : fmt == ORW_FMT_BF16 ? 256 : 0; }
int orw_elem_bytes(int fmt) { return fmt == ORW_FMT_E5M2 ? 1 : fmt == ORW_FMT_BF16 ? 2 : 0; }

/* element i of x -> exponent field (the coded symbol) and the remaining bits, sign on top */
static void split(int fmt, const uint8_t *x, uint64_t i, uint32_t *sym, uint32_t *rem)
{
    if (fmt == ORW_FMT_E5M2) {
        uint32_t b = x[i];
        *sym = (b >> 2) & 31u;
        *rem = ((b >> 7) << 2) | (b & 3u);
    } else {
        uint32_t v = (uint32_t)x[2 * i] | ((uint32_t)x[2 * i + 1] << 8);
        *sym = (v >> 7) & 255u;
        *rem = ((v >> 15) << 7) | (v & 127u);
    }
}

static void join(int fmt, uint8_t *x, uint64_t i, uint32_t sym, uint32_t rem)
{
    if (fmt == ORW_FMT_E5M2) {
        x[i] = (uint8_t)(((rem >> 2) << 7) | (sym << 2) | (rem & 3u));
    } else {
        uint32_t v = ((rem >> 7) << 15) | (sym << 7) | (rem & 127u);
        x[2 * i] = (uint8_t)(v & 255u);
        x[2 * i + 1] = (uint8_t)(v >> 8);
    }
}

void orw_split(int fmt, const uint8_t *x, uint64_t n, uint8_t *sym, uint8_t *rem)
{
    for (uint64_t i = 0; i < n; i++) {
        uint32_t s, r;
        split(fmt, x, i, &s, &r);
        sym[i] = (uint8_t)s;
        rem[i] = (uint8_t)r;
    }
}

/* Section 3.1, histogram of the exponent field */
int orw_histogram(int fmt, const uint8_t *x, uint64_t n, uint64_t *freq)
{
    int A = orw_alphabet(fmt);
    if (!A) return ORW_E_ARG;
    for (int s = 0; s < A; s++) freq[s] = 0;
    for (uint64_t i = 0; i < n; i++) {
        uint32_t s, r;
        split(fmt, x, i, &s, &r);
        freq[s]++;
    }
    return ORW_OK;
}

/* ---- code lengths ---- */

/* Plain Huffman: merge the two lightest trees until one is left (Section 3.1,
 * code generation).  len[s] = depth of leaf s; one symbol alone gets length 1. */
int orw_huffman_lengths(const uint64_t *freq, int A, uint8_t *len)
{
    /* forest as parent links over at most 2A-1 nodes */
    uint64_t w[2 * ORW_MAX_ALPHABET];
    int parent[2 * ORW_MAX_ALPHABET], alive[2 * ORW_MAX_ALPHABET], leaf_of[ORW_MAX_ALPHABET];
    int n = 0, m = 0;
    if (A < 1 || A > ORW_MAX_ALPHABET) return ORW_E_ARG;
    for (int s = 0; s < A; s++) {
        len[s] = 0;
        leaf_of[s] = -1;
        if (freq[s]) {
            w[n] = freq[s];
            parent[n] = -1;
            alive[n] = 1;
            leaf_of[s] = n++;
        }
    }
    m = n;
    if (m == 0) return ORW_E_ARG;
    if (m == 1) {
        for (int s = 0; s < A; s++)
            if (freq[s]) len[s] = 1;
        return ORW_OK;
    }
    for (int round = 0; round < m - 1; round++) {
        int a = -1, b = -1;
        for (int i = 0; i < n; i++) {
            if (!alive[i]) continue;
            if (a < 0 || w[i] < w[a]) { b = a; a = i; }
            else if (b < 0 || w[i] < w[b]) b = i;
        }
        w[n] = w[a] + w[b];
        parent[n] = -1;
        alive[n] = 1;
        alive[a] = alive[b] = 0;
        parent[a] = parent[b] = n;
        n++;
    }
    for (int s = 0; s < A; s++) {
        if (leaf_of[s] < 0) continue;
        int d = 0;
        for (int i = leaf_of[s]; parent[i] >= 0; i = parent[i]) d++;
        if (d > 255) return ORW_E_CODE;
        len[s] = (uint8_t)d;
    }
    return ORW_OK;
}

/* Cheapest prefix code with every length <= L (1 <= L <= 16): the knapsack of
 * the header comment.  best[b] after i symbols = least sum f l over the first i
 * present symbols that uses at most b of the 2^L units of code space.
 * *cost_out = the optimum; len[] = one optimal assignment. */
int orw_lengths_limited(const uint64_t *freq, int A, int L, uint8_t *len, uint64_t *cost_out)
{
    const uint64_t INF = ~(uint64_t)0;
    int sym[ORW_MAX_ALPHABET], m = 0;
    if (A < 1 || A > ORW_MAX_ALPHABET || L < 1 || L > ORW_MAX_LEN) return ORW_E_ARG;
    for (int s = 0; s < A; s++) {
        len[s] = 0;
        if (freq[s]) sym[m++] = s;
    }
    if (m == 0) return ORW_E_ARG;
    if ((uint64_t)m > ((uint64_t)1 << L)) return ORW_E_CODE;      /* no prefix code that short */
    const uint32_t B = (uint32_t)1 << L;
    uint64_t *prev = (uint64_t *)malloc((B + 1) * sizeof(uint64_t));
    uint64_t *cur = (uint64_t *)malloc((B + 1) * sizeof(uint64_t));
    uint8_t *choice = (uint8_t *)malloc((size_t)m * (B + 1));
    if (!prev || !cur || !choice) { free(prev); free(cur); free(choice); return ORW_E_CAPACITY; }
    for (uint32_t b = 0; b <= B; b++) prev[b] = 0;                /* no symbols: nothing to pay */
    for (int i = 0; i < m; i++) {
        const uint64_t f = freq[sym[i]];
        for (uint32_t b = 0; b <= B; b++) {
            uint64_t best = INF;
            uint8_t bl = 0;
            for (int l = 1; l <= L; l++) {
                const uint32_t units = (uint32_t)1 << (L - l);
                if (units > b || prev[b - units] == INF) continue;
                const uint64_t c = prev[b - units] + f * (uint64_t)l;
                if (c < best) { best = c; bl = (uint8_t)l; }
            }
            cur[b] = best;
            choice[(size_t)i * (B + 1) + b] = bl;
        }
        uint64_t *t = prev; prev = cur; cur = t;
    }
    int rc = ORW_OK;
    if (prev[B] == INF) rc = ORW_E_CODE;
    else {
        uint32_t b = B;
        if (cost_out) *cost_out = prev[B];
        for (int i = m - 1; i >= 0; i--) {
            const uint8_t l = choice[(size_t)i * (B + 1) + b];
            len[sym[i]] = l;
            b -= (uint32_t)1 << (L - l);
        }
    }
    free(prev); free(cur); free(choice);
    return rc;
}

/* Canonical codewords ordered by (length, symbol), as numbers with the first bit
 * most significant.  ORW_E_CODE if the lengths overfill the code space. */
int orw_canonical(const uint8_t *len, int A, uint32_t *code)
{
    uint64_t kraft = 0;
    uint32_t next = 0;
    int any = 0;
    for (int s = 0; s < A; s++) {
        code[s] = 0;
        if (len[s] > ORW_MAX_LEN) return ORW_E_CODE;
        if (len[s]) { kraft += (uint64_t)1 << (ORW_MAX_LEN - len[s]); any = 1; }
    }
    if (!any || kraft > ((uint64_t)1 << ORW_MAX_LEN)) return ORW_E_CODE;
    for (int l = 1; l <= ORW_MAX_LEN; l++) {
        for (int s = 0; s < A; s++)
            if (len[s] == l) code[s] = next++;
        next <<= 1;
    }
    return ORW_OK;
}

uint64_t orw_stream_bits(const uint64_t *freq, const uint8_t *len, int A)
{
    uint64_t b = 0;
    for (int s = 0; s < A; s++) b += freq[s] * len[s];
    return b;
}

/* ---- the container ---- */

static uint64_t up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }
static uint64_t rd64(const uint8_t *p) { uint64_t v = 0; for (int i = 7; i >= 0; i--) v = (v << 8) | p[i]; return v; }
static uint32_t rd32(const uint8_t *p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24); }
static void wr64(uint8_t *p, uint64_t v) { for (int i = 0; i < 8; i++) p[i] = (uint8_t)(v >> (8 * i)); }
static void wr32(uint8_t *p, uint32_t v) { for (int i = 0; i < 4; i++) p[i] = (uint8_t)(v >> (8 * i)); }

typedef struct {
    int fmt;
    uint32_t N, G, P;
    uint64_t n;
} orw_layout;

static int layout_ok(const orw_layout *y)
{
    if (!orw_alphabet(y->fmt) || y->n == 0) return 0;
    if (y->N != 64 && y->N != 128) return 0;
    if (y->G < 1 || y->G > 64 || (y->G & (y->G - 1))) return 0;
    return 1;
}

/* element index of the k-th symbol of lane l of chunk c (may be >= n: absent) */
static uint64_t lane_element(const orw_layout *y, uint64_t c, uint32_t l, uint32_t k)
{
    const uint64_t E = 64ull * y->N, P = y->P;
    const uint64_t F = y->n / (y->G * E);
    uint64_t base, stride;
    if (c < y->G * F) {
        base = (c - c % y->G) * E + (c % y->G) * 64 * P;
        stride = y->G * 64 * P;
    } else {
        base = c * E;
        stride = 64 * P;
    }
    return base + (k / P) * stride + (uint64_t)l * P + k % P;
}

typedef struct {
    uint64_t n_chunks, off_len, off_freq, off_cb, off_lb, off_st, off_pl, off_sg, st_bytes, pl_bytes, sg_bytes, total;
} orw_sections;

static void sections(const orw_layout *y, uint64_t bits, orw_sections *s)
{
    const uint64_t A = (uint64_t)orw_alphabet(y->fmt);
    s->n_chunks = (y->n + 64ull * y->N - 1) / (64ull * y->N);
    s->off_len = 256;
    s->off_freq = s->off_len + up(A, 256);
    s->off_cb = s->off_freq + up(8 * A, 256);
    s->off_lb = s->off_cb + up(8 * (s->n_chunks + 1), 256);
    s->off_st = s->off_lb + up(2 * 64 * s->n_chunks, 256);
    s->st_bytes = up((bits + 7) / 8 + 8, 16);
    s->off_pl = s->off_st + up(s->st_bytes, 256);
    if (y->fmt == ORW_FMT_BF16) {
        s->pl_bytes = s->n_chunks * 64 * y->N;
        s->sg_bytes = 0;
        s->off_sg = 0;
        s->total = s->off_pl + up(s->pl_bytes, 256);
    } else {
        s->pl_bytes = s->n_chunks * 16 * y->N;
        s->sg_bytes = s->n_chunks * 8 * y->N;
        s->off_sg = s->off_pl + up(s->pl_bytes, 256);
        s->total = s->off_sg + up(s->sg_bytes, 256);
    }
}

uint64_t orw_container_size(int fmt, uint64_t n, uint64_t bits, uint32_t N)
{
    orw_layout y = {fmt, N, 1, (uint32_t)(16 / (orw_elem_bytes(fmt) ? orw_elem_bytes(fmt) : 1)), n};
    orw_sections s;
    if (!layout_ok(&y)) return 0;
    sections(&y, bits, &s);
    return s.total;
}

static void put_bit(uint8_t *st, uint64_t i, uint32_t v) { if (v) st[i >> 3] |= (uint8_t)(1u << (i & 7)); }
static uint32_t get_bit(const uint8_t *st, uint64_t i) { return (st[i >> 3] >> (i & 7)) & 1u; }

static void put_rem(const orw_layout *y, uint8_t *plane, uint8_t *sign, uint64_t i, uint32_t rem)
{
    static const int swap[4] = {0, 2, 1, 3};
    if (y->fmt == ORW_FMT_BF16) {
        plane[(i / 4) * 4 + swap[i % 4]] = (uint8_t)rem;
    } else {
        const uint64_t g = i / 16;
        const uint32_t d = (uint32_t)(i % 16) / 4, j = (uint32_t)(i % 4);
        uint32_t w = rd32(plane + 4 * g) | ((rem & 3u) << (8 * j + 2 * d));
        wr32(plane + 4 * g, w);
        if (rem >> 2) sign[2 * g + (i % 16) / 8] |= (uint8_t)(1u << (i % 8));
    }
}

static uint32_t get_rem(const orw_layout *y, const uint8_t *plane, const uint8_t *sign, uint64_t i)
{
    static const int swap[4] = {0, 2, 1, 3};
    if (y->fmt == ORW_FMT_BF16) return plane[(i / 4) * 4 + swap[i % 4]];
    const uint64_t g = i / 16;
    const uint32_t d = (uint32_t)(i % 16) / 4, j = (uint32_t)(i % 4);
    const uint32_t m = (rd32(plane + 4 * g) >> (8 * j + 2 * d)) & 3u;
    const uint32_t s = (sign[2 * g + (i % 16) / 8] >> (i % 8)) & 1u;
    return (s << 2) | m;
}

/*
 * Writes the container for x (rows*cols elements of fmt) with the code given by
 * len[] (a prefix code covering every exponent field that occurs).
 */
int orw_container_encode(int fmt, const uint8_t *x, uint64_t rows, uint64_t cols, uint32_t N, uint32_t G,
                         const uint8_t *len, uint8_t *blob, uint64_t cap, uint64_t *size_out)
{
    const int A = orw_alphabet(fmt);
    if (!A || !x || !len || !blob || rows == 0 || cols == 0) return ORW_E_ARG;
    orw_layout y = {fmt, N, G, (uint32_t)(16 / orw_elem_bytes(fmt)), rows * cols};
    if (!layout_ok(&y)) return ORW_E_ARG;
    uint64_t freq[ORW_MAX_ALPHABET];
    uint32_t code[ORW_MAX_ALPHABET];
    orw_histogram(fmt, x, y.n, freq);
    if (orw_canonical(len, A, code)) return ORW_E_CODE;
    uint32_t maxlen = 0, nsym = 0;
    for (int s = 0; s < A; s++) {
        if (freq[s] && !len[s]) return ORW_E_CODE;
        if (freq[s]) nsym++;
        if (len[s] > maxlen) maxlen = len[s];
    }
    const uint64_t bits = orw_stream_bits(freq, len, A);
    orw_sections sc;
    sections(&y, bits, &sc);
    if (sc.total > cap) return ORW_E_CAPACITY;
    memset(blob, 0, sc.total);
    wr32(blob + 0, 0x57464345u);
    wr32(blob + 4, 1);
    wr64(blob + 8, sc.total);
    wr64(blob + 16, y.n);
    wr64(blob + 24, rows);
    wr64(blob + 32, cols);
    wr32(blob + 40, (uint32_t)fmt);
    wr32(blob + 44, N);
    wr32(blob + 48, G);
    wr32(blob + 52, maxlen);
    wr32(blob + 56, (uint32_t)A);
    wr32(blob + 60, nsym);
    wr64(blob + 64, sc.n_chunks);
    wr64(blob + 72, bits);
    wr64(blob + 80, sc.off_len);
    wr64(blob + 88, sc.off_freq);
    wr64(blob + 96, sc.off_cb);
    wr64(blob + 104, sc.off_lb);
    wr64(blob + 112, sc.off_st);
    wr64(blob + 120, sc.off_pl);
    wr64(blob + 128, sc.off_sg);
    wr64(blob + 136, sc.st_bytes);
    wr64(blob + 144, sc.pl_bytes);
    wr64(blob + 152, sc.sg_bytes);
    for (int s = 0; s < A; s++) {
        blob[sc.off_len + s] = len[s];
        wr64(blob + sc.off_freq + 8 * s, freq[s]);
    }
    uint8_t *st = blob + sc.off_st, *plane = blob + sc.off_pl, *sign = blob + sc.off_sg;
    uint64_t pos = 0;
    for (uint64_t c = 0; c < sc.n_chunks; c++) {
        wr64(blob + sc.off_cb + 8 * c, pos);
        for (uint32_t l = 0; l < 64; l++) {
            uint32_t lane_bits = 0;
            for (uint32_t k = 0; k < N; k++) {
                const uint64_t i = lane_element(&y, c, l, k);
                if (i >= y.n) continue;
                uint32_t s, r;
                split(fmt, x, i, &s, &r);
                lane_bits += len[s];
            }
            uint64_t up_pos = pos, down_pos = pos + lane_bits;    /* next forward bit, one past the next backward bit */
            for (uint32_t k = 0; k < N; k++) {
                const uint64_t i = lane_element(&y, c, l, k);
                if (i >= y.n) continue;
                uint32_t s, r;
                split(fmt, x, i, &s, &r);
                put_rem(&y, plane, sign, i, r);
                for (int b = len[s] - 1; b >= 0; b--) {           /* first bit of the codeword first */
                    const uint32_t v = (code[s] >> b) & 1u;
                    if (k < N / 2) put_bit(st, up_pos++, v);
                    else put_bit(st, --down_pos, v);
                }
            }
            if (up_pos != down_pos) return ORW_E_META;
            blob[sc.off_lb + 2 * (64 * c + l)] = (uint8_t)(lane_bits & 255u);
            blob[sc.off_lb + 2 * (64 * c + l) + 1] = (uint8_t)(lane_bits >> 8);
            pos += lane_bits;
        }
    }
    wr64(blob + sc.off_cb + 8 * sc.n_chunks, pos);
    if (pos != bits) return ORW_E_META;
    if (size_out) *size_out = sc.total;
    return ORW_OK;
}

/* one codeword read bit by bit from position *p in direction dir (+1 / -1) */
static int read_symbol(const uint8_t *st, uint64_t *p, int dir, uint64_t lo, uint64_t hi, const uint8_t *len,
                       const uint32_t *code, int A, uint32_t *sym)
{
    uint32_t v = 0;
    for (int l = 1; l <= ORW_MAX_LEN; l++) {
        if (dir > 0) { if (*p >= hi) return ORW_E_META; v = (v << 1) | get_bit(st, (*p)++); }
        else { if (*p <= lo) return ORW_E_META; v = (v << 1) | get_bit(st, --(*p)); }
        for (int s = 0; s < A; s++)
            if (len[s] == l && code[s] == v) { *sym = (uint32_t)s; return ORW_OK; }
    }
    return ORW_E_CODE;
}

/*
 * Reads a container back into elements, checking every structural fact on the
 * way (sizes, offsets, metadata consistent with the stream).
 */
int orw_container_decode(const uint8_t *blob, uint64_t size, uint8_t *out, uint64_t out_cap_elems, uint64_t *n_out,
                         uint64_t *bits_out)
{
    if (!blob || size < 256) return ORW_E_FORMAT;
    if (rd32(blob) != 0x57464345u || rd32(blob + 4) != 1) return ORW_E_FORMAT;
    const int fmt = (int)rd32(blob + 40);
    const int A = orw_alphabet(fmt);
    if (!A || (int)rd32(blob + 56) != A) return ORW_E_FORMAT;
    orw_layout y = {fmt, rd32(blob + 44), rd32(blob + 48), (uint32_t)(16 / orw_elem_bytes(fmt)), rd64(blob + 16)};
    if (!layout_ok(&y)) return ORW_E_FORMAT;
    if (rd64(blob + 24) * rd64(blob + 32) != y.n) return ORW_E_FORMAT;
    const uint64_t bits = rd64(blob + 72);
    orw_sections sc;
    sections(&y, bits, &sc);
    if (rd64(blob + 8) != sc.total || size < sc.total || rd64(blob + 64) != sc.n_chunks) return ORW_E_FORMAT;
    if (rd64(blob + 80) != sc.off_len || rd64(blob + 88) != sc.off_freq || rd64(blob + 96) != sc.off_cb ||
        rd64(blob + 104) != sc.off_lb || rd64(blob + 112) != sc.off_st || rd64(blob + 120) != sc.off_pl ||
        rd64(blob + 128) != sc.off_sg || rd64(blob + 136) != sc.st_bytes || rd64(blob + 144) != sc.pl_bytes ||
        rd64(blob + 152) != sc.sg_bytes)
        return ORW_E_FORMAT;
    if (y.n > out_cap_elems) return ORW_E_CAPACITY;
    const uint8_t *len = blob + sc.off_len;
    uint32_t code[ORW_MAX_ALPHABET];
    uint64_t freq[ORW_MAX_ALPHABET], seen[ORW_MAX_ALPHABET];
    if (orw_canonical(len, A, code)) return ORW_E_CODE;
    uint32_t maxlen = 0, nsym = 0;
    for (int s = 0; s < A; s++) {
        freq[s] = rd64(blob + sc.off_freq + 8 * s);
        seen[s] = 0;
        if (freq[s]) nsym++;
        if (freq[s] && !len[s]) return ORW_E_CODE;
        if (len[s] > maxlen) maxlen = len[s];
    }
    if (rd32(blob + 52) != maxlen || rd32(blob + 60) != nsym) return ORW_E_FORMAT;
    if (orw_stream_bits(freq, len, A) != bits) return ORW_E_META;
    const uint8_t *st = blob + sc.off_st, *plane = blob + sc.off_pl, *sign = blob + sc.off_sg;
    uint64_t pos = 0;
    for (uint64_t c = 0; c < sc.n_chunks; c++) {
        if (rd64(blob + sc.off_cb + 8 * c) != pos) return ORW_E_META;
        for (uint32_t l = 0; l < 64; l++) {
            const uint32_t lane_bits = (uint32_t)blob[sc.off_lb + 2 * (64 * c + l)] |
                                       ((uint32_t)blob[sc.off_lb + 2 * (64 * c + l) + 1] << 8);
            if (pos + lane_bits > bits) return ORW_E_META;
            uint64_t up_pos = pos, down_pos = pos + lane_bits;
            for (uint32_t k = 0; k < y.N; k++) {
                const uint64_t i = lane_element(&y, c, l, k);
                if (i >= y.n) continue;
                uint32_t s = 0;
                int rc = k < y.N / 2 ? read_symbol(st, &up_pos, +1, pos, down_pos, len, code, A, &s)
                                     : read_symbol(st, &down_pos, -1, up_pos, pos + lane_bits, len, code, A, &s);
                if (rc) return rc;
                seen[s]++;
                join(fmt, out, i, s, get_rem(&y, plane, sign, i));
            }
            if (up_pos != down_pos) return ORW_E_META;
            pos += lane_bits;
        }
    }
    if (rd64(blob + sc.off_cb + 8 * sc.n_chunks) != pos || pos != bits) return ORW_E_META;
    for (int s = 0; s < A; s++)
        if (seen[s] != freq[s]) return ORW_E_META;
    if (n_out) *n_out = y.n;
    if (bits_out) *bits_out = bits;
    return ORW_OK;
}
