/*
 * ECF8 CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded, obviously-correct implementation of what the
 * ECF8 path computes: entropy coding of the 4-bit exponent field of FP8 E4M3
 * weights with an optimal prefix code, raw storage of sign+mantissa, and
 * bit-serial decoding back to the exact original bytes.
 *
 * Nothing in the product (the HIP library, its host encoder, the Python
 * binding) may include, link or call this file; only tests, the smoke check
 * and the CPU-baseline leg of the benchmark use it.  It shares no code, table
 * or constant with the product.
 *
 * Every function cites the passage of the paper it follows (Section 3.1 =
 * "Encoding", Section 3.2 = "Decoding", Table 4 = notation table of the
 * appendix, Algorithm 1 = block-level decompression pseudocode).
 *
 * Pins (tests/test_oracle_*.py): identity round trip over all 256 byte values,
 * Kraft equality, entropy sandwich H <= Lbar < H+1, brute-force optimal code
 * on tiny alphabets, the worked example of Figure 2 (29 bits for 13 symbols),
 * dyadic / uniform / two-symbol / single-symbol special cases, and a
 * hand-derived four-byte example.
 *
 * Plain C99, no SIMD, no lookup-table decoding, no threads.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#define ORC_NSYM 16
#define ORC_MSB_FIRST 0 /* Algorithm 1: oldest bit is the most significant */
#define ORC_LSB_FIRST 1 /* bit i of the stream is bit (i&7) of byte (i>>3)  */

#define ORC_OK 0
#define ORC_E_ARG (-1)
#define ORC_E_FORMAT (-2)
#define ORC_E_CAPACITY (-3)
#define ORC_E_CODE (-4)     /* bit pattern that is no codeword               */
#define ORC_E_META (-5)     /* side metadata disagrees with the stream       */

/* ------------------------------------------------------------------ */
/* O1: field split / join.  Section 3.1: an FP8 weight spends 4 bits   */
/* on the exponent; Algorithm 1 (byte assembly) fixes the positions:   */
/* byte = exponent<<3 | sign<<7 | mantissa.                            */
/* ------------------------------------------------------------------ */
void orc_split(uint8_t v, uint8_t *s, uint8_t *e, uint8_t *m)
{
    *s = (uint8_t)(v >> 7);
    *e = (uint8_t)((v >> 3) & 15);
    *m = (uint8_t)(v & 7);
}

uint8_t orc_join(uint8_t s, uint8_t e, uint8_t m)
{
    return (uint8_t)((e << 3) | (s << 7) | m);
}

/* O2: empirical exponent distribution p(x), x in 0..15 (Section 3.1). */
void orc_histogram(const uint8_t *x, uint64_t n, uint64_t freq[ORC_NSYM])
{
    for (int i = 0; i < ORC_NSYM; i++) freq[i] = 0;
    for (uint64_t i = 0; i < n; i++) {
        uint8_t s, e, m;
        orc_split(x[i], &s, &e, &m);
        freq[e]++;
    }
}

/* Shannon entropy of the histogram in bits (Section 2, H(E)). */
double orc_entropy_bits(const uint64_t freq[ORC_NSYM])
{
    double tot = 0.0, h = 0.0;
    for (int i = 0; i < ORC_NSYM; i++) tot += (double)freq[i];
    if (tot == 0.0) return 0.0;
    for (int i = 0; i < ORC_NSYM; i++) {
        if (freq[i] == 0) continue;
        double p = (double)freq[i] / tot;
        h -= p * log2(p);
    }
    return h;
}

/* ------------------------------------------------------------------ */
/* O3: Huffman code lengths (Section 3.1, "Huffman code generation":   */
/* the optimal tree minimising the expected code length).  Textbook    */
/* construction: repeatedly merge the two live nodes of least weight,  */
/* found by a plain scan.  Symbols of zero frequency get no code       */
/* (length 0).  Reading for the degenerate case of one distinct        */
/* symbol: it gets the 1-bit code "0".  With 16 symbols the depth is   */
/* at most 15, so the paper's 16-bit cap never binds.                  */
/* Returns the maximum length, or a negative error.                    */
/* ------------------------------------------------------------------ */
int orc_huffman_lengths(const uint64_t freq[ORC_NSYM], uint8_t len[ORC_NSYM])
{
    uint64_t w[2 * ORC_NSYM];
    int parent[2 * ORC_NSYM];
    int alive[2 * ORC_NSYM];
    int nn = 0, live = 0;
    int leaf_of[ORC_NSYM];

    for (int i = 0; i < ORC_NSYM; i++) {
        len[i] = 0;
        leaf_of[i] = -1;
        if (freq[i] > 0) {
            w[nn] = freq[i];
            parent[nn] = -1;
            alive[nn] = 1;
            leaf_of[i] = nn;
            nn++;
            live++;
        }
    }
    if (live == 0) return ORC_E_ARG;
    if (live == 1) {
        for (int i = 0; i < ORC_NSYM; i++)
            if (freq[i] > 0) len[i] = 1;
        return 1;
    }
    while (live > 1) {
        int a = -1, b = -1; /* a: least, b: second least */
        for (int i = 0; i < nn; i++) {
            if (!alive[i]) continue;
            if (a < 0 || w[i] < w[a]) { b = a; a = i; }
            else if (b < 0 || w[i] < w[b]) { b = i; }
        }
        w[nn] = w[a] + w[b];
        parent[nn] = -1;
        alive[nn] = 1;
        alive[a] = alive[b] = 0;
        parent[a] = parent[b] = nn;
        nn++;
        live--;
    }
    int maxlen = 0;
    for (int i = 0; i < ORC_NSYM; i++) {
        if (leaf_of[i] < 0) continue;
        int d = 0;
        for (int j = leaf_of[i]; parent[j] >= 0; j = parent[j]) d++;
        len[i] = (uint8_t)d;
        if (d > maxlen) maxlen = d;
    }
    return maxlen;
}

/* ------------------------------------------------------------------ */
/* O3b: code lengths under a cap (Section 3.1 caps the code length and  */
/* adjusts the frequencies to get there; the reading taken here is the  */
/* best any such adjustment can reach): among all prefix codes with     */
/* every length <= lmax, one that minimises sum f(x) * len(x).  Written */
/* out as a search: in a cheapest code a more frequent symbol is never  */
/* longer than a less frequent one (swapping the two would not cost     */
/* more), so it is enough to walk the symbols from most to least        */
/* frequent, try every non-decreasing length sequence whose Kraft sum   */
/* stays <= 1, and keep the cheapest.  One distinct symbol: length 1.   */
/* Returns the maximum length, or a negative error (lmax too small for  */
/* the number of symbols, lmax > 15).                                   */
/* ------------------------------------------------------------------ */
typedef struct {
    int k, lmax;
    uint64_t f[ORC_NSYM];
    int cur[ORC_NSYM], best[ORC_NSYM];
    uint64_t best_cost;
    int found;
} orc_ll_search;

static void orc_ll_walk(orc_ll_search *S, int i, int minlen, uint64_t used, uint64_t cost)
{
    /* used: Kraft sum so far in units of 2^-lmax */
    const uint64_t cap = 1ull << S->lmax;
    if (S->found && cost >= S->best_cost) return;
    if (i == S->k) {
        S->best_cost = cost;
        S->found = 1;
        for (int j = 0; j < S->k; j++) S->best[j] = S->cur[j];
        return;
    }
    for (int l = minlen; l <= S->lmax; l++) {
        uint64_t u = used + (1ull << (S->lmax - l));
        /* every later symbol needs at least one unit */
        if (u + (uint64_t)(S->k - i - 1) > cap) continue;
        S->cur[i] = l;
        orc_ll_walk(S, i + 1, l, u, cost + S->f[i] * (uint64_t)l);
    }
}

int orc_huffman_lengths_limited(const uint64_t freq[ORC_NSYM], int lmax, uint8_t len[ORC_NSYM])
{
    orc_ll_search S;
    int order[ORC_NSYM];
    S.k = 0;
    for (int i = 0; i < ORC_NSYM; i++) {
        len[i] = 0;
        if (freq[i] > 0) order[S.k++] = i;
    }
    if (S.k == 0 || lmax < 1 || lmax > 15) return ORC_E_ARG;
    if (S.k == 1) { len[order[0]] = 1; return 1; }
    if ((1 << lmax) < S.k) return ORC_E_ARG;
    /* most frequent first (insertion sort, ties by symbol value) */
    for (int a = 1; a < S.k; a++) {
        int v = order[a], b = a - 1;
        while (b >= 0 && freq[order[b]] < freq[v]) { order[b + 1] = order[b]; b--; }
        order[b + 1] = v;
    }
    for (int j = 0; j < S.k; j++) S.f[j] = freq[order[j]];
    S.lmax = lmax;
    S.found = 0;
    S.best_cost = 0;
    orc_ll_walk(&S, 0, 1, 0, 0);
    if (!S.found) return ORC_E_ARG;
    int maxlen = 0;
    for (int j = 0; j < S.k; j++) {
        len[order[j]] = (uint8_t)S.best[j];
        if (S.best[j] > maxlen) maxlen = S.best[j];
    }
    return maxlen;
}

/* ------------------------------------------------------------------ */
/* O4: canonical code assignment.  The paper leaves the 0/1 labelling  */
/* of the tree open; the reading taken: order symbols by (length,      */
/* symbol value), first code all zeros, each next code = previous + 1  */
/* shifted left by the growth in length.  Codes are numbers whose most */
/* significant bit is the first bit of the codeword.                   */
/* ------------------------------------------------------------------ */
int orc_canonical_codes(const uint8_t len[ORC_NSYM], uint16_t code[ORC_NSYM])
{
    int prev_len = 0;
    uint32_t next = 0;
    int first = 1;
    for (int i = 0; i < ORC_NSYM; i++) code[i] = 0;
    for (int l = 1; l <= 15; l++) {
        for (int s = 0; s < ORC_NSYM; s++) {
            if (len[s] != l) continue;
            if (first) { next = 0; first = 0; }
            else next = (next + 1) << (l - prev_len);
            if (next >> l) return ORC_E_CODE; /* Kraft sum above one */
            code[s] = (uint16_t)next;
            prev_len = l;
        }
    }
    for (int s = 0; s < ORC_NSYM; s++)
        if (len[s] > 15) return ORC_E_ARG;
    return ORC_OK;
}

/* bit access in either order */
static int get_bit(const uint8_t *s, uint64_t i, int order)
{
    if (order == ORC_MSB_FIRST) return (s[i >> 3] >> (7 - (i & 7))) & 1;
    return (s[i >> 3] >> (i & 7)) & 1;
}

static void put_bit(uint8_t *s, uint64_t i, int bit, int order)
{
    if (!bit) return;
    if (order == ORC_MSB_FIRST) s[i >> 3] |= (uint8_t)(1u << (7 - (i & 7)));
    else s[i >> 3] |= (uint8_t)(1u << (i & 7));
}

/* Sum over symbols of freq*len: the exact stream length in bits. */
uint64_t orc_stream_bits(const uint64_t freq[ORC_NSYM], const uint8_t len[ORC_NSYM])
{
    uint64_t t = 0;
    for (int i = 0; i < ORC_NSYM; i++) t += freq[i] * (uint64_t)len[i];
    return t;
}

/* ------------------------------------------------------------------ */
/* O5: bit-serial encoder (Section 3.1, "Encoding and synchronization  */
/* metadata generation": symbols x_1..x_n are processed in order and   */
/* their codewords concatenated into one continuous bitstream).  The   */
/* stream buffer must be zero-filled by the caller; unused bits of the */
/* last byte stay zero.  Writes the bit position of every codeword     */
/* start that is a multiple of `mark_every` symbols into marks[] when  */
/* marks != NULL (marks[j] = start bit of symbol j*mark_every).        */
/* ------------------------------------------------------------------ */
int orc_encode_exponents(const uint8_t *x, uint64_t n,
                         const uint8_t len[ORC_NSYM], const uint16_t code[ORC_NSYM],
                         int order, uint8_t *stream, uint64_t stream_cap_bytes,
                         uint64_t *nbits_out,
                         uint64_t mark_every, uint64_t *marks)
{
    uint64_t pos = 0;
    for (uint64_t i = 0; i < n; i++) {
        uint8_t s, e, m;
        orc_split(x[i], &s, &e, &m);
        int l = len[e];
        if (l == 0) return ORC_E_CODE;
        if (marks && mark_every && (i % mark_every) == 0) marks[i / mark_every] = pos;
        if (((pos + (uint64_t)l + 7) >> 3) > stream_cap_bytes) return ORC_E_CAPACITY;
        for (int b = l - 1; b >= 0; b--) { /* first bit of the codeword = its MSB */
            put_bit(stream, pos, (code[e] >> b) & 1, order);
            pos++;
        }
    }
    *nbits_out = pos;
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* O6: sign/mantissa plane in the paper's layout (Table 4, "packed":   */
/* ceil(n/2) bytes of nibbles sign<<3 | mantissa; Algorithm 1's merge  */
/* step reads element o from byte o/2, even o in the high nibble).     */
/* ------------------------------------------------------------------ */
void orc_pack_nibbles_paper(const uint8_t *x, uint64_t n, uint8_t *packed)
{
    uint64_t nb = (n + 1) / 2;
    for (uint64_t i = 0; i < nb; i++) packed[i] = 0;
    for (uint64_t i = 0; i < n; i++) {
        uint8_t s, e, m;
        orc_split(x[i], &s, &e, &m);
        uint8_t q = (uint8_t)((s << 3) | m);
        if ((i & 1) == 0) packed[i >> 1] |= (uint8_t)(q << 4);
        else packed[i >> 1] |= q;
    }
}

static uint8_t nibble_paper(const uint8_t *packed, uint64_t i)
{
    uint8_t b = packed[i >> 1];
    return (i & 1) == 0 ? (uint8_t)(b >> 4) : (uint8_t)(b & 15);
}

/* Explicit binary code tree: child[node][bit], leaf symbol or -1. */
typedef struct {
    int child[2 * ORC_NSYM * 16][2];
    int sym[2 * ORC_NSYM * 16];
    int n;
} orc_tree;

static int tree_build(orc_tree *t, const uint8_t len[ORC_NSYM], const uint16_t code[ORC_NSYM])
{
    t->n = 1;
    t->child[0][0] = t->child[0][1] = -1;
    t->sym[0] = -1;
    for (int s = 0; s < ORC_NSYM; s++) {
        if (len[s] == 0) continue;
        int node = 0;
        for (int b = len[s] - 1; b >= 0; b--) {
            int bit = (code[s] >> b) & 1;
            if (t->sym[node] >= 0) return ORC_E_CODE; /* a codeword is a prefix of another */
            if (t->child[node][bit] < 0) {
                int nn = t->n++;
                t->child[nn][0] = t->child[nn][1] = -1;
                t->sym[nn] = -1;
                t->child[node][bit] = nn;
            }
            node = t->child[node][bit];
        }
        if (t->sym[node] >= 0 || t->child[node][0] >= 0 || t->child[node][1] >= 0) return ORC_E_CODE;
        t->sym[node] = s;
    }
    return ORC_OK;
}

/* Walk the tree one bit at a time from *pos; returns the symbol or a negative error. */
static int tree_walk(const orc_tree *t, const uint8_t *stream, uint64_t limit_bits,
                     int order, uint64_t *pos)
{
    int node = 0;
    while (t->sym[node] < 0) {
        if (*pos >= limit_bits) return ORC_E_FORMAT;
        int bit = get_bit(stream, *pos, order);
        (*pos)++;
        node = t->child[node][bit];
        if (node < 0) return ORC_E_CODE;
    }
    return t->sym[node];
}

/* ------------------------------------------------------------------ */
/* O7: bit-serial decoder.  Starts at bit 0, walks the code tree one   */
/* bit at a time, emits n symbols and rebuilds each byte from the      */
/* exponent and its nibble exactly as Algorithm 1's assembly step      */
/* (exponent<<3 | sign bit to bit 7 | mantissa).  Uses no side         */
/* metadata at all.                                                    */
/* ------------------------------------------------------------------ */
int orc_decode_serial(const uint8_t *stream, uint64_t nbits, int order,
                      const uint8_t len[ORC_NSYM], const uint8_t *packed_paper,
                      uint64_t n, uint8_t *out)
{
    uint16_t code[ORC_NSYM];
    orc_tree t;
    int rc = orc_canonical_codes(len, code);
    if (rc) return rc;
    rc = tree_build(&t, len, code);
    if (rc) return rc;
    uint64_t pos = 0;
    for (uint64_t i = 0; i < n; i++) {
        int e = tree_walk(&t, stream, nbits, order, &pos);
        if (e < 0) return e;
        uint8_t q = nibble_paper(packed_paper, i);
        out[i] = orc_join((uint8_t)(q >> 3), (uint8_t)e, (uint8_t)(q & 7));
    }
    if (pos != nbits) return ORC_E_FORMAT;
    return ORC_OK;
}

/* Directional variant for containers whose lanes hold a forward and a backward
 * run of codewords: decodes n symbols starting at bit `start`, stepping +1 or
 * -1 per bit (a codeword's first bit is read first either way); bits outside
 * [lo, hi) are an error.  *next receives the index of the next unread bit. */
int orc_decode_symbols_dir(const uint8_t *stream, int64_t start, int dir, int64_t lo, int64_t hi,
                           int order, const uint8_t len[ORC_NSYM], uint64_t n, uint8_t *sym_out,
                           int64_t *next)
{
    uint16_t code[ORC_NSYM];
    orc_tree t;
    int rc = orc_canonical_codes(len, code);
    if (rc) return rc;
    rc = tree_build(&t, len, code);
    if (rc) return rc;
    int64_t pos = start;
    for (uint64_t i = 0; i < n; i++) {
        int node = 0;
        while (t.sym[node] < 0) {
            if (pos < lo || pos >= hi) return ORC_E_FORMAT;
            int bit = get_bit(stream, (uint64_t)pos, order);
            pos += dir;
            node = t.child[node][bit];
            if (node < 0) return ORC_E_CODE;
        }
        sym_out[i] = (uint8_t)t.sym[node];
    }
    *next = pos;
    return ORC_OK;
}

/* Whole-tensor round trip in the paper's own terms: histogram -> lengths ->
 * canonical codes -> stream (Algorithm 1 bit order) + paper nibble plane ->
 * bit-serial decode.  out must hold n bytes.  Returns stream bits via *nbits. */
int orc_roundtrip(const uint8_t *x, uint64_t n, uint8_t *out, uint64_t *nbits,
                  uint8_t len_out[ORC_NSYM])
{
    uint64_t freq[ORC_NSYM];
    uint16_t code[ORC_NSYM];
    if (n == 0) return ORC_E_ARG;
    orc_histogram(x, n, freq);
    int rc = orc_huffman_lengths(freq, len_out);
    if (rc < 0) return rc;
    rc = orc_canonical_codes(len_out, code);
    if (rc) return rc;
    uint64_t bits = orc_stream_bits(freq, len_out);
    uint64_t sbytes = (bits + 7) / 8;
    uint8_t *stream = (uint8_t *)calloc(sbytes ? sbytes : 1, 1);
    uint8_t *packed = (uint8_t *)calloc((n + 1) / 2, 1);
    if (!stream || !packed) { free(stream); free(packed); return ORC_E_CAPACITY; }
    uint64_t got = 0;
    rc = orc_encode_exponents(x, n, len_out, code, ORC_MSB_FIRST, stream, sbytes, &got, 0, NULL);
    if (rc == ORC_OK && got != bits) rc = ORC_E_FORMAT;
    if (rc == ORC_OK) {
        orc_pack_nibbles_paper(x, n, packed);
        rc = orc_decode_serial(stream, bits, ORC_MSB_FIRST, len_out, packed, n, out);
    }
    *nbits = bits;
    free(stream);
    free(packed);
    return rc;
}
