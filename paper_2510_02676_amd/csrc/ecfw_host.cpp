// Host side of the wide-alphabet codec (ecfw.h): encoder for E5M2 and BF16
// (Section 3.1 with the 5- or 8-bit exponent field as the symbol), header
// checks and the metadata validator.  The code under the length cap of
// Section 3.1 is built by package-merge, which is optimal under the cap.
#include "ecfw.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <thread>
#include <vector>

#include "ecf8_plan.h"
#include "ecfw_plan.h"

namespace {

inline uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

struct Format {
    uint32_t fmt, alphabet, elem_bytes, piece;   // piece = elements per 16 output bytes
};

bool format_of(uint32_t fmt, Format *f)
{
    if (fmt == ECFW_FMT_E5M2) { *f = {fmt, 32, 1, 16}; return true; }
    if (fmt == ECFW_FMT_BF16) { *f = {fmt, 256, 2, 8}; return true; }
    return false;
}

// exponent field and the remaining bits (sign on top) of element i
template <uint32_t FMT>
inline void split(const uint8_t *x, uint64_t i, uint32_t &sym, uint32_t &rem)
{
    if (FMT == ECFW_FMT_E5M2) {
        const uint32_t b = x[i];
        sym = (b >> 2) & 31u;
        rem = ((b >> 5) & 4u) | (b & 3u);
    } else {
        uint16_t v;
        std::memcpy(&v, x + 2 * i, 2);
        sym = (v >> 7) & 255u;
        rem = ((v >> 8) & 128u) | (v & 127u);
    }
}

bool lane_syms_ok(uint32_t n) { return n == 64 || n == 128; }
bool group_ok(uint32_t g) { return g >= 1 && g <= 64 && (g & (g - 1)) == 0; }

struct Sections {
    uint64_t n_chunks, off_len, off_freq, off_cb, off_lb, off_st, off_pl, off_sg, st_bytes, pl_bytes, sg_bytes, total;
};

Sections make_sections(const Format &f, uint64_t n, uint64_t bits, uint32_t N)
{
    Sections s;
    s.n_chunks = (n + 64ull * N - 1) / (64ull * N);
    s.off_len = 256;
    s.off_freq = s.off_len + round_up(f.alphabet, 256);
    s.off_cb = s.off_freq + round_up(8ull * f.alphabet, 256);
    s.off_lb = s.off_cb + round_up(8 * (s.n_chunks + 1), 256);
    s.off_st = s.off_lb + round_up(128 * s.n_chunks, 256);
    s.st_bytes = round_up((bits + 7) / 8 + 8, 16);
    s.off_pl = s.off_st + round_up(s.st_bytes, 256);
    if (f.fmt == ECFW_FMT_BF16) {
        s.pl_bytes = s.n_chunks * 64 * N;
        s.sg_bytes = 0;
        s.off_sg = 0;
        s.total = s.off_pl + round_up(s.pl_bytes, 256);
    } else {
        s.pl_bytes = s.n_chunks * 16 * N;
        s.sg_bytes = s.n_chunks * 8 * N;
        s.off_sg = s.off_pl + round_up(s.pl_bytes, 256);
        s.total = s.off_sg + round_up(s.sg_bytes, 256);
    }
    return s;
}

// First element of piece q of lane l of chunk c (see the stream section of ecfw.h).
struct ChunkMap {
    uint64_t E, P, G, whole;   // whole = chunks that lie in complete groups
    ChunkMap(uint64_t n, uint32_t N, uint32_t group, uint32_t piece)
        : E(64ull * N), P(piece), G(group), whole(n / (group * 64ull * N) * group) {}
    uint64_t piece(uint64_t c, uint32_t l, uint32_t q) const
    {
        if (c < whole) return (c - c % G) * E + (c % G) * 64 * P + q * (G * 64 * P) + l * P;
        return c * E + q * 64 * P + l * P;
    }
};

// Package-merge (Larmore & Hirschberg): cheapest prefix code with lengths <= lmax.
// Each of the m present symbols is a coin of its weight at every level 1..lmax;
// starting at the deepest level, the items of a level are paired into packages
// that join the next level's coins; the 2m-2 cheapest items of the top level say
// how many levels each symbol was taken at = its code length.
bool capped_lengths(const uint64_t *freq, uint32_t A, uint32_t lmax, uint8_t *len)
{
    std::vector<uint32_t> sym;
    for (uint32_t s = 0; s < A; s++) { len[s] = 0; if (freq[s]) sym.push_back(s); }
    const size_t m = sym.size();
    if (m == 0 || lmax < 1 || lmax > ECFW_MAX_CODE_LEN || (uint64_t)m > (1ull << lmax)) return false;
    if (m == 1) { len[sym[0]] = 1; return true; }
    std::stable_sort(sym.begin(), sym.end(), [&](uint32_t a, uint32_t b) { return freq[a] < freq[b]; });
    struct Item { uint64_t w; std::vector<uint8_t> taken; };   // taken[i]: how often coin i is inside
    std::vector<Item> coins(m);
    for (size_t i = 0; i < m; i++) {
        coins[i].w = freq[sym[i]];
        coins[i].taken.assign(m, 0);
        coins[i].taken[i] = 1;
    }
    std::vector<Item> cur = coins;
    for (uint32_t level = 1; level < lmax; level++) {
        std::vector<Item> packages;
        for (size_t i = 0; i + 1 < cur.size(); i += 2) {
            Item p{cur[i].w + cur[i + 1].w, cur[i].taken};
            for (size_t j = 0; j < m; j++) p.taken[j] = (uint8_t)(p.taken[j] + cur[i + 1].taken[j]);
            packages.push_back(std::move(p));
        }
        std::vector<Item> merged;
        merged.reserve(m + packages.size());
        size_t a = 0, b = 0;
        while (a < m || b < packages.size()) {
            if (b >= packages.size() || (a < m && coins[a].w <= packages[b].w)) merged.push_back(coins[a++]);
            else merged.push_back(std::move(packages[b++]));
        }
        cur.swap(merged);
    }
    std::vector<uint32_t> total(m, 0);
    for (size_t i = 0; i < 2 * m - 2; i++)
        for (size_t j = 0; j < m; j++) total[j] += cur[i].taken[j];
    for (size_t j = 0; j < m; j++) len[sym[j]] = (uint8_t)total[j];
    return true;
}

// Canonical codes ordered by (length, symbol): code = codeword as a number (first bit most
// significant), rcode = the same bit-reversed (first bit = bit 0).  False unless the lengths
// form a prefix code (Kraft sum in (0, 1]).
bool canonical(const uint8_t *len, uint32_t A, uint32_t *code, uint32_t *rcode)
{
    uint32_t count[ECFW_MAX_CODE_LEN + 2] = {0}, next[ECFW_MAX_CODE_LEN + 2] = {0};
    uint64_t kraft = 0;
    for (uint32_t s = 0; s < A; s++) {
        if (len[s] > ECFW_MAX_CODE_LEN) return false;
        if (len[s]) { count[len[s]]++; kraft += 1ull << (ECFW_MAX_CODE_LEN - len[s]); }
    }
    if (kraft == 0 || kraft > (1ull << ECFW_MAX_CODE_LEN)) return false;
    uint32_t c = 0;
    for (uint32_t l = 1; l <= ECFW_MAX_CODE_LEN; l++) { c = (c + count[l - 1]) << 1; next[l] = c; }
    for (uint32_t s = 0; s < A; s++) {
        code[s] = rcode[s] = 0;
        const uint32_t l = len[s];
        if (!l) continue;
        const uint32_t v = next[l]++;
        uint32_t r = 0;
        for (uint32_t b = 0; b < l; b++) r |= ((v >> (l - 1 - b)) & 1u) << b;
        code[s] = v;
        rcode[s] = r;
    }
    return true;
}

template <class F>
void parallel_for(uint64_t n_items, unsigned n_threads, F f)
{
    if (n_threads <= 1 || n_items < 2) { f(0, n_items); return; }
    if (n_threads > n_items) n_threads = (unsigned)n_items;
    std::vector<std::thread> th;
    for (unsigned t = 0; t < n_threads; t++) {
        uint64_t a = n_items * t / n_threads, b = n_items * (t + 1) / n_threads;
        th.emplace_back([=]() { f(a, b); });
    }
    for (auto &t : th) t.join();
}

// Appends bits at an arbitrary bit position of a zeroed buffer shared with other writers: the
// first and last byte a writer touches may hold a neighbour's bits and are OR-ed in atomically.
struct BitWriter {
    uint8_t *buf;
    uint64_t byte;
    uint64_t acc = 0;
    unsigned fill;
    bool first = true;
    BitWriter(uint8_t *b, uint64_t bit) : buf(b), byte(bit >> 3), fill((unsigned)(bit & 7)) {}
    void put(uint32_t bits, unsigned len)
    {
        acc |= (uint64_t)bits << fill;
        fill += len;
        while (fill >= 8) {
            const uint8_t v = (uint8_t)acc;
            if (first) { __atomic_fetch_or(&buf[byte], v, __ATOMIC_RELAXED); first = false; }
            else buf[byte] = v;
            byte++;
            acc >>= 8;
            fill -= 8;
        }
    }
    void finish() { if (fill) __atomic_fetch_or(&buf[byte], (uint8_t)acc, __ATOMIC_RELAXED); }
};

} // namespace

namespace ecfw_internal {

int check_options(const ecfw_encode_opts *opts, uint64_t rows, uint64_t cols, uint32_t *N, uint32_t *group, uint32_t *lmax)
{
    if (!opts || rows == 0 || cols == 0) return ECF8_E_ARG;
    if (cols > UINT64_MAX / rows || rows * cols > (1ull << 48)) return ECF8_E_ARG;
    Format f;
    if (!format_of(opts->fmt, &f)) return ECF8_E_ARG;
    for (uint32_t r : opts->reserved)
        if (r) return ECF8_E_ARG;
    *N = opts->lane_syms ? opts->lane_syms : (f.fmt == ECFW_FMT_BF16 ? 64u : 128u);
    *group = opts->group_chunks ? opts->group_chunks : 32u;
    *lmax = opts->max_code_len ? opts->max_code_len : ECFW_TABLE_BITS;
    if (!lane_syms_ok(*N) || !group_ok(*group) || *lmax > ECFW_MAX_CODE_LEN) return ECF8_E_ARG;
    return ECF8_OK;
}

int plan_encode(const uint64_t *freq, uint32_t fmt, uint64_t rows, uint64_t cols, uint32_t N, uint32_t group,
                uint32_t lmax, WPlan *out)
{
    Format f;
    if (!format_of(fmt, &f)) return ECF8_E_ARG;
    const uint32_t A = f.alphabet;
    const uint64_t n = rows * cols;
    uint64_t fsum = 0;
    for (uint32_t s = 0; s < A; s++) fsum += freq[s];
    if (fsum != n) return ECF8_E_ARG;
    std::memset(out, 0, sizeof(*out));
    if (!capped_lengths(freq, A, lmax, out->len)) return ECF8_E_ARG;   // cap too small for the alphabet in use
    if (!canonical(out->len, A, out->code, out->rcode)) return ECF8_E_FORMAT;
    uint64_t bits = 0;
    uint32_t maxlen = 0, nsym = 0;
    for (uint32_t s = 0; s < A; s++) {
        bits += freq[s] * out->len[s];
        maxlen = std::max<uint32_t>(maxlen, out->len[s]);
        nsym += freq[s] != 0;
    }
    const Sections L = make_sections(f, n, bits, N);
    ecfw_header &h = out->hdr;
    h.magic = ECFW_MAGIC;
    h.version = ECFW_VERSION;
    h.total_size = L.total;
    h.n_elem = n;
    h.rows = rows;
    h.cols = cols;
    h.fmt = fmt;
    h.lane_syms = N;
    h.group_chunks = group;
    h.max_code_len = maxlen;
    h.n_alphabet = A;
    h.n_symbols = nsym;
    h.n_chunks = L.n_chunks;
    h.stream_bits = bits;
    h.off_code_len = L.off_len;
    h.off_freq = L.off_freq;
    h.off_chunk_bit = L.off_cb;
    h.off_lane_bits = L.off_lb;
    h.off_stream = L.off_st;
    h.off_plane = L.off_pl;
    h.off_sign = L.off_sg;
    h.stream_bytes = L.st_bytes;
    h.plane_bytes = L.pl_bytes;
    h.sign_bytes = L.sg_bytes;
    return ECF8_OK;
}

int encode_bound(uint32_t fmt, uint64_t rows, uint64_t cols, uint32_t N, uint32_t lmax, uint64_t *bytes)
{
    Format f;
    if (!format_of(fmt, &f)) return ECF8_E_ARG;
    *bytes = make_sections(f, rows * cols, rows * cols * lmax, N).total;   // the longest stream the cap allows
    return ECF8_OK;
}

} // namespace ecfw_internal

namespace {

template <uint32_t FMT>
int encode_as(const uint8_t *x, uint64_t rows, uint64_t cols, const Format &f, uint32_t N, uint32_t group,
              uint32_t lmax, unsigned nt, ecf8_blob **out)
{
    const uint64_t n = rows * cols;
    const uint32_t A = f.alphabet, P = f.piece, pieces = N / P;
    const ChunkMap map(n, N, group, P);

    // stage 1: histogram of the exponent field
    std::vector<uint64_t> part((size_t)nt * A, 0);
    parallel_for(nt, nt, [&](uint64_t t0, uint64_t t1) {
        for (uint64_t t = t0; t < t1; t++) {
            uint64_t *h = part.data() + t * A;
            for (uint64_t i = n * t / nt, e = n * (t + 1) / nt; i < e; i++) {
                uint32_t s, r;
                split<FMT>(x, i, s, r);
                h[s]++;
            }
        }
    });
    uint64_t freq[256] = {};
    for (unsigned t = 0; t < nt; t++)
        for (uint32_t s = 0; s < A; s++) freq[s] += part[(size_t)t * A + s];

    // stage 2: the code, the layout, the header
    ecfw_internal::WPlan plan;
    const int prc = ecfw_internal::plan_encode(freq, FMT, rows, cols, N, group, lmax, &plan);
    if (prc) return prc;
    const uint8_t *len = plan.len;
    const uint32_t *code = plan.code, *rcode = plan.rcode;
    const ecfw_header &h = plan.hdr;
    const Sections L = make_sections(f, n, h.stream_bits, N);
    uint8_t *blob = (uint8_t *)std::aligned_alloc(256, L.total);
    if (!blob) return ECF8_E_NOMEM;
    std::memset(blob, 0, L.off_st);
    std::memcpy(blob, &h, sizeof(h));
    std::memcpy(blob + L.off_len, len, A);
    std::memcpy(blob + L.off_freq, freq, 8ull * A);

    uint64_t *chunk_bit = (uint64_t *)(blob + L.off_cb);
    uint16_t *lane_bits = (uint16_t *)(blob + L.off_lb);
    uint8_t *stream = blob + L.off_st;
    uint8_t *plane = blob + L.off_pl;
    uint8_t *sign = blob + L.off_sg;

    // stage 3a: code bits of every lane; zero the payload sections in the same sweep
    parallel_for(L.n_chunks, nt, [&](uint64_t c0, uint64_t c1) {
        for (uint64_t c = c0; c < c1; c++) {
            uint64_t tot = 0;
            for (uint32_t l = 0; l < 64; l++) {
                uint32_t lb = 0;
                for (uint32_t q = 0; q < pieces; q++) {
                    const uint64_t a = map.piece(c, l, q), b = std::min<uint64_t>(a + P, n);
                    for (uint64_t i = a; i < b; i++) {
                        uint32_t s, r;
                        split<FMT>(x, i, s, r);
                        lb += len[s];
                    }
                }
                lane_bits[c * 64 + l] = (uint16_t)lb;
                tot += lb;
            }
            chunk_bit[c + 1] = tot;   // turned into a running sum below
        }
        const uint64_t sa = L.st_bytes * c0 / L.n_chunks, sb = L.st_bytes * c1 / L.n_chunks;
        std::memset(stream + sa, 0, sb - sa);
    });
    chunk_bit[0] = 0;
    for (uint64_t c = 0; c < L.n_chunks; c++) chunk_bit[c + 1] += chunk_bit[c];
    std::memset(blob + L.off_st + L.st_bytes, 0, L.total - (L.off_st + L.st_bytes));   // planes and all padding

    // stage 3b: the stream, and the planes of the same stretch of elements
    parallel_for(L.n_chunks, nt, [&](uint64_t c0, uint64_t c1) {
        BitWriter bw(stream, chunk_bit[c0]);
        uint64_t lbuf[34];   // 2048 bits = 16 bits * 128 symbols, + slack for the straddling store
        for (uint64_t c = c0; c < c1; c++)
            for (uint32_t l = 0; l < 64; l++) {
                const uint32_t lb = lane_bits[c * 64 + l];
                if (lb == 0) continue;
                for (uint32_t wi = 0; wi < (lb + 63) / 64 + 1; wi++) lbuf[wi] = 0;
                uint32_t fwd = 0, bwd = lb;
                auto put_local = [&](uint32_t at, uint32_t v, uint32_t nb) {
                    lbuf[at >> 6] |= (uint64_t)v << (at & 63);
                    if ((at & 63) + nb > 64) lbuf[(at >> 6) + 1] |= (uint64_t)v >> (64 - (at & 63));
                };
                for (uint32_t q = 0; q < pieces; q++) {
                    const uint64_t a = map.piece(c, l, q), b = std::min<uint64_t>(a + P, n);
                    for (uint64_t i = a; i < b; i++) {
                        uint32_t s, r;
                        split<FMT>(x, i, s, r);
                        if (q < pieces / 2) { put_local(fwd, rcode[s], len[s]); fwd += len[s]; }
                        else { bwd -= len[s]; put_local(bwd, code[s], len[s]); }
                    }
                }
                for (uint32_t at = 0; at < lb; at += 32) {
                    const uint32_t nb = std::min<uint32_t>(32, lb - at);
                    const uint64_t v = lbuf[at >> 6] >> (at & 63) | ((at & 63) > 32 ? lbuf[(at >> 6) + 1] << (64 - (at & 63)) : 0);
                    bw.put((uint32_t)(nb == 32 ? v : (v & ((1ull << nb) - 1))), nb);
                }
            }
        bw.finish();
        // planes: indexed by element, so a stretch of whole chunks' worth of elements is private to this thread
        const uint64_t a = c0 * map.E, b = std::min<uint64_t>(c1 * map.E, n);
        static const uint32_t swap[4] = {0, 2, 1, 3};
        for (uint64_t i = a; i < b; i++) {
            uint32_t s, r;
            split<FMT>(x, i, s, r);
            if (FMT == ECFW_FMT_BF16) {
                plane[(i / 4) * 4 + swap[i % 4]] = (uint8_t)r;
            } else {
                const uint64_t g = i / 16;
                const uint32_t e = (uint32_t)(i % 16), d = e / 4, j = e % 4;
                uint32_t w;
                std::memcpy(&w, plane + 4 * g, 4);
                w |= (r & 3u) << (8 * j + 2 * d);
                std::memcpy(plane + 4 * g, &w, 4);
                if (r & 4u) sign[2 * g + e / 8] |= (uint8_t)(1u << (e % 8));
            }
        }
    });

    ecf8_blob *bl = new (std::nothrow) ecf8_blob{blob, L.total};
    if (!bl) { std::free(blob); return ECF8_E_NOMEM; }
    *out = bl;
    return ECF8_OK;
}

int check_header(const ecfw_header &h, uint64_t size, Format *f)
{
    if (h.magic != ECFW_MAGIC || h.version != ECFW_VERSION) return ECF8_E_FORMAT;
    if (!format_of(h.fmt, f) || h.n_alphabet != f->alphabet) return ECF8_E_FORMAT;
    if (h.total_size != size || h.n_elem == 0) return ECF8_E_FORMAT;
    if (h.rows == 0 || h.cols == 0 || h.n_elem / h.rows != h.cols || h.n_elem % h.rows) return ECF8_E_FORMAT;
    if (!lane_syms_ok(h.lane_syms) || !group_ok(h.group_chunks)) return ECF8_E_FORMAT;
    if (h.max_code_len < 1 || h.max_code_len > ECFW_MAX_CODE_LEN) return ECF8_E_FORMAT;
    if (h.stream_bits > h.n_elem * ECFW_MAX_CODE_LEN) return ECF8_E_FORMAT;
    const Sections L = make_sections(*f, h.n_elem, h.stream_bits, h.lane_syms);
    if (h.n_chunks != L.n_chunks || h.total_size != L.total) return ECF8_E_FORMAT;
    if (h.off_code_len != L.off_len || h.off_freq != L.off_freq || h.off_chunk_bit != L.off_cb ||
        h.off_lane_bits != L.off_lb || h.off_stream != L.off_st || h.off_plane != L.off_pl ||
        h.off_sign != L.off_sg || h.stream_bytes != L.st_bytes || h.plane_bytes != L.pl_bytes ||
        h.sign_bytes != L.sg_bytes)
        return ECF8_E_FORMAT;
    for (size_t i = 0; i < sizeof(h.reserved); i++)
        if (h.reserved[i]) return ECF8_E_FORMAT;
    return ECF8_OK;
}

int describe(const void *blob_host, uint64_t size, ecfw_header *hdr, Format *f)
{
    if (!blob_host || !hdr) return ECF8_E_ARG;
    if (size < sizeof(ecfw_header)) return ECF8_E_FORMAT;
    std::memcpy(hdr, blob_host, sizeof(ecfw_header));
    int rc = check_header(*hdr, size, f);
    if (rc) return rc;
    const uint8_t *b = (const uint8_t *)blob_host;
    const uint8_t *len = b + hdr->off_code_len;
    uint32_t code[256], rcode[256];
    if (!canonical(len, f->alphabet, code, rcode)) return ECF8_E_FORMAT;
    uint64_t bits = 0, total = 0;
    uint32_t maxlen = 0, nsym = 0;
    for (uint32_t s = 0; s < f->alphabet; s++) {
        uint64_t fr;
        std::memcpy(&fr, b + hdr->off_freq + 8ull * s, 8);
        if (fr && !len[s]) return ECF8_E_FORMAT;
        if (fr > hdr->n_elem) return ECF8_E_FORMAT;
        bits += fr * len[s];
        total += fr;
        nsym += fr != 0;
        maxlen = std::max<uint32_t>(maxlen, len[s]);
    }
    if (bits != hdr->stream_bits || total != hdr->n_elem || maxlen != hdr->max_code_len || nsym != hdr->n_symbols)
        return ECF8_E_FORMAT;
    return ECF8_OK;
}

bool all_zero(const uint8_t *p, uint64_t n)
{
    for (uint64_t i = 0; i < n; i++)
        if (p[i]) return false;
    return true;
}

} // namespace

extern "C" {

int ecfw_encode(const void *elems, uint64_t rows, uint64_t cols, const ecfw_encode_opts *opts, ecf8_blob **out)
{
    if (!elems || !out) return ECF8_E_ARG;
    uint32_t N, group, lmax;
    const int orc = ecfw_internal::check_options(opts, rows, cols, &N, &group, &lmax);
    if (orc) return orc;
    Format f;
    format_of(opts->fmt, &f);
    unsigned nt = opts->n_threads ? opts->n_threads : std::thread::hardware_concurrency();
    if (nt == 0) nt = 1;
    if (nt > 64) nt = 64;
    if (rows * cols < (1u << 16)) nt = 1;
    try {
        const uint8_t *x = (const uint8_t *)elems;
        return f.fmt == ECFW_FMT_BF16 ? encode_as<ECFW_FMT_BF16>(x, rows, cols, f, N, group, lmax, nt, out)
                                      : encode_as<ECFW_FMT_E5M2>(x, rows, cols, f, N, group, lmax, nt, out);
    } catch (const std::bad_alloc &) {
        return ECF8_E_NOMEM;
    } catch (...) {
        return ECF8_E_ARG;
    }
}

int ecfw_blob_describe(const void *blob_host, uint64_t size, ecfw_header *hdr)
{
    Format f;
    return describe(blob_host, size, hdr, &f);
}

int ecfw_blob_validate(const void *blob_host, uint64_t size)
{
    ecfw_header h;
    Format f;
    int rc = describe(blob_host, size, &h, &f);
    if (rc) return rc;
    const uint8_t *b = (const uint8_t *)blob_host;
    const uint64_t *cb = (const uint64_t *)(b + h.off_chunk_bit);
    const uint16_t *lb = (const uint16_t *)(b + h.off_lane_bits);
    if (cb[0] != 0 || cb[h.n_chunks] != h.stream_bits) return ECF8_E_FORMAT;
    const uint64_t E = 64ull * h.lane_syms;
    for (uint64_t c = 0; c < h.n_chunks; c++) {
        uint64_t tot = 0;
        const bool whole = (c + 1) * E <= h.n_elem || c < h.n_elem / (h.group_chunks * E) * h.group_chunks;
        for (uint32_t l = 0; l < 64; l++) {
            const uint32_t v = lb[c * 64 + l];
            if (v > h.lane_syms * h.max_code_len) return ECF8_E_FORMAT;
            if (whole && v < h.lane_syms) return ECF8_E_FORMAT;   // N codewords of at least one bit each
            tot += v;
        }
        if (cb[c + 1] < cb[c] || cb[c + 1] - cb[c] != tot) return ECF8_E_FORMAT;
    }
    // padding: between sections, behind the stream's last bit, behind the last element's plane bits
    auto gap_zero = [&](uint64_t from, uint64_t to) { return from <= to && all_zero(b + from, to - from); };
    if (!gap_zero(sizeof(ecfw_header), h.off_code_len) || !gap_zero(h.off_code_len + f.alphabet, h.off_freq) ||
        !gap_zero(h.off_freq + 8ull * f.alphabet, h.off_chunk_bit) ||
        !gap_zero(h.off_chunk_bit + 8 * (h.n_chunks + 1), h.off_lane_bits) ||
        !gap_zero(h.off_lane_bits + 128 * h.n_chunks, h.off_stream))
        return ECF8_E_FORMAT;
    const uint64_t used = (h.stream_bits + 7) / 8;
    if (h.stream_bits % 8 && (b[h.off_stream + used - 1] >> (h.stream_bits % 8))) return ECF8_E_FORMAT;
    if (!gap_zero(h.off_stream + used, h.off_plane)) return ECF8_E_FORMAT;
    if (h.fmt == ECFW_FMT_BF16) {
        // bytes of elements >= n_elem: whole groups of four past the end, and the tail group's unused slots
        const uint64_t full = round_up(h.n_elem, 4);
        if (!gap_zero(h.off_plane + full, h.total_size)) return ECF8_E_FORMAT;
        static const uint32_t swap[4] = {0, 2, 1, 3};
        for (uint64_t i = h.n_elem; i < full; i++)
            if (b[h.off_plane + (i / 4) * 4 + swap[i % 4]]) return ECF8_E_FORMAT;
    } else {
        const uint64_t pieces = (h.n_elem + 15) / 16;
        if (!gap_zero(h.off_plane + 4 * pieces, h.off_sign) || !gap_zero(h.off_sign + 2 * pieces, h.total_size))
            return ECF8_E_FORMAT;
        for (uint64_t i = h.n_elem; i < pieces * 16; i++) {
            const uint32_t e = (uint32_t)(i % 16), d = e / 4, j = e % 4;
            uint32_t w;
            std::memcpy(&w, b + h.off_plane + 4 * (i / 16), 4);
            if ((w >> (8 * j + 2 * d)) & 3u) return ECF8_E_FORMAT;
            if ((b[h.off_sign + 2 * (i / 16) + e / 8] >> (e % 8)) & 1u) return ECF8_E_FORMAT;
        }
    }
    return ECF8_OK;
}

} // extern "C"
