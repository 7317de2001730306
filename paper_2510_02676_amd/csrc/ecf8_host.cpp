// Host side of the ECF8 library: encoder, container parsing and validation.
//
// Encoder stages follow Section 3.1 of the paper: exponent histogram and
// optimal prefix code ("Huffman code generation"), then the bitstream with
// synchronisation metadata ("Encoding and synchronization metadata
// generation").  The paper's metadata (a 4-bit gap per fixed-size byte window
// and an output position per block) is replaced by the number of stream bits
// of every lane's N codewords, which removes the decoder's counting pass.
// The stream is the concatenation of the lanes' bits chunk by chunk, lane by
// lane; lane l codes the 16-element pieces l, l+64, ... of its chunk, so that
// what the 64 lanes decode in the same step is contiguous in the output.  The
// first half of a lane's symbols is written forward from the lane's first bit,
// the second half backward from its last bit: the decoder runs both halves as
// two independent dependency chains without any extra metadata.
#include "ecf8.h"
#include "ecf8_table.h"
#include "ecf8_plan.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <thread>
#include <vector>

namespace {

inline uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

bool lane_syms_ok(uint32_t n) { return n == 32 || n == 64 || n == 128; }
bool group_ok(uint32_t g) { return g >= 1 && g <= 64 && (g & (g - 1)) == 0; }

// Where chunk c's pieces lie: piece q of lane l is the 16 elements from piece(c, l, q).
// Linear layout: chunks of whole groups are interleaved KiB by KiB, the rest of the tensor is
// chunk-major.  Row-tiled layout: a chunk is a block of 16 rows x 4N columns, lane l works on
// row l % 16, its piece q on columns 64 q + 16 (l / 16) of the block.
struct ChunkMap {
    uint64_t E, G, grouped; // elements per chunk, chunks per group, chunks that lie in whole groups
    uint64_t cols, KC;      // row-tiled: columns of the matrix, chunks per block of rows; KC = 0: linear
    ChunkMap(uint64_t n, uint64_t cols_, uint32_t N, uint32_t group, uint32_t tile_rows)
        : E(64ull * N), G(group), grouped(n / (group * 64ull * N) * group), cols(cols_),
          KC(tile_rows ? cols_ / (4ull * N) : 0) {}
    uint64_t piece(uint64_t c, uint32_t l, uint32_t q) const
    {
        if (KC) return ((c / KC) * 16 + (l & 15)) * cols + (c % KC) * (E / 16) + 64ull * q + 16ull * (l >> 4);
        if (c < grouped) return (c - c % G) * E + (c % G) * 1024 + q * G * 1024 + l * 16ull;
        return c * E + q * 1024ull + l * 16ull;
    }
};
bool tiling_ok(uint32_t tile_rows, uint32_t group, uint64_t rows, uint64_t cols, uint32_t N)
{
    if (tile_rows == 0) return true;
    // at most 2^40 elements: the decode kernels number a row-tiled tensor's chunks in 32 bits
    return tile_rows == 16 && group == 1 && rows % 16 == 0 && cols != 0 && cols % (4ull * N) == 0 && rows <= (1ull << 40) / cols;
}

// Optimal prefix-code lengths by the two-queue method: leaves sorted by weight
// in one queue, merged nodes (created in non-decreasing weight) in a second;
// each step joins the two smallest heads.  16 symbols give depth <= 15.
void huffman_lengths(const uint64_t freq[16], uint8_t len[16])
{
    struct Node { uint64_t w; int left, right; };
    std::vector<Node> nodes;
    std::vector<int> leaves;
    for (int s = 0; s < 16; s++) {
        len[s] = 0;
        if (freq[s]) { nodes.push_back({freq[s], -1 - s, -1 - s}); leaves.push_back((int)nodes.size() - 1); }
    }
    if (leaves.empty()) return;
    if (leaves.size() == 1) { len[-1 - nodes[leaves[0]].left] = 1; return; } // lone symbol: code "0"
    std::stable_sort(leaves.begin(), leaves.end(), [&](int a, int b) { return nodes[a].w < nodes[b].w; });
    std::vector<int> merged;
    size_t li = 0, mi = 0;
    auto take = [&]() {
        bool use_leaf = li < leaves.size() && (mi >= merged.size() || nodes[leaves[li]].w <= nodes[merged[mi]].w);
        return use_leaf ? leaves[li++] : merged[mi++];
    };
    size_t remaining = leaves.size();
    while (remaining > 1) {
        int a = take(), b = take();
        nodes.push_back({nodes[a].w + nodes[b].w, a, b});
        merged.push_back((int)nodes.size() - 1);
        remaining--;
    }
    // depth of every leaf, iteratively from the root
    std::vector<std::pair<int, int>> stack{{merged.back(), 0}};
    while (!stack.empty()) {
        auto [n, d] = stack.back();
        stack.pop_back();
        if (nodes[n].left < 0) { len[-1 - nodes[n].left] = (uint8_t)d; continue; }
        stack.push_back({nodes[n].left, d + 1});
        stack.push_back({nodes[n].right, d + 1});
    }
}

// Cheapest code with every length <= lmax (package-merge): every symbol is a coin of weight
// f at each of the lmax levels; level by level from the deepest, neighbouring pairs of the
// sorted list are packaged and merged with the next level's coins; the 2k-2 cheapest items
// of the last list say how often each symbol was taken = its code length.  A package is its
// weight plus a 4-bit counter per symbol (a symbol enters at most once per level, lmax <= 15).
void capped_lengths(const uint64_t freq[16], uint32_t lmax, uint8_t len[16])
{
    huffman_lengths(freq, len);
    uint32_t mx = 0, k = 0;
    for (int s = 0; s < 16; s++) { mx = std::max<uint32_t>(mx, len[s]); k += freq[s] != 0; }
    if (mx <= lmax || k < 2) return;   // the cap does not bind
    struct Item { uint64_t w, taken; };
    std::vector<Item> coins;
    for (int s = 0; s < 16; s++)
        if (freq[s]) coins.push_back({freq[s], 1ull << (4 * s)});
    auto by_weight = [](const Item &a, const Item &b) { return a.w < b.w; };
    std::stable_sort(coins.begin(), coins.end(), by_weight);
    std::vector<Item> cur = coins, next;
    for (uint32_t level = 1; level < lmax; level++) {
        next.clear();
        for (size_t i = 0; i + 1 < cur.size(); i += 2) next.push_back({cur[i].w + cur[i + 1].w, cur[i].taken + cur[i + 1].taken});
        std::vector<Item> merged(coins.size() + next.size());
        std::merge(coins.begin(), coins.end(), next.begin(), next.end(), merged.begin(), by_weight);
        cur.swap(merged);
    }
    uint64_t taken = 0;
    for (size_t i = 0; i < 2 * (size_t)k - 2; i++) taken += cur[i].taken;
    for (int s = 0; s < 16; s++) len[s] = (uint8_t)((taken >> (4 * s)) & 15);
}

// Canonical codes ordered by (length, symbol).  code = the codeword as a number
// (first bit most significant); rcode = the same with its bit order reversed, so
// that its first bit is bit 0.  Forward runs place rcode at ascending stream
// bits, backward runs place code so that its first bit is the highest.
bool canonical(const uint8_t len[16], uint32_t rcode[16], uint32_t code_out[16] = nullptr)
{
    uint32_t count[17] = {0}, next[17] = {0};
    for (int s = 0; s < 16; s++) { if (len[s] > 15) return false; count[len[s]]++; }
    count[0] = 0;
    uint32_t code = 0;
    for (int l = 1; l <= 15; l++) { code = (code + count[l - 1]) << 1; next[l] = code; }
    uint64_t kraft = 0;
    for (int s = 0; s < 16; s++) {
        rcode[s] = 0;
        if (code_out) code_out[s] = 0;
        int l = len[s];
        if (!l) continue;
        kraft += 1ull << (15 - l);
        uint32_t c = next[l]++;
        uint32_t r = 0;
        for (int b = 0; b < l; b++) r |= ((c >> (l - 1 - b)) & 1u) << b;
        rcode[s] = r;
        if (code_out) code_out[s] = c;
    }
    return kraft <= (1ull << 15) && kraft > 0;
}

// The decoder's pair table (entry format in ecf8_table.h) from the code lengths.
void build_pair_table(const uint8_t len[16], uint16_t *tbl)
{
    uint32_t rcode[16];
    canonical(len, rcode);
    std::vector<uint16_t> one(ECF8_TBL_ENTRIES, 0); // single-symbol facts: symbol | length << 4
    for (uint32_t s = 0; s < 16; s++) {
        uint32_t l = len[s];
        if (l == 0 || l > ECF8_TB) continue;
        for (uint32_t j = 0; j < (1u << (ECF8_TB - l)); j++) one[rcode[s] | (j << l)] = (uint16_t)(s | (l << 4));
    }
    for (uint32_t idx = 0; idx < ECF8_TBL_ENTRIES; idx++) {
        uint32_t t1 = one[idx], l1 = t1 >> 4;
        uint32_t t2 = l1 ? one[idx >> l1] : 0;
        tbl[idx] = ecf8_pair_entry(t1 & 15u, l1, t2 & 15u, t2 >> 4);
    }
}

struct Layout {
    uint64_t n_chunks, off_cb, off_lb, off_st, st_bytes, off_pl, pl_bytes, total;
};

Layout make_layout(uint64_t n, uint64_t bits, uint32_t N, uint32_t table_bits)
{
    Layout L;
    uint64_t chunk = (uint64_t)ECF8_LANES * N;
    L.n_chunks = (n + chunk - 1) / chunk;
    L.off_cb = 256 + (table_bits ? (2ull << table_bits) : 0);
    L.off_lb = round_up(L.off_cb + 8 * (L.n_chunks + 1), 256);
    L.off_st = round_up(L.off_lb + 2 * L.n_chunks * ECF8_LANES, 256);
    L.st_bytes = round_up((bits + 7) / 8 + 8, 16);
    L.off_pl = round_up(L.off_st + L.st_bytes, 256);
    L.pl_bytes = L.n_chunks * 32ull * N;
    L.total = round_up(L.off_pl + L.pl_bytes, 256);
    return L;
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

// Appends code bits at an arbitrary bit position of a zero-initialised buffer
// shared with other writers: the first and the last byte a writer touches may
// also hold a neighbour's bits and are OR-ed in atomically; bytes in between
// belong to this writer alone.
struct BitWriter {
    uint8_t *buf;
    uint64_t byte;
    uint64_t acc = 0;
    unsigned fill;
    bool first = true;
    BitWriter(uint8_t *b, uint64_t bit) : buf(b), byte(bit >> 3), fill((unsigned)(bit & 7)) {}
    void put(uint32_t rcode, unsigned len)
    {
        acc |= (uint64_t)rcode << fill;
        fill += len;
        while (fill >= 8) {
            uint8_t v = (uint8_t)acc;
            if (first) { __atomic_fetch_or(&buf[byte], v, __ATOMIC_RELAXED); first = false; }
            else buf[byte] = v;
            byte++;
            acc >>= 8;
            fill -= 8;
        }
    }
    void finish()
    {
        if (fill) __atomic_fetch_or(&buf[byte], (uint8_t)acc, __ATOMIC_RELAXED);
    }
};

int check_header(const ecf8_header &h, uint64_t size)
{
    if (h.magic != ECF8_MAGIC || h.version != ECF8_VERSION) return ECF8_E_FORMAT;
    if (h.total_size != size || h.n_elem == 0) return ECF8_E_FORMAT;
    if (h.rows == 0 || h.cols == 0 || h.n_elem / h.rows != h.cols || h.n_elem % h.rows) return ECF8_E_FORMAT;
    if ((h.table_bits != 0 && h.table_bits != ECF8_TB) || !lane_syms_ok(h.lane_syms) || !group_ok(h.group_chunks) ||
        !tiling_ok(h.tile_rows, h.group_chunks, h.rows, h.cols, h.lane_syms))
        return ECF8_E_FORMAT;
    if (h.stream_bits > h.n_elem * 15 || h.stream_bits < h.n_elem) return ECF8_E_FORMAT;
    Layout L = make_layout(h.n_elem, h.stream_bits, h.lane_syms, h.table_bits);
    if (h.n_chunks != L.n_chunks || h.off_chunk_bit != L.off_cb || h.off_lane_bits != L.off_lb ||
        h.off_stream != L.off_st || h.off_plane != L.off_pl || h.stream_bytes != L.st_bytes ||
        h.plane_bytes != L.pl_bytes || h.total_size != L.total)
        return ECF8_E_FORMAT;
    uint32_t rc[16];
    if (!canonical(h.code_len, rc)) return ECF8_E_FORMAT;
    uint64_t fsum = 0, wsum = 0;
    for (int s = 0; s < 16; s++) {
        if ((h.freq[s] != 0) != (h.code_len[s] != 0)) return ECF8_E_FORMAT;
        fsum += h.freq[s];
        wsum += h.freq[s] * h.code_len[s];
    }
    if (fsum != h.n_elem || wsum != h.stream_bits) return ECF8_E_FORMAT;
    return ECF8_OK;
}

} // namespace

namespace ecf8_internal {

int check_options(uint64_t rows, uint64_t cols, const ecf8_encode_opts *opts, uint32_t *lane_syms,
                  uint32_t *group_chunks, uint32_t *max_code_len, uint32_t *tile_rows, uint32_t *table_mode)
{
    if (rows == 0 || cols == 0) return ECF8_E_ARG;
    if (rows > (1ull << 40) / cols) return ECF8_E_ARG;
    const uint32_t tr = opts ? opts->tile_rows : 0;
    const uint32_t group = (opts && opts->group_chunks) ? opts->group_chunks : (tr ? 1 : 32);
    const uint32_t lmax = (opts && opts->max_code_len) ? opts->max_code_len : ECF8_TB / 2;
    // symbols per lane: 128 under the default cap; 64 where longer codewords are allowed, the shape the
    // decode kernels for such codes run fastest at (more waves, a chunk's pieces stored in one burst)
    const uint32_t N = (opts && opts->lane_syms) ? opts->lane_syms : (lmax > ECF8_TB / 2 ? 64 : 128);
    const uint32_t tmode = opts ? opts->table_mode : 0;
    if (!lane_syms_ok(N) || !group_ok(group) || lmax < 4 || lmax > 15 || tmode > 2) return ECF8_E_ARG;
    if (!tiling_ok(tr, group, rows, cols, N)) return ECF8_E_ARG;
    *lane_syms = N;
    *group_chunks = group;
    *max_code_len = lmax;
    *tile_rows = tr;
    *table_mode = tmode;
    return ECF8_OK;
}

int plan_encode(const uint64_t freq[16], uint64_t rows, uint64_t cols, const ecf8_encode_opts *opts, Plan *out)
{
    uint32_t N, group, lmax, tile_rows, tmode;
    int rc = check_options(rows, cols, opts, &N, &group, &lmax, &tile_rows, &tmode);
    if (rc) return rc;
    const uint64_t n = rows * cols;
    uint64_t fsum = 0;
    for (int s = 0; s < 16; s++) fsum += freq[s];
    if (fsum != n) return ECF8_E_ARG;
    uint8_t len[16];
    capped_lengths(freq, lmax, len);
    if (!canonical(len, out->rcode, out->code)) return ECF8_E_FORMAT;
    uint64_t bits = 0;
    for (int s = 0; s < 16; s++) bits += freq[s] * len[s];
    const uint32_t table_bits = (tmode == 1 || (tmode == 0 && n >= (1ull << 22))) ? ECF8_TB : 0;
    const Layout L = make_layout(n, bits, N, table_bits);
    ecf8_header &h = out->hdr;
    std::memset(&h, 0, sizeof(h));
    h.magic = ECF8_MAGIC;
    h.version = ECF8_VERSION;
    h.total_size = L.total;
    h.n_elem = n;
    h.rows = rows;
    h.cols = cols;
    h.lane_syms = N;
    h.table_bits = (uint16_t)table_bits;
    h.group_chunks = (uint8_t)group;
    h.tile_rows = (uint8_t)tile_rows;
    h.n_chunks = L.n_chunks;
    h.stream_bits = bits;
    std::memcpy(h.code_len, len, 16);
    h.off_chunk_bit = L.off_cb;
    h.off_lane_bits = L.off_lb;
    h.off_stream = L.off_st;
    h.off_plane = L.off_pl;
    h.stream_bytes = L.st_bytes;
    h.plane_bytes = L.pl_bytes;
    std::memcpy(h.freq, freq, 16 * sizeof(uint64_t));
    return ECF8_OK;
}

int encode_bound(uint64_t rows, uint64_t cols, const ecf8_encode_opts *opts, uint64_t *bytes)
{
    uint32_t N, group, lmax, tile_rows, tmode;
    int rc = check_options(rows, cols, opts, &N, &group, &lmax, &tile_rows, &tmode);
    if (rc) return rc;
    const uint64_t n = rows * cols;
    // longest stream and an embedded table, whatever the histogram turns out to be
    *bytes = make_layout(n, n * lmax, N, tmode == 2 ? 0 : ECF8_TB).total;
    return ECF8_OK;
}

void build_pair_table_host(const uint8_t len[16], uint16_t *tbl) { build_pair_table(len, tbl); }

} // namespace ecf8_internal

extern "C" {

int ecf8_encode(const uint8_t *x, uint64_t rows, uint64_t cols, const ecf8_encode_opts *opts,
                ecf8_blob **out)
{
    if (!x || !out) return ECF8_E_ARG;
    uint32_t N, group, lmax, tile_rows, tmode;
    int orc = ecf8_internal::check_options(rows, cols, opts, &N, &group, &lmax, &tile_rows, &tmode);
    if (orc) return orc;
    const uint64_t n = rows * cols;
    const ChunkMap map(n, cols, N, group, tile_rows);
    unsigned nt = (opts && opts->n_threads) ? opts->n_threads : std::thread::hardware_concurrency();
    if (nt == 0) nt = 1;
    if (nt > 64) nt = 64;
    if (n < (1u << 16)) nt = 1;

    try {
        // stage 1: histogram of the exponent field, per thread then summed
        std::vector<uint64_t> part((size_t)nt * 16, 0);
        {
            std::vector<std::thread> th;
            for (unsigned t = 0; t < nt; t++)
                th.emplace_back([&, t]() {
                    uint64_t a = n * t / nt, b = n * (t + 1) / nt;
                    uint64_t h[4][16] = {};
                    uint64_t i = a;
                    for (; i + 4 <= b; i += 4) {
                        h[0][(x[i] >> 3) & 15]++;
                        h[1][(x[i + 1] >> 3) & 15]++;
                        h[2][(x[i + 2] >> 3) & 15]++;
                        h[3][(x[i + 3] >> 3) & 15]++;
                    }
                    for (; i < b; i++) h[0][(x[i] >> 3) & 15]++;
                    for (int s = 0; s < 16; s++) part[(size_t)t * 16 + s] = h[0][s] + h[1][s] + h[2][s] + h[3][s];
                });
            for (auto &t : th) t.join();
        }
        uint64_t freq[16] = {};
        for (unsigned t = 0; t < nt; t++)
            for (int s = 0; s < 16; s++) freq[s] += part[(size_t)t * 16 + s];

        ecf8_internal::Plan plan;
        int prc = ecf8_internal::plan_encode(freq, rows, cols, opts, &plan);
        if (prc) return prc;
        const uint8_t *len = plan.hdr.code_len;
        const uint32_t *rcode = plan.rcode, *code = plan.code;
        Layout L = make_layout(n, plan.hdr.stream_bits, N, plan.hdr.table_bits);
        uint8_t *blob = (uint8_t *)std::aligned_alloc(256, L.total);
        if (!blob) return ECF8_E_NOMEM;
        std::memset(blob, 0, L.off_st); // header and metadata; payload sections are zeroed by their writers
        std::memcpy(blob, &plan.hdr, sizeof(ecf8_header));
        if (plan.hdr.table_bits) build_pair_table(len, (uint16_t *)(blob + 256));

        uint64_t *chunk_bit = (uint64_t *)(blob + L.off_cb);
        uint16_t *lane_bits = (uint16_t *)(blob + L.off_lb);
        uint8_t *stream = blob + L.off_st;
        uint8_t *plane = blob + L.off_pl;
        const uint64_t chunk_elems = (uint64_t)ECF8_LANES * N;

        // stage 2a: code bits of every lane; zero the payload sections in the same sweep
        parallel_for(L.n_chunks, nt, [&](uint64_t c0, uint64_t c1) {
            for (uint64_t c = c0; c < c1; c++) {
                uint64_t tot = 0;
                for (uint32_t l = 0; l < ECF8_LANES; l++) {
                    uint32_t lb = 0;
                    for (uint32_t q = 0; q < N / 16; q++) {
                        uint64_t a = map.piece(c, l, q);
                        uint64_t b = std::min<uint64_t>(a + 16, n);
                        for (uint64_t i = a; i < b; i++) lb += len[(x[i] >> 3) & 15];
                    }
                    lane_bits[c * ECF8_LANES + l] = (uint16_t)lb;
                    tot += lb;
                }
                chunk_bit[c + 1] = tot; // turned into a running sum below
            }
            uint64_t pa = L.pl_bytes * c0 / L.n_chunks, pb = L.pl_bytes * c1 / L.n_chunks;
            std::memset(plane + pa, 0, pb - pa);
            uint64_t sa = L.st_bytes * c0 / L.n_chunks, sb = L.st_bytes * c1 / L.n_chunks;
            std::memset(stream + sa, 0, sb - sa);
        });
        chunk_bit[0] = 0;
        for (uint64_t c = 0; c < L.n_chunks; c++) chunk_bit[c + 1] += chunk_bit[c];
        std::memset(blob + L.off_pl + L.pl_bytes, 0, L.total - (L.off_pl + L.pl_bytes));
        std::memset(blob + L.off_st + L.st_bytes, 0, L.off_pl - (L.off_st + L.st_bytes));

        // stage 2b: emit the stream and the regrouped nibble plane
        parallel_for(L.n_chunks, nt, [&](uint64_t c0, uint64_t c1) {
            BitWriter bw(stream, chunk_bit[c0]);
            uint64_t a = c0 * chunk_elems, b = std::min<uint64_t>(c1 * chunk_elems, n);
            // A lane's bits are assembled in a local buffer: the first half of its pieces
            // forward from bit 0, the second half backward from its last bit; then the
            // buffer is appended to the stream.  Lanes follow each other lane by lane.
            uint64_t lbuf[32]; // 2048 bits >= 15 bits * 128 symbols
            const uint32_t P = N / 16;
            for (uint64_t c = c0; c < c1; c++)
                for (uint32_t l = 0; l < ECF8_LANES; l++) {
                    const uint32_t lb = lane_bits[c * ECF8_LANES + l];
                    if (lb == 0) continue;
                    const uint32_t words = (lb + 63) / 64;
                    for (uint32_t wi = 0; wi < words; wi++) lbuf[wi] = 0;
                    uint32_t fwd = 0, bwd = lb;
                    auto put_local = [&](uint32_t at, uint32_t bits, uint32_t nb) {
                        lbuf[at >> 6] |= (uint64_t)bits << (at & 63);
                        if ((at & 63) + nb > 64) lbuf[(at >> 6) + 1] |= (uint64_t)bits >> (64 - (at & 63));
                    };
                    for (uint32_t q = 0; q < P; q++) {
                        uint64_t pa = map.piece(c, l, q);
                        uint64_t pb = std::min<uint64_t>(pa + 16, n);
                        for (uint64_t i = pa; i < pb; i++) {
                            uint32_t e = (x[i] >> 3) & 15;
                            if (q < P / 2) { put_local(fwd, rcode[e], len[e]); fwd += len[e]; }
                            else { bwd -= len[e]; put_local(bwd, code[e], len[e]); }
                        }
                    }
                    for (uint32_t at = 0; at < lb; at += 32) {
                        uint32_t nb = std::min<uint32_t>(32, lb - at);
                        uint64_t v = lbuf[at >> 6] >> (at & 63);
                        bw.put((uint32_t)(nb == 32 ? v : (v & ((1ull << nb) - 1))), nb);
                    }
                }
            bw.finish();
            // plane: 8 elements -> 4 bytes, element j pairs with element j+4
            uint64_t i = a;
            for (; i + 8 <= b; i += 8) {
                uint8_t *p = plane + (i / 8) * 4;
                for (int j = 0; j < 4; j++) {
                    uint8_t lo = x[i + j], hi = x[i + 4 + j];
                    uint8_t ql = (uint8_t)(((lo >> 4) & 8) | (lo & 7));
                    uint8_t qh = (uint8_t)(((hi >> 4) & 8) | (hi & 7));
                    p[j] = (uint8_t)(ql | (qh << 4));
                }
            }
            for (; i < b; i++) {
                uint8_t v = x[i];
                uint8_t q = (uint8_t)(((v >> 4) & 8) | (v & 7));
                uint8_t *p = plane + (i / 8) * 4 + (i % 4);
                *p |= ((i % 8) < 4) ? q : (uint8_t)(q << 4);
            }
        });

        ecf8_blob *bl = new (std::nothrow) ecf8_blob{blob, L.total};
        if (!bl) { std::free(blob); return ECF8_E_NOMEM; }
        *out = bl;
        return ECF8_OK;
    } catch (const std::bad_alloc &) {
        return ECF8_E_NOMEM;
    } catch (...) {
        return ECF8_E_ARG;
    }
}

void ecf8_blob_free(ecf8_blob *b)
{
    if (!b) return;
    std::free(b->data);
    delete b;
}

const void *ecf8_blob_data(const ecf8_blob *b) { return b ? b->data : nullptr; }
uint64_t ecf8_blob_size(const ecf8_blob *b) { return b ? b->size : 0; }

int ecf8_blob_describe(const void *blob, uint64_t size, ecf8_header *hdr)
{
    if (!blob || !hdr) return ECF8_E_ARG;
    if (size < sizeof(ecf8_header)) return ECF8_E_FORMAT;
    ecf8_header h;
    std::memcpy(&h, blob, sizeof(h));
    int rc = check_header(h, size);
    if (rc) return rc;
    *hdr = h;
    return ECF8_OK;
}

int ecf8_blob_validate(const void *blob, uint64_t size)
{
    ecf8_header h;
    int rc = ecf8_blob_describe(blob, size, &h);
    if (rc) return rc;
    const uint8_t *p = (const uint8_t *)blob;
    const uint32_t N = h.lane_syms;
    if (h.table_bits) {
        std::vector<uint16_t> want(ECF8_TBL_ENTRIES);
        build_pair_table(h.code_len, want.data());
        if (std::memcmp(want.data(), p + 256, 2ull << h.table_bits) != 0) return ECF8_E_FORMAT;
    }
    const ChunkMap map(h.n_elem, h.cols, N, h.group_chunks, h.tile_rows);
    uint64_t prev;
    std::memcpy(&prev, p + h.off_chunk_bit, 8);
    if (prev != 0) return ECF8_E_FORMAT;
    for (uint64_t c = 0; c < h.n_chunks; c++) {
        uint64_t next;
        std::memcpy(&next, p + h.off_chunk_bit + 8 * (c + 1), 8);
        uint64_t tot = 0;
        for (uint32_t l = 0; l < ECF8_LANES; l++) {
            uint16_t lb;
            std::memcpy(&lb, p + h.off_lane_bits + 2 * (c * ECF8_LANES + l), 2);
            uint64_t cnt = 0; // elements of the lane's pieces that exist
            for (uint32_t q = 0; q < N / 16; q++) {
                uint64_t a = map.piece(c, l, q);
                if (a < h.n_elem) cnt += std::min<uint64_t>(16, h.n_elem - a);
            }
            if (lb > 15 * cnt || lb < cnt) return ECF8_E_FORMAT;
            tot += lb;
        }
        if (next < prev || next - prev != tot) return ECF8_E_FORMAT;
        prev = next;
    }
    if (prev != h.stream_bits) return ECF8_E_FORMAT;
    // zero padding after the last stream bit
    const uint8_t *st = p + h.off_stream;
    for (uint64_t b = h.stream_bits; b < h.stream_bytes * 8; b++) {
        if ((b & 7) == 0 && b + 8 <= h.stream_bytes * 8) {
            if (st[b >> 3]) return ECF8_E_FORMAT;
            b += 7;
        } else if ((st[b >> 3] >> (b & 7)) & 1) return ECF8_E_FORMAT;
    }
    return ECF8_OK;
}

int ecf8_blob_stats(const ecf8_header *h, ecf8_stats *s)
{
    if (!h || !s || h->n_elem == 0) return ECF8_E_ARG;
    double n = (double)h->n_elem, H = 0;
    uint32_t mx = 0, ns = 0;
    for (int i = 0; i < 16; i++) {
        if (!h->freq[i]) continue;
        double p = (double)h->freq[i] / n;
        H -= p * std::log2(p);
        ns++;
        mx = std::max<uint32_t>(mx, h->code_len[i]);
    }
    s->entropy_bits = H;
    s->avg_code_bits = (double)h->stream_bits / n;
    s->bits_per_weight = 8.0 * (double)h->total_size / n;
    s->ratio = (double)h->total_size / n;
    s->max_code_len = mx;
    s->n_symbols = ns;
    return ECF8_OK;
}

int ecf8_batch_prepare(const ecf8_header *hdrs, const void *const *d_blobs, void *const *d_outs,
                       const uint64_t *caps, uint32_t n, ecf8_batch_item *items, ecf8_batch_info *info)
{
    if (!hdrs || !d_blobs || !d_outs || !caps || !items || !info || n == 0) return ECF8_E_ARG;
    uint64_t first = 0;
    uint32_t max_len = 0;
    bool all_tiled = true;
    for (uint32_t i = 0; i < n; i++) {
        const ecf8_header &h = hdrs[i];
        int rc = check_header(h, h.total_size);
        if (rc) return rc;
        if (h.lane_syms != hdrs[0].lane_syms) return ECF8_E_ARG;
        if (!d_blobs[i] || !d_outs[i]) return ECF8_E_ARG;
        if (((uintptr_t)d_blobs[i] | (uintptr_t)d_outs[i]) & 15) return ECF8_E_ALIGN;
        if (caps[i] < h.n_elem) return ECF8_E_CAPACITY;
        ecf8_batch_item &it = items[i];
        std::memset(&it, 0, sizeof(it));
        it.d_blob = (uint64_t)(uintptr_t)d_blobs[i];
        it.d_out = (uint64_t)(uintptr_t)d_outs[i];
        it.n_elem = h.n_elem;
        it.n_chunks = h.n_chunks;
        it.first_chunk = first;
        it.off_chunk_bit = h.off_chunk_bit;
        it.off_lane_bits = h.off_lane_bits;
        it.off_stream = h.off_stream;
        it.off_plane = h.off_plane;
        it.stream_bytes = h.stream_bytes;
        it.off_table = h.table_bits ? 256 : 0;
        it.group_chunks = h.group_chunks;
        it.tile_cols = h.tile_rows ? h.cols : 0;
        std::memcpy(it.code_len, h.code_len, 16);
        for (int s = 0; s < 16; s++) max_len = std::max<uint32_t>(max_len, h.code_len[s]);
        if (!h.tile_rows) all_tiled = false;
        first += h.n_chunks;
    }
    info->total_chunks = first;
    info->lane_syms = hdrs[0].lane_syms;
    info->max_code_len = max_len;
    info->max_workgroups = 0;
    info->row_tiled = all_tiled ? 1u : 0u;
    return ECF8_OK;
}

const char *ecf8_strerror(int code)
{
    switch (code) {
    case ECF8_OK: return "ok";
    case ECF8_E_ARG: return "invalid argument";
    case ECF8_E_FORMAT: return "not a valid ECF8 container";
    case ECF8_E_CAPACITY: return "output buffer too small";
    case ECF8_E_ALIGN: return "device pointer not 16-byte aligned";
    case ECF8_E_HIP: return "HIP runtime error";
    case ECF8_E_NOMEM: return "out of host memory";
    default: return "unknown error";
    }
}

uint32_t ecf8_version(void) { return ECF8_VERSION; }

} // extern "C"
