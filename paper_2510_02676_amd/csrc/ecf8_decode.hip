// ECF8 -> FP8 decode kernels for gfx950 (MI355X), wave64.
//
// What is computed is Algorithm 1 of the paper (block-level decompression:
// load the compressed span, locate each lane's first codeword, decode through
// a lookup table held next to the ALUs, merge the sign/mantissa nibble, write
// back coalesced).  How it is computed is specific to CDNA4:
//
//  * one wavefront decodes one chunk = 64 lanes x N elements; the encoder
//    recorded how many stream bits each lane's N codewords take, so a DPP
//    prefix scan over those 64 numbers gives every lane its start bit, and
//    output positions are fixed by construction (lane l owns the 16-byte
//    pieces l, l+64, ... of the chunk).  The paper's first decoding pass,
//    which exists only to count symbols per thread, is gone;
//  * the chunk's span of the stream is copied to LDS with dwordx4 loads, 1 KiB
//    contiguous per wave instruction; lanes pull aligned 64-bit windows from
//    LDS (unaligned LDS accesses serialise per lane on this chip, so every LDS
//    access here is naturally aligned);
//  * the code table is a 2^TB-entry LDS table of 16-bit entries indexed by the
//    next TB stream bits; one lookup yields TWO symbols, already shifted to
//    their place in the output bytes, and the bits they consume.  A lane
//    always decodes four symbols (two lookups) per step, so every lane of the
//    wave runs the same number of steps, nothing diverges, and each step ends
//    with one finished output dword in a register.  A lane's bits hold two runs,
//    one read forward from its first bit and one read backward from its last
//    bit, so every lane advances two independent dependency chains at once
//    (twice the LDS latency hidden per wave).  Pairs that do not fit in TB bits and
//    codewords longer than TB bits take a second level (per-symbol walk that
//    reuses the table's first-symbol fields, then a 16-entry canonical match);
//    a wave holds 256 pairs per step, so even a 1e-3 miss rate sends a third of
//    the steps there.  Under the encoder's default cap of TB/2 bits per codeword
//    every pair is a table hit and the PAIRFIT kernels carry no second level.
//    The 32 KiB table is copied from the blob when the encoder embedded it (one
//    L2-resident read per workgroup), else built in LDS from the 16 code lengths;
//  * after four steps a lane holds one 16-byte piece; the 64 lanes' pieces are
//    adjacent, so each dwordx4 store instruction of the wave writes 1 KiB of
//    contiguous output, merged in registers with the nibble plane that was
//    fetched (coalesced, 512 B per instruction) a whole chunk earlier.  Decoded
//    bytes never pass through LDS.  The PAIRFIT kernels hold a chunk's pieces
//    and store them in one burst; with the container's group interleave (a
//    wave's consecutive pieces G KiB apart, the workgroup's other waves in
//    between) HBM takes such bursts about 15 % faster than 1 KiB stores
//    trickling out of every wave;
//  * persistent workgroups own contiguous chunk ranges, so a table is set up
//    once per (workgroup, tensor); inside a workgroup the waves draw chunks
//    from an LDS ticket counter (the hardware favours a SIMD's oldest wave, so
//    equal static shares would finish up to 50 % apart).  No global atomics.
#include "ecf8_device.h"

#include <cstddef>
#include <type_traits>

namespace {

// Stream, plane and output are touched exactly once: nontemporal accesses keep them from
// displacing the table and the metadata in L2.
#define LD_STREAM(p) __builtin_nontemporal_load(p)
#define ST_STREAM(v, p) __builtin_nontemporal_store((v), (p))

struct KArgs {
    ecf8_batch_item single;               // used when items == nullptr
    const GLOBAL ecf8_batch_item *items;  // device array for the batched call
    uint32_t n_items;
    uint64_t total_chunks;
    uint32_t max_code_len;                // longest codeword of any tensor of the launch
    uint32_t max_workgroups;              // 0 = one per compute unit
    uint32_t row_tiled;                   // every tensor of the launch is in the row-tiled layout
};

template <int N, int WAVES, bool PAIRFIT, bool TILED = false>
struct Cfg {
    // bytes of stream staged per chunk: under the cap of TB/2 bits per codeword the worst case
    // (so no chunk of a PAIRFIT launch is ever oversize), else a good 4 bits per symbol
    static constexpr int STAGE = PAIRFIT ? 64 * N * (TB / 2) / 8 + 64 : N * 32 + 64;
    static constexpr int PIECES = N / 16;             // 16-byte output pieces per lane
    static constexpr int SEGS = (STAGE / 16 + 63) / 64;  // dwordx4 loads per lane that cover STAGE
    // LDS map (byte offsets into one array)
    static constexpr int OFF_TBL = 0;
    static constexpr int OFF_SYM = OFF_TBL + TBL_ENTRIES * 2;  // s_len[16], s_code[16]
    static constexpr int OFF_CTL = OFF_SYM + 128;              // ticket counter, oversize count, oversize list
    static constexpr int LIST_MAX = 60;                        // oversize chunks remembered per (workgroup, tensor)
    static constexpr int OFF_WAVES = OFF_CTL + 16 + 4 * LIST_MAX;
    // After the pipelined loop the waves' stages together serve as a few wide slots, each large
    // enough for the longest span any code can produce (15 bits per symbol), for the chunks whose
    // span did not fit a stage.
    static constexpr int SLOT = 64 * N * 15 / 8 + 64;
    static constexpr int SLOTS = (WAVES * STAGE / SLOT) < WAVES ? (WAVES * STAGE / SLOT) : WAVES;
    static_assert(PAIRFIT || SLOTS >= 1, "wide slots must fit the stage area");
    static_assert(OFF_WAVES % 16 == 0 && SLOT % 16 == 0, "16-byte LDS stores");
    static constexpr int WAVES_BYTES = WAVES * STAGE > TBL_ENTRIES * 2 ? WAVES * STAGE : TBL_ENTRIES * 2;
    // TILED: a 16 x 256-byte tile per wave in which a decoded chunk of a row-tiled blob is turned from the
    // lanes' pieces (16 bytes of row l % 16 each) into whole 256-byte row segments before it is stored
    static constexpr int OFF_TILE = OFF_WAVES + WAVES_BYTES;  // table-build scratch aliases the stages
    static constexpr int TILE_BYTES = 16 * 4 * N;
    static_assert(!TILED || (PAIRFIT && N == 64), "the tile turn is built for the fused GEMM's layout");
    // the decode steps read one dword past a window's two, so the last stage is followed by a pad
    static constexpr int TOTAL = OFF_TILE + (TILED ? WAVES * TILE_BYTES : 0) + 16;
    static_assert(TOTAL <= 160 * 1024, "LDS of one gfx950 CU");
};

// PAIRFIT: every tensor of the launch has codewords of at most TB/2 bits (the encoder's
// default cap), so the pipelined loop needs no second level and is one straight line.
// LONG (general kernels only): some codeword of the launch is longer than TB bits.  BURST: 1 = a chunk's pieces are
// held in registers and stored together at its end, 2 = half the chunk's pieces at a time, 0 = each piece as it is decoded.
template <int N, int WAVES, bool PAIRFIT, bool TILED = false, bool LONG = !PAIRFIT, int BURST = PAIRFIT>
__global__ __launch_bounds__(WAVES * 64) void ecf8_decode_kernel(KArgs a)
{
    using C = Cfg<N, WAVES, PAIRFIT, TILED>;
    __shared__ __attribute__((aligned(16))) uint8_t smem[C::TOTAL];
    uint16_t *tbl = (uint16_t *)(smem + C::OFF_TBL);
    uint32_t *s_len = (uint32_t *)(smem + C::OFF_SYM);
    uint32_t *s_code = s_len + 16;
    uint32_t *s_ticket = (uint32_t *)(smem + C::OFF_CTL);
    uint32_t *s_oversize = s_ticket + 1;                  // number of oversize chunks met in the loop
    uint32_t *s_list = s_ticket + 4;                      // their chunk numbers, relative to c

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = (int)uniform32((uint32_t)tid >> 6);         // the same for every lane: chunk numbers and addresses stay in scalar registers
    const uint32_t stage_off = C::OFF_WAVES + wave * C::STAGE;   // byte offset into smem
    uint8_t *stage = smem + stage_off;

    // contiguous range of the batch's chunks for this workgroup, cut at multiples of 64 or 8 chunks
    // where that leaves every workgroup at least 16 such units (shares then differ by 1/16 at most),
    // so that the waves of a workgroup share the interleaved groups of the layout
    const uint64_t NWG = gridDim.x, wg = blockIdx.x;
    const uint64_t unit = a.total_chunks >= NWG * 1024 ? 64 : a.total_chunks >= NWG * 128 ? 8 : 1;   // >= 16 units each: shares differ by 1/16 at most
    const uint64_t units = (a.total_chunks + unit - 1) / unit;
    uint64_t c = units * wg / NWG * unit;
    uint64_t c_end = units * (wg + 1) / NWG * unit;
    if (c_end > a.total_chunks) c_end = a.total_chunks;
    while (c < c_end) {
        // which tensor holds chunk c (uniform)
        uint64_t d_blob, d_out, n_elem, n_chunks, first_chunk, off_cb, off_lb, off_st, off_pl, st_bytes;
        uint64_t len_lo, len_hi, off_tbl, group, tcols;
        if (a.items) {
            // 64-way search, a round trip to memory per level instead of one per halving: lane l probes the
            // l-th of 64 evenly spaced items of the remaining range (first_chunk is increasing, so the lanes
            // that pass form a prefix)
            uint32_t lo = 0, n = a.n_items;
            while (n > 1) {
                const uint32_t stride = (n + 63) / 64;
                const uint32_t at = (uint32_t)lane * stride;
                const bool pass = at < n && a.items[lo + at].first_chunk <= c;
                const uint32_t k = (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(pass));
                const uint32_t step = k ? (k - 1) * stride : 0;       // k >= 1 for a valid table: items[lo].first_chunk <= c
                lo += step;
                n = n - step < stride ? n - step : stride;
            }
            // the item's 16 words by one load of 16 lanes, then into scalar registers: the fields are the same
            // for every lane and live as long as the tensor
            const uint64_t word = ((const GLOBAL uint64_t *)(a.items + lo))[lane & 15];
            auto field = [&](int k) -> uint64_t {
                return (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)word, k) |
                       ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(word >> 32), k) << 32);
            };
            static_assert(sizeof(ecf8_batch_item) == 128 && offsetof(ecf8_batch_item, code_len) == 80 &&
                          offsetof(ecf8_batch_item, tile_cols) == 112, "field numbers below");
            d_blob = field(0); d_out = field(1); n_elem = field(2); n_chunks = field(3); first_chunk = field(4);
            off_cb = field(5); off_lb = field(6); off_st = field(7); off_pl = field(8); st_bytes = field(9);
            len_lo = field(10); len_hi = field(11); off_tbl = field(12); group = field(13); tcols = field(14);
        } else {
            d_blob = a.single.d_blob; d_out = a.single.d_out; n_elem = a.single.n_elem;
            n_chunks = a.single.n_chunks; first_chunk = 0; off_cb = a.single.off_chunk_bit;
            off_lb = a.single.off_lane_bits; off_st = a.single.off_stream; off_pl = a.single.off_plane;
            st_bytes = a.single.stream_bytes;
            off_tbl = a.single.off_table; group = a.single.group_chunks; tcols = a.single.tile_cols;
            __builtin_memcpy(&len_lo, a.single.code_len, 8);
            __builtin_memcpy(&len_hi, a.single.code_len + 8, 8);
        }
        const uint64_t t_end = first_chunk + n_chunks;
        const uint64_t seg_end = c_end < t_end ? c_end : t_end;
        if (seg_end <= c) break; // item table does not cover chunk c: stop rather than spin
        GLOBAL uint8_t *out = (GLOBAL uint8_t *)d_out;
        const GLOBAL uint64_t *chunk_bit = (const GLOBAL uint64_t *)(d_blob + off_cb);
        const GLOBAL uint16_t *lane_bits = (const GLOBAL uint16_t *)(d_blob + off_lb);
        const GLOBAL uint8_t *stream = (const GLOBAL uint8_t *)(d_blob + off_st);
        const GLOBAL uint8_t *plane = (const GLOBAL uint8_t *)(d_blob + off_pl);
        // Element layout: chunk cl's piece q of lane l starts at element
        // base + q*stride + l*16.  Chunks of whole groups of `group` chunks are interleaved
        // KiB by KiB (a wave's consecutive pieces lie group KiB apart, the other waves of
        // the workgroup fill the gaps: HBM serves that markedly faster than a wave
        // walking 1 KiB steps); the rest of the tensor is chunk-major.
        // Row-tiled layout (tcols != 0): chunk cl is the block of 16 rows x 4N columns number cl
        // of a tcols-wide matrix, lane l works on row l % 16, its piece q on columns
        // 64 q + 16 (l / 16) of the block.  lane_off is the lane's share of all of this.
        if (group == 0) group = 1;
        const uint64_t grouped = (n_elem / (64ull * N)) & ~(group - 1);   // chunks in whole groups (group is a power of two)
        const uint64_t blocks_per_row = tcols ? tcols / (4ull * N) : 1;
        // Row-tiled: chunk number -> (block of rows, block of columns) is a division by blocks_per_row, which the
        // hardware does not have: a 64-bit one takes more instructions than the decode of a chunk.  Chunk numbers
        // and blocks_per_row fit 32 bits (n_elem <= 2^40, checked by the encoder), so the division is a
        // multiplication by a reciprocal worked out once per tensor (Granlund and Montgomery's round-up method:
        // q = (t + ((n - t) >> sh1)) >> sh2 with t = mulhi(n, mul), exact for every 32-bit n).
        const uint32_t bpr32 = (uint32_t)blocks_per_row;
        uint32_t dv_l = 0;
        while (dv_l < 32 && (1ull << dv_l) < bpr32) dv_l++;
        const uint32_t dv_mul = (uint32_t)((((1ull << dv_l) - bpr32) << 32) / bpr32 + 1);
        const uint32_t dv_sh1 = dv_l < 1 ? dv_l : 1, dv_sh2 = dv_l > 1 ? dv_l - 1 : 0;
        auto chunk_base = [&](uint64_t cl) -> uint64_t {
            if (tcols) {
                const uint32_t t = __umulhi((uint32_t)cl, dv_mul);
                const uint32_t rb = (t + (((uint32_t)cl - t) >> dv_sh1)) >> dv_sh2;
                return (uint64_t)rb * 16 * tcols + ((uint32_t)cl - rb * bpr32) * (4ull * N);
            }
            const uint64_t w = cl & (group - 1);
            return cl < grouped ? (cl - w) * (64ull * N) + w * 1024 : cl * (64ull * N);
        };
        auto chunk_stride = [&](uint64_t cl) -> uint32_t {
            return tcols ? 64u : cl < grouped ? (uint32_t)group * 1024u : 1024u;
        };
        const uint64_t lane_off = tcols ? (uint64_t)(lane & 15) * tcols + (uint64_t)(lane >> 4) * 16 : (uint64_t)lane * 16;

        __syncthreads(); // every wave is done with the previous tensor's table and its scratch
        // the first two chunks of a wave are fixed (c + wave, c + WAVES + wave); later ones are drawn
        if (tid == 0) { *s_ticket = 2 * WAVES; *s_oversize = 0; }

        // Per-wave software pipeline over its chunks cg = c + wave, + WAVES, ...:
        // metadata is loaded two chunks ahead, stream span and nibble plane one chunk
        // ahead (into registers), so HBM latency is covered by the decode of the
        // chunk in hand.
        struct Meta { uint64_t b0, b1; uint32_t lb; };
        auto load_meta = [&](uint64_t cl) {
            Meta m;
            m.b0 = chunk_bit[cl];
            m.b1 = chunk_bit[cl + 1];
            m.lb = lane_bits[cl * 64 + lane];
            return m;
        };
        // span of the stream a chunk needs: 16-byte aligned start, 8 bytes of look-ahead.  The chunk's two
        // start bits are the same in every lane, so the arithmetic is done once, in scalar registers.
        auto span_of = [&](const Meta &m, uint64_t &byte0) {
            const uint64_t b0 = uniform64(m.b0), b1 = uniform64(m.b1);
            uint64_t byte_end = ((b1 + 7) >> 3) + 8;
            if (byte_end > st_bytes) byte_end = st_bytes;
            byte0 = (b0 >> 3) & ~15ull;
            if (byte0 > byte_end) byte0 = byte_end;
            return byte_end - byte0;
        };
        // The span's 16-byte units into `seg` (unit lane + 64 k into seg[k]).  Units beyond the span keep what
        // they held, and so does all of `seg` when the span does not fit a stage: no codeword of a chunk that the
        // loop decodes for good reaches into them.
        const uint32_t lane16 = (uint32_t)lane * 16;
        auto load_stream = [&](const Meta &m, u32x4 (&seg)[C::SEGS]) {
            uint64_t byte0;
            const uint64_t span64 = span_of(m, byte0);
            const uint32_t span = span64 <= (uint64_t)C::STAGE ? (uint32_t)span64 : 0u;
            const GLOBAL uint8_t *sp = stream + byte0;
#pragma unroll
            for (int k = 0; k < C::SEGS; k++) {
                const uint32_t i = lane16 + 1024 * k;
                if (i < span) seg[k] = LD_STREAM((const GLOBAL u32x4 *)(sp + i));
            }
        };
        // nibble plane of chunk cl: this lane's piece j at plane_of(cl) + j * (chunk_stride(cl) / 2)
        auto plane_of = [&](uint64_t cl) -> const GLOBAL uint8_t * { return plane + chunk_base(cl) / 2 + lane_off / 2; };

        // The pipelined loop takes only chunks that are entirely inside the tensor, so its
        // stores are unconditional: between the issue of a prefetch and its use every path
        // holds the same stores, and the wait for the prefetch never drains them.  A chunk
        // whose span does not fit the stage is decoded from stale LDS there (harmless garbage,
        // in bounds) and redone by the generic pass below, as is a ragged last chunk.
        const bool ragged_tail = (n_elem % (64ull * N)) != 0;
        const uint64_t fast_end = (ragged_tail && seg_end == t_end) ? seg_end - 1 : seg_end;
        // next chunk of this workgroup's range, drawn from the LDS ticket counter (wave-uniform)
        auto draw = [&]() -> uint64_t {
            uint32_t t = 0;
            if (lane == 0) t = __hip_atomic_fetch_add(s_ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            return c + uniform32(t);
        };

        // Start-up: the loads of the table, of the first chunks' metadata and of the first chunk's
        // payload are all in flight before the table is written to LDS, so a workgroup pays about
        // two HBM round trips, not four, before its first decode step.
        uint64_t cg = c + wave;
        uint64_t cg1 = cg + WAVES;
        uint64_t cg2 = fast_end;    // drawn when cg1 is taken up
        u32x4 tv[(TBL_ENTRIES * 2 / 16 + WAVES * 64 - 1) / (WAVES * 64)];
        if (off_tbl) {
            // the encoder embedded the table: copy it (L2-resident after the first workgroup)
            const GLOBAL u32x4 *src = (const GLOBAL u32x4 *)(d_blob + off_tbl);
#pragma unroll
            for (int j = 0; j < (int)(sizeof(tv) / sizeof(tv[0])); j++) {
                const int i = tid + j * WAVES * 64;
                tv[j] = u32x4{0, 0, 0, 0};
                if (i < TBL_ENTRIES * 2 / 16) tv[j] = src[i];
            }
        }
        Meta m_cur{0, 0, 0}, m_next{0, 0, 0};
        u32x4 seg[C::SEGS];
        u32x2 pl[C::PIECES];
#pragma unroll
        for (int k = 0; k < C::SEGS; k++) seg[k] = u32x4{0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < C::PIECES; j++) pl[j] = u32x2{0, 0};
        if (cg < fast_end) {
            m_cur = load_meta(cg - first_chunk);
            m_next = m_cur;
            if (cg1 < fast_end) m_next = load_meta(cg1 - first_chunk);
            load_stream(m_cur, seg);
            const GLOBAL uint8_t *pp = plane_of(cg - first_chunk);
            const uint32_t pstride = chunk_stride(cg - first_chunk) / 2;
#pragma unroll
            for (int j = 0; j < C::PIECES; j++) pl[j] = LD_STREAM((const GLOBAL u32x2 *)(pp + j * pstride));
        }
        if (off_tbl) {
#pragma unroll
            for (int j = 0; j < (int)(sizeof(tv) / sizeof(tv[0])); j++) {
                const int i = tid + j * WAVES * 64;
                if (i < TBL_ENTRIES * 2 / 16) ((u32x4 *)tbl)[i] = tv[j];
            }
            build_symbol_arrays(len_lo, len_hi, s_len, s_code, tid);
            __syncthreads();
        } else {
            build_tables(len_lo, len_hi, tbl, s_len, s_code, (uint16_t *)(smem + C::OFF_WAVES), tid, WAVES * 64);
        }

        // Decode of one full chunk whose span sits in LDS from bit `first_bit` (smem-relative) on,
        // merge with the nibble plane, stores.  With `reload` set, each piece of the nibble plane gives its
        // registers, once merged, to the same piece of the chunk whose plane starts at next_pl.
        auto decode_store = [&](auto reload, uint32_t first_bit, uint32_t lb, u32x2 (&pl)[C::PIECES], GLOBAL uint8_t *out_c,
                                uint32_t ostride, const GLOBAL uint8_t *next_pl, uint32_t next_pstride) {
            constexpr bool RELOAD = decltype(reload)::value;
            // LDS bit addresses, kept one bit off as quad_step2 wants them: bpA = the forward
            // run's next codeword - 1; bpB = one past the backward run's next codeword - 31
            uint32_t bpA = first_bit - 1;
            uint32_t bpB = bpA + lb - 30;
            HeldRuns runs;                 // PAIRFIT: the runs' windows stay in registers
            if constexpr (PAIRFIT) runs.begin(smem, bpA, bpB);
            // BURST: the chunk's pieces (or half of them) are kept in registers and stored
            // together.  With the interleaved layout the workgroup's waves then write runs of
            // adjacent KiBs close in time, which HBM takes ~15 % faster than single KiBs
            // trickling out of every wave as they are decoded.  The general kernels have the
            // registers for a full burst at N = 64 and for half bursts at N = 128.
            u32x4 ov[BURST == 1 ? C::PIECES : BURST == 2 ? 4 : 1];
#pragma unroll
            for (int Q = 0; Q < C::PIECES / 2; Q++) {
                uint32_t dwA[4], dwB[4];
#pragma unroll
                for (int t = 0; t < 4; t++) {
                    if constexpr (PAIRFIT) quad_step_held(smem, tbl, runs, dwA[t], dwB[t]);
                    else quad_step2<PAIRFIT, LONG>(smem, tbl, s_len, s_code, bpA, bpB, dwA[t], dwB[t]);
                }
                const u32x4 oA = merge_piece(dwA, pl[Q]);
                const u32x4 oB = merge_piece(dwB, pl[Q + C::PIECES / 2]);
                if constexpr (RELOAD) {
                    pl[Q] = LD_STREAM((const GLOBAL u32x2 *)(next_pl + Q * next_pstride));
                    pl[Q + C::PIECES / 2] = LD_STREAM((const GLOBAL u32x2 *)(next_pl + (Q + C::PIECES / 2) * next_pstride));
                }
                if constexpr (BURST == 1) {
                    ov[Q] = oA;
                    ov[Q + C::PIECES / 2] = oB;
                } else if constexpr (BURST == 2) {
                    // half bursts: the pieces of two steps leave together
                    ov[2 * (Q & 1)] = oA;
                    ov[2 * (Q & 1) + 1] = oB;
                    if (Q & 1) {
                        __builtin_amdgcn_sched_barrier(0);
                        ST_STREAM(ov[0], (GLOBAL u32x4 *)(out_c + (Q - 1) * ostride));
                        ST_STREAM(ov[1], (GLOBAL u32x4 *)(out_c + (Q - 1 + C::PIECES / 2) * ostride));
                        ST_STREAM(ov[2], (GLOBAL u32x4 *)(out_c + Q * ostride));
                        ST_STREAM(ov[3], (GLOBAL u32x4 *)(out_c + (Q + C::PIECES / 2) * ostride));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else {
                    ST_STREAM(oA, (GLOBAL u32x4 *)(out_c + Q * ostride));
                    ST_STREAM(oB, (GLOBAL u32x4 *)(out_c + (Q + C::PIECES / 2) * ostride));
                }
            }
            if constexpr (TILED) {
                // Row-tiled blob: lane (r = l % 16, g = l / 16) holds columns 64 Q + 16 g of row r, so a store of
                // piece Q as it is would cover 16 rows x 64 bytes.  Through the wave's tile the pieces become whole
                // row segments: store j covers rows 4 j .. 4 j + 3 x 256 bytes, lane l row 4 j + l / 16, columns
                // 16 (l % 16).  The 16-byte units of a row are swizzled by the row number against bank conflicts.
                uint8_t *tile = smem + C::OFF_TILE + wave * C::TILE_BYTES;
                const uint32_t r = lane & 15, g = lane >> 4;
#pragma unroll
                for (int Q = 0; Q < C::PIECES; Q++) *(u32x4 *)(tile + r * 256 + (((4 * Q + g) ^ r) & 15) * 16) = ov[Q];
                GLOBAL uint8_t *out_t = out_c - lane_off + (uint64_t)g * tcols + r * 16;       // row l / 16, columns 16 (l % 16)
#pragma unroll
                for (int j = 0; j < 4; j++) ov[j] = *(const u32x4 *)(tile + (4 * j + g) * 256 + ((r ^ (4 * j + g)) & 15) * 16);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < 4; j++) ST_STREAM(ov[j], (GLOBAL u32x4 *)(out_t + (uint64_t)(4 * j) * tcols));
                __builtin_amdgcn_sched_barrier(0);
            } else if constexpr (BURST == 1) {
                __builtin_amdgcn_sched_barrier(0);   // keep the stores together, after the decode
#pragma unroll
                for (int Q = 0; Q < C::PIECES; Q++) ST_STREAM(ov[Q], (GLOBAL u32x4 *)(out_c + Q * ostride));
                __builtin_amdgcn_sched_barrier(0);
            }
        };

        if (cg < fast_end) {
            // Drain the prologue's loads here (vmcnt(0), other counters untouched), so that
            // the wait at the loop head is decided by the back edge alone, where the four
            // stores of the previous chunk are younger than the prefetch and stay in flight.
            __builtin_amdgcn_s_waitcnt(0x0F70);
            for (;;) {
                const uint64_t cl = cg - first_chunk;            // chunk index inside the tensor
                GLOBAL uint8_t *out_c = out + chunk_base(cl) + lane_off;   // this lane's piece 0
                const uint32_t ostride = chunk_stride(cl);
                const uint64_t b0 = uniform64(m_cur.b0);
                uint64_t byte0;
                const uint64_t span64 = span_of(m_cur, byte0);
                const bool staged = __builtin_amdgcn_readfirstlane((uint32_t)(span64 <= (uint64_t)C::STAGE)) != 0;

                // lane start bit = chunk start + exclusive DPP scan of the lanes' bit counts
                const uint32_t rel = wave_incl_scan(m_cur.lb) - m_cur.lb;
                const uint32_t bit_in = (uint32_t)(b0 - byte0 * 8) + rel; // bits from byte0

#pragma unroll
                for (int k = 0; k < C::SEGS; k++) {
                    const uint32_t i = lane16 + 1024 * k;
                    if (i < (uint32_t)C::STAGE && (!PAIRFIT || i < (uint32_t)span64)) *(u32x4 *)(stage + i) = seg[k];
                }

                // prefetch: the next chunk's span of the stream into the registers just written out, the metadata
                // of the chunk after it; the next chunk's nibble plane follows piece by piece inside the decode
                // (after the last chunk: this chunk's plane again, not a branch around the loads)
                const bool has_next = cg1 < fast_end;
                Meta m_next2 = m_next;
                if (has_next) {
                    load_stream(m_next, seg);
                    cg2 = draw();
                    if (cg2 < fast_end) m_next2 = load_meta(cg2 - first_chunk);
                }
                const uint64_t cl_pl = (has_next ? cg1 : cg) - first_chunk;

                if (!staged && lane == 0) {
                    const uint32_t at = __hip_atomic_fetch_add(s_oversize, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    if (at < (uint32_t)C::LIST_MAX) s_list[at] = (uint32_t)(cg - c);
                }
                // a chunk whose span was not staged decodes stale bits (redone after the loop): its runs are
                // pinned to the start of the wave's stage, so that every window stays inside this kernel's LDS
                decode_store(std::true_type{}, stage_off * 8 + (staged ? bit_in : 64u), staged ? m_cur.lb : 0u, pl, out_c, ostride,
                             plane_of(cl_pl), chunk_stride(cl_pl) / 2);

                if (!has_next) break;
                m_cur = m_next;
                m_next = m_next2;
                cg = cg1;
                cg1 = cg2;
            }
        }
        __syncthreads();

        // Chunks whose span did not fit a stage (they code far worse than 4 bits per symbol; the
        // loop decoded garbage for them, in bounds): the stage area now serves as SLOTS wide slots.
        // Round by round the workgroup copies up to SLOTS such spans in, and one wave per slot
        // decodes with the loop's own steps.  PAIRFIT launches never get here with a valid blob.
        const uint32_t n_over = *s_oversize;
        bool scan_all = fast_end != seg_end;          // the ragged last chunk always takes the symbol pass
        if (n_over != 0) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // the loop's stores land first
            if (PAIRFIT || n_over > (uint32_t)C::LIST_MAX) {
                scan_all = true;                      // too many to remember: symbol pass over everything
            } else {
                for (uint32_t r0 = 0; r0 < n_over; r0 += C::SLOTS) {
                    __syncthreads();                  // slots free (first round: every wave is out of the loop)
                    for (uint32_t k = 0; k < (uint32_t)C::SLOTS && r0 + k < n_over; k++) {
                        const uint64_t cl = c + s_list[r0 + k] - first_chunk;
                        const uint64_t sb0 = chunk_bit[cl], sb1 = chunk_bit[cl + 1];
                        uint64_t byte_end = ((sb1 + 7) >> 3) + 8;
                        if (byte_end > st_bytes) byte_end = st_bytes;
                        uint64_t byte0 = (sb0 >> 3) & ~15ull;
                        if (byte0 > byte_end) byte0 = byte_end;
                        const uint64_t span = byte_end - byte0;
                        uint8_t *slot = smem + C::OFF_WAVES + k * C::SLOT;
                        for (uint32_t i = tid * 16; i < (uint32_t)C::SLOT && i < span; i += WAVES * 64 * 16)
                            *(u32x4 *)(slot + i) = *(const GLOBAL u32x4 *)(stream + byte0 + i);
                    }
                    __syncthreads();
                    if ((uint32_t)wave < (uint32_t)C::SLOTS && r0 + wave < n_over) {
                        const uint64_t cl = c + s_list[r0 + wave] - first_chunk;
                        const Meta m = load_meta(cl);
                        uint64_t byte0;
                        const uint64_t span = span_of(m, byte0);
                        if (span <= (uint64_t)C::SLOT) {          // else: a corrupt blob, left as decoded in the loop
                            u32x2 pl_s[C::PIECES];
                            const GLOBAL uint8_t *plane_c = plane_of(cl);
                            const uint32_t pstride = chunk_stride(cl) / 2;
#pragma unroll
                            for (int j = 0; j < C::PIECES; j++) pl_s[j] = *(const GLOBAL u32x2 *)(plane_c + j * pstride);
                            const uint32_t rel = wave_incl_scan(m.lb) - m.lb;
                            const uint64_t b0 = uniform64(m.b0);
                            decode_store(std::false_type{}, (C::OFF_WAVES + wave * C::SLOT) * 8 + (uint32_t)(b0 - byte0 * 8) + rel, m.lb, pl_s,
                                         out + chunk_base(cl) + lane_off, chunk_stride(cl), plane_c, 0u);
                        }
                    }
                }
            }
        }
        // Symbol pass, with windows and nibbles read straight from HBM: the ragged last chunk of
        // the tensor (and everything oversize when the list above did not apply).
        if (scan_all) {
            // The chunks redone here were stored (as garbage) by whichever wave drew them in the loop, not
            // necessarily by the wave that redoes them: every wave's loop stores are complete (fence)
            // before any wave issues a store of this pass (barrier; scan_all is uniform).
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            __syncthreads();
            for (uint64_t cg2 = c + wave; cg2 < seg_end; cg2 += WAVES) {
                const uint64_t cl = cg2 - first_chunk;
                Meta m = load_meta(cl);
                uint64_t byte0;
                const uint64_t span64 = span_of(m, byte0);
                const bool redo = cg2 >= fast_end || (span64 > (uint64_t)C::STAGE && (PAIRFIT || n_over > (uint32_t)C::LIST_MAX));
                if (!__builtin_amdgcn_readfirstlane((uint32_t)redo)) continue;
                const uint64_t elem0 = chunk_base(cl);
                const uint32_t estride = chunk_stride(cl);
                const uint32_t rel = wave_incl_scan(m.lb) - m.lb;
                const GLOBAL uint8_t *sp = stream + byte0;
                uint64_t bA = (m.b0 - byte0 * 8) + rel;   // forward run: next bit
                uint64_t bB = bA + m.lb;                  // backward run: one past the next bit
#pragma unroll 1
                for (int Q = 0; Q < C::PIECES; Q++) {
                    const uint64_t o = elem0 + (uint64_t)Q * estride + lane_off;
                    const bool fwd = Q < C::PIECES / 2;
#pragma unroll 1
                    for (uint32_t i = 0; i < 16 && o + i < n_elem; i++) {
                        const uint32_t w = fwd ? global_window<+1>(sp, bA) : global_window<-1>(sp, bB);
                        const uint32_t r = decode_one<LONG>(w, tbl, s_len, s_code);
                        if (fwd) bA += r >> 8; else bB -= r >> 8;
                        const uint64_t el = o + i;
                        const uint32_t pb = plane[(el >> 3) * 4 + (el & 3)];
                        const uint32_t nib = (el & 4) ? pb >> 4 : pb & 15u;
                        out[el] = (uint8_t)(((r & 15u) << 3) | ((nib & 8u) << 4) | (nib & 7u));
                    }
                }
            }
        }
        c = seg_end;
    }
}

template <int N, int WAVES, bool PAIRFIT, bool TILED = false, bool LONG = !PAIRFIT, int BURST = PAIRFIT>
int launch_as(const KArgs &a, int wgs_per_cu, hipStream_t s)
{
    int cus = device_cus();
    if (cus <= 0) return ECF8_E_HIP;
    uint64_t want = (a.total_chunks + WAVES - 1) / WAVES;       // at least one chunk per wave
    uint64_t cap = (uint64_t)cus * wgs_per_cu;
    if (a.max_workgroups && a.max_workgroups < cap) cap = a.max_workgroups;
    uint32_t grid = (uint32_t)(want < cap ? want : cap);
    if (grid == 0) grid = 1;
    hipLaunchKernelGGL((ecf8_decode_kernel<N, WAVES, PAIRFIT, TILED, LONG, BURST>), dim3(grid), dim3(WAVES * 64), 0, s, a);
    return hipGetLastError() == hipSuccess ? ECF8_OK : ECF8_E_HIP;
}

// Workgroup shapes.  PAIRFIT kernels: N = 128 runs 8 waves of ~200 VGPRs, which is what holding a chunk's 8
// output pieces for the store burst takes; it has compute to spare (6 waves measured the same, 4 a sixth slower);
// N = 64 runs 12 waves (2 % faster than 16).  General kernels: 12 waves, the most that
// leaves registers for a burst (N = 64: the whole chunk; N = 128: half a chunk at a time); N = 32 runs 16 waves
// and stores piece by piece, which measured faster there.
int dispatch(const KArgs &a, uint32_t lane_syms, hipStream_t s)
{
    if (a.max_code_len == 0 || a.max_code_len > 15) return ECF8_E_ARG;
    const bool pairfit = 2 * a.max_code_len <= (uint32_t)TB;
    const bool lng = a.max_code_len > (uint32_t)TB;      // a codeword the table cannot hold: the kernels with the out-of-line matcher
    switch (lane_syms) {
    case 32:
        if (pairfit) return launch_as<32, 16, true>(a, 1, s);
        return lng ? launch_as<32, 16, false, false, true, 0>(a, 1, s) : launch_as<32, 16, false, false, false, 0>(a, 1, s);
    case 64:
        // the fused GEMM's blobs (row-tiled, capped codes): decoded chunks leave as whole row segments
        if (pairfit && a.row_tiled) return launch_as<64, 16, true, true>(a, 1, s);
        if (pairfit) return launch_as<64, 12, true>(a, 1, s);
        return lng ? launch_as<64, 12, false, false, true, 1>(a, 1, s) : launch_as<64, 12, false, false, false, 1>(a, 1, s);
    case 128:
        if (pairfit) return launch_as<128, 8, true>(a, 1, s);
        return lng ? launch_as<128, 12, false, false, true, 2>(a, 1, s) : launch_as<128, 12, false, false, false, 2>(a, 1, s);
    default: return ECF8_E_ARG;
    }
}

} // namespace

extern "C" {

int ecf8_decode(const ecf8_header *h, const void *d_blob, void *d_out, uint64_t out_capacity, void *stream)
{
    if (!h || !d_blob || !d_out) return ECF8_E_ARG;
    if (h->magic != ECF8_MAGIC || h->version != ECF8_VERSION || h->n_elem == 0 || h->n_chunks == 0 ||
        (h->table_bits != 0 && h->table_bits != ECF8_TB) || h->group_chunks == 0 || h->group_chunks > 64 ||
        (h->group_chunks & (h->group_chunks - 1)))
        return ECF8_E_FORMAT;
    if (h->tile_rows != 0 && (h->tile_rows != 16 || h->group_chunks != 1 || h->rows % 16 != 0 || h->cols == 0 ||
                              h->cols % (4ull * h->lane_syms) != 0 || h->rows > (1ull << 40) / h->cols || h->n_elem != h->rows * h->cols))
        return ECF8_E_FORMAT;
    if (h->n_chunks != (h->n_elem + 64ull * h->lane_syms - 1) / (64ull * h->lane_syms)) return ECF8_E_FORMAT;
    if (h->off_plane + h->plane_bytes > h->total_size || h->off_stream + h->stream_bytes > h->off_plane ||
        h->plane_bytes != h->n_chunks * 32ull * h->lane_syms)
        return ECF8_E_FORMAT;
    if (out_capacity < h->n_elem) return ECF8_E_CAPACITY;
    if (((uintptr_t)d_blob | (uintptr_t)d_out) & 15) return ECF8_E_ALIGN;
    KArgs a{};
    a.single.d_blob = (uint64_t)(uintptr_t)d_blob;
    a.single.d_out = (uint64_t)(uintptr_t)d_out;
    a.single.n_elem = h->n_elem;
    a.single.n_chunks = h->n_chunks;
    a.single.first_chunk = 0;
    a.single.off_chunk_bit = h->off_chunk_bit;
    a.single.off_lane_bits = h->off_lane_bits;
    a.single.off_stream = h->off_stream;
    a.single.off_plane = h->off_plane;
    a.single.stream_bytes = h->stream_bytes;
    a.single.off_table = h->table_bits ? 256 : 0;
    a.single.group_chunks = h->group_chunks;
    a.single.tile_cols = h->tile_rows ? h->cols : 0;
    for (int i = 0; i < 16; i++) a.single.code_len[i] = h->code_len[i];
    a.items = nullptr;
    a.n_items = 1;
    a.total_chunks = h->n_chunks;
    a.row_tiled = h->tile_rows != 0;
    for (int i = 0; i < 16; i++) a.max_code_len = h->code_len[i] > a.max_code_len ? h->code_len[i] : a.max_code_len;
    return dispatch(a, h->lane_syms, (hipStream_t)stream);
}

int ecf8_decode_batched(const ecf8_batch_item *d_items, uint32_t n_tensors, const ecf8_batch_info *info,
                        void *stream)
{
    if (!d_items || !info || n_tensors == 0 || info->total_chunks == 0) return ECF8_E_ARG;
    if ((uintptr_t)d_items & 15) return ECF8_E_ALIGN;
    KArgs a{};
    a.items = (const GLOBAL ecf8_batch_item *)(uintptr_t)d_items;
    a.n_items = n_tensors;
    a.total_chunks = info->total_chunks;
    a.max_code_len = info->max_code_len;
    a.max_workgroups = info->max_workgroups;
    a.row_tiled = info->row_tiled;
    return dispatch(a, info->lane_syms, (hipStream_t)stream);
}

} // extern "C"
