/*
 * ecfw.h -- C ABI of the wide-alphabet sibling of ECF8 (see ecf8.h).
 *
 * The paper's scheme (Section 3.1: histogram of the exponent field, prefix code
 * under a length cap, one stream of codewords, raw remaining bits; Section 3.2:
 * table-driven parallel decoding) carried over to formats whose exponent field is
 * wider than E4M3's four bits -- the direction Section 1 leaves open:
 *   ECFW_FMT_E5M2  1 byte  / element: sign(1) exponent(5) mantissa(2),  32 symbols
 *   ECFW_FMT_BF16  2 bytes / element: sign(1) exponent(8) mantissa(7), 256 symbols
 * (BF16 elements are little-endian 16-bit words.)  With these alphabets plain
 * Huffman codes grow past the 16 bits Section 3.1 allows a codeword, so the code
 * is the cheapest one under a cap (package-merge); with the default cap of 12,
 * the index width of the decoder's lookup table, every codeword resolves in one
 * lookup (measured cost on synthetic weights: 0.004 bits per element).
 *
 * E5M2, second way of storing it (declared here, implemented by ecf8.h): the FP8
 * container of ecf8.h never interprets its bytes -- it codes bits 6..3 of a byte and
 * keeps bits 7, 2, 1, 0 raw -- so an E5M2 tensor given to ecf8_encode /
 * ecf8_encode_gpu is stored with the UPPER FOUR of its five exponent bits as the
 * coded symbol and the sign, the lowest exponent bit and the mantissa in the raw
 * nibble; ecf8_decode / ecf8_decode_batched return the exact bytes.  One exponent
 * bit goes uncoded (0.750 of the raw size against 0.726 for ECFW_FMT_E5M2 on the
 * synthetic weights), and the decoder is the pair-table one of ecf8.h, two symbols
 * per lookup, which this chip runs about 1.4 x faster than the one-symbol-per-lookup
 * decoder a 32-symbol alphabet needs.  Use ECFW_FMT_E5M2 for the smaller blob, the
 * FP8 container for the faster decode.
 *
 * Boundary rules are those of ecf8.h: plain pointers and sizes, "host" = CPU
 * memory, "device" = HIP memory of the current device owned by the caller, no
 * allocation or synchronisation of the device by the library, return value
 * ECF8_OK or a negative ECF8_E_* code.  Blobs are ecf8_blob objects: query and
 * free them with ecf8_blob_data / ecf8_blob_size / ecf8_blob_free.
 *
 * Container "ECFW", integers little-endian, every section at a multiple of 256
 * bytes from the start, in this order:
 *   header (256 B): struct ecfw_header
 *   code_len  : u8[n_alphabet]   length of the codeword of exponent field x, 0 = absent
 *   freq      : u64[n_alphabet]  histogram of the exponent field
 *   chunk_bit : u64[n_chunks+1]  stream bit at which chunk c starts; last = stream_bits
 *   lane_bits : u16[n_chunks*64] code bits of lane l of chunk c
 *   stream    : stream bit i is bit (i & 7) of byte (i >> 3); the lanes' bits follow
 *               each other chunk by chunk, lane by lane.  A piece is P = 16 / (bytes
 *               per element) consecutive elements, i.e. 16 bytes of output; the k-th
 *               symbol (k = 0..N-1, N = lane_syms) of lane l of chunk c is element
 *                   base(c) + (k/P)*stride(c) + l*P + k%P
 *               where, with E = 64N elements per chunk, G = group_chunks and
 *               F = n_elem / (G*E) whole groups,
 *                 c <  G*F: base = (c - c%G)*E + (c%G)*64P, stride = G*64P
 *                 c >= G*F: base = c*E,                     stride = 64P
 *               (the KiB-wise interleave of ecf8.h); elements >= n_elem do not exist
 *               and are skipped.  Symbols k < N/2 are written forward from the lane's
 *               first bit (a codeword's first = most significant bit lowest), symbols
 *               k >= N/2 backward from the lane's last bit (first bit highest), k = N/2
 *               at the top; the two runs meet exactly.  Codewords are the canonical
 *               code of code_len[] ordered by (length, symbol).  Zero padded to
 *               stream_bytes = roundup16(ceil(stream_bits/8) + 8)
 *   plane     : BF16: one byte sign<<7 | mantissa per element, element i in byte
 *               (i/4)*4 + {0,2,1,3}[i%4]  (so that a 32-bit word of the plane holds
 *               the bytes of two output words in their final lanes);
 *               plane_bytes = n_chunks*64N.
 *               E5M2: one u32 per piece g = i/16 with the mantissas: element
 *               i = 16g + 4d + j (d, j in 0..3) in bits 8j+2d and 8j+2d+1 (a shift by
 *               2d leaves the mantissas of output word d in the low bits of its four
 *               bytes); plane_bytes = n_chunks*16N
 *   sign      : E5M2 only: one u16 per piece, bit i%16 = sign of element i;
 *               sign_bytes = n_chunks*8N.  Both planes are zero padded.
 */
#ifndef ECFW_H
#define ECFW_H

#include <stdint.h>

#include "ecf8.h"

#ifdef __cplusplus
extern "C" {
#endif

#define ECFW_MAGIC 0x57464345u /* "ECFW" */
#define ECFW_VERSION 1u
#define ECFW_FMT_E5M2 1u
#define ECFW_FMT_BF16 2u
#define ECFW_TABLE_BITS 12u    /* index width of the decoder's lookup table         */
#define ECFW_MAX_CODE_LEN 16u  /* Section 3.1's cap on the length of a codeword     */

typedef struct ecfw_header {
    uint32_t magic;          /* ECFW_MAGIC                                          */
    uint32_t version;        /* ECFW_VERSION                                        */
    uint64_t total_size;     /* bytes of the whole blob                             */
    uint64_t n_elem;         /* rows * cols                                         */
    uint64_t rows, cols;
    uint32_t fmt;            /* ECFW_FMT_*                                          */
    uint32_t lane_syms;      /* N: symbols per lane, 64 or 128                      */
    uint32_t group_chunks;   /* G: chunks interleaved per group, power of two <= 64 */
    uint32_t max_code_len;   /* longest codeword in use (<= 16)                     */
    uint32_t n_alphabet;     /* 32 (E5M2) or 256 (BF16)                             */
    uint32_t n_symbols;      /* distinct exponent fields present                    */
    uint64_t n_chunks;       /* ceil(n_elem / (64 N))                               */
    uint64_t stream_bits;    /* sum over elements of their code length              */
    uint64_t off_code_len, off_freq, off_chunk_bit, off_lane_bits, off_stream, off_plane;
    uint64_t off_sign;       /* 0 for BF16                                          */
    uint64_t stream_bytes, plane_bytes, sign_bytes;
    uint8_t reserved[96];    /* zero                                                */
} ecfw_header;

typedef struct ecfw_encode_opts {
    uint32_t fmt;          /* ECFW_FMT_E5M2 or ECFW_FMT_BF16 (required)              */
    uint32_t lane_syms;    /* 0 = default: 128 for E5M2, 64 for BF16 (8 KiB of output */
    /*                        per chunk either way)                                  */
    uint32_t n_threads;    /* host threads, 0 = all hardware threads                 */
    uint32_t group_chunks; /* 0 = default (32)                                       */
    uint32_t max_code_len; /* cap on the code length, up to 16; 0 = default (12 =    */
    /*                        ECFW_TABLE_BITS: the decoder's branch-free form).  A   */
    /*                        cap too small for the number of distinct exponent      */
    /*                        fields (2^cap < their count) is ECF8_E_ARG             */
    uint32_t reserved[3];
} ecfw_encode_opts;

/*
 * ecfw_encode (Section 3.1, all stages, for the formats above).  HOST ONLY.
 * Reads rows*cols elements (row-major; every bit pattern is legal: fields are
 * opaque to the codec, so zeros, subnormals, infinities and NaN payloads round-
 * trip) and returns a new blob in *out.  rows*cols == 0 -> ECF8_E_ARG.
 */
int ecfw_encode(const void *elems_host, uint64_t rows, uint64_t cols, const ecfw_encode_opts *opts,
                ecf8_blob **out);

/*
 * ecfw_encode_gpu (Section 3.1 on the device for the formats above).  d_elems: DEVICE,
 * rows*cols elements, 16-byte aligned; d_blob: DEVICE buffer of blob_capacity bytes,
 * 256-byte aligned, that receives the container -- byte for byte the one ecfw_encode
 * writes for the same input and options (n_threads is ignored).  ecfw_encode_bound
 * gives a capacity that always suffices; ECF8_E_CAPACITY if the blob turns out larger
 * than blob_capacity.  *hdr_out receives the header.  The call synchronises `stream`
 * ONCE (it reads the histogram back to build the code on the host), then queues the
 * rest asynchronously.  Uses no memory besides its input and output.
 */
int ecfw_encode_bound(uint64_t rows, uint64_t cols, const ecfw_encode_opts *opts, uint64_t *bytes);
int ecfw_encode_gpu(const void *d_elems, uint64_t rows, uint64_t cols, const ecfw_encode_opts *opts,
                    void *d_blob, uint64_t blob_capacity, ecfw_header *hdr_out, void *stream);

/*
 * Header parse + structural checks of a container held in HOST memory (sizes,
 * offsets, alignment, code lengths form a prefix code that covers the histogram).
 * Fills *hdr, which is what ecfw_decode needs on the host at launch time.
 */
int ecfw_blob_describe(const void *blob_host, uint64_t size, ecfw_header *hdr);

/*
 * Full metadata check of a HOST container before it is trusted on the device:
 * describe() plus chunk_bit consistent with lane_bits, lane_bits within what N
 * codewords can take, histogram consistent with stream_bits, zero padding.  The
 * decode call does not read device memory from the host: validate before upload.
 */
int ecfw_blob_validate(const void *blob_host, uint64_t size);

/*
 * ecfw_decode (Section 3.2 / Algorithm 1 for the formats above, restructured as in
 * ecf8_decode: one wavefront per chunk, stream staged in LDS, two independent runs
 * per lane, one 12-bit lookup per codeword, 16-byte stores).
 * d_blob: DEVICE copy of the whole blob, 256-byte aligned.  hdr: HOST header of
 * that blob (from ecfw_blob_describe).  d_out: DEVICE buffer of out_capacity
 * bytes >= n_elem * bytes per element, 16-byte aligned; receives the exact
 * original elements.  Asynchronous on `stream`; no device memory besides the
 * arguments is touched.  max_workgroups: 0 = one per compute unit.
 */
int ecfw_decode(const void *d_blob, const ecfw_header *hdr, void *d_out, uint64_t out_capacity,
                uint32_t max_workgroups, void *stream);

/*
 * Batched decode: many tensors of one format and one lane_syms in ONE launch, so
 * that the per-launch costs (code set-up per workgroup, first loads, tail) are paid
 * once per batch; a workgroup's contiguous range of chunks may cross tensors, and
 * the code is set up again at each crossing.
 * ecfw_batch_prepare: HOST.  Checks each header and buffer as ecfw_decode does and
 * fills items_host[n] (the caller copies them to the device, 8-byte aligned) and
 * *info (the caller may then set info->max_workgroups, 0 = one per compute unit).
 * ecfw_decode_batched: asynchronous on `stream`; d_items is the DEVICE copy.
 */
typedef struct ecfw_batch_item {
    uint64_t d_blob, d_out;      /* device addresses                                   */
    uint64_t n_elem, n_chunks;
    uint64_t first_chunk;        /* running sum of n_chunks over the earlier items     */
    uint64_t stream_bytes;
    uint64_t off_code_len, off_chunk_bit, off_lane_bits, off_stream, off_plane, off_sign;
    uint64_t group_chunks;
    uint64_t reserved[3];
} ecfw_batch_item;

typedef struct ecfw_batch_info {
    uint64_t total_chunks;
    uint32_t fmt, lane_syms;
    uint32_t max_code_len;       /* longest codeword of any tensor of the batch        */
    uint32_t max_workgroups;
    uint64_t reserved;
} ecfw_batch_info;

int ecfw_batch_prepare(const ecfw_header *hdrs, const void *const *d_blobs, void *const *d_outs,
                       const uint64_t *out_capacities, uint32_t n, ecfw_batch_item *items_host,
                       ecfw_batch_info *info);
int ecfw_decode_batched(const void *d_items, uint32_t n, const ecfw_batch_info *info, void *stream);

/*
 * Just-in-time decode of layers held in this container: the two set-up steps of an
 * ecf8_jit manager (see ecf8.h) for a layer of E5M2 / BF16 tensors.  A manager may hold
 * layers of both kinds; ecf8_jit_prefetch / _acquire / _release do not care.  offsets[i]
 * receives the byte offset of tensor i inside the layer's buffer (256-byte aligned);
 * items_host[n] is what the caller copies to the device and hands to the commit call.
 */
int ecfw_jit_layer_prepare(ecf8_jit *jit, uint32_t layer, const ecfw_header *hdrs, const void *const *d_blobs,
                           uint32_t n_tensors, ecfw_batch_item *items_host, uint64_t *offsets);
int ecfw_jit_layer_commit(ecf8_jit *jit, uint32_t layer, const ecfw_batch_item *d_items);

#ifdef __cplusplus
}
#endif

#endif
