/*
 * ecf8.h -- C ABI of the MI355X-native ECF8 library.
 *
 * ECF8 (paper Section 3) stores FP8 E4M3 weights losslessly as
 *   - a prefix-coded stream of the 4-bit exponent fields (optimal Huffman code
 *     over the tensor's own exponent histogram, Section 3.1 "Huffman code
 *     generation"),
 *   - the raw sign+mantissa nibbles (Table 4, "packed"),
 *   - synchronisation metadata that lets independent GPU lanes start decoding
 *     in the middle of the stream (Section 3.1 "Encoding and synchronization
 *     metadata generation"),
 * and reconstructs the exact bytes on the GPU just before use (Section 3.2,
 * Algorithm 1; Section 3.3).
 *
 * Boundary: plain pointers and sizes only.  "host" pointers are ordinary CPU
 * memory; "device" pointers are HIP device memory of the current device that
 * the CALLER owns (e.g. a PyTorch tensor's data_ptr()).  The library keeps no
 * device memory of its own and never allocates or frees device memory; the
 * decode calls never synchronise the device and use no global atomics (the
 * device encoder reads its histogram back once and uses atomics on its own
 * output; the split-K GEMM calls use them on the counters in their workspace).  `stream` arguments are
 * a hipStream_t passed as void* (NULL = the default stream).
 *
 * All functions return ECF8_OK (0) or a negative ECF8_E_* code; nothing throws
 * or aborts across this boundary.
 *
 * Container ("blob"), all integers little-endian, every section at a multiple
 * of 256 bytes from the start of the blob, in this order:
 *   header (256 B): see struct ecf8_header
 *   table     : optional, u16[2^table_bits] (table_bits = 14), directly after
 *               the header: the decoder's pair lookup table, stored with the
 *               tensor like the paper's LUT array (Table 4) so that a workgroup
 *               loads it instead of building it.  Entry i describes the
 *               codewords spelled by the bits of i, bit 0 first: with (s1, l1)
 *               the first codeword's symbol and length and (s2, l2) the next
 *               one's,  bits 3..6 = s1, bits 0..2 and 15 = l1 (low three bits,
 *               high bit), and, when l1 + l2 <= table_bits, bits 11..14 = s2
 *               and bits 7..10 = l1 + l2, else those bits are 0; an entry
 *               whose first codeword needs more than table_bits bits is 0
 *   chunk_bit : u64[n_chunks+1]  stream bit at which chunk c's first codeword
 *                                starts; last entry = stream_bits
 *   lane_bits : u16[n_chunks*64] code bits of lane l of chunk c (N = lane_syms
 *                                symbols, fewer in the ragged last chunk);
 *                                0 for empty lanes
 *   stream    : the lanes' bits concatenated chunk by chunk, lane by lane;
 *               stream bit i is bit (i & 7) of byte (i >> 3).  Lane l of chunk
 *               c owns bits [S, S + lane_bits), S = chunk_bit[c] + lane_bits of
 *               the chunk's earlier lanes, and codes N/16 16-element pieces:
 *               its k-th symbol is element
 *                   base(c) + (k/16)*stride(c) + l*16 + k%16
 *               (elements >= n_elem do not exist and are skipped).  With
 *               E = 64N elements per chunk, G = group_chunks and F = the
 *               number of whole groups, n_elem / (G*E):
 *                 c <  G*F (grouped): base = (c - c%G)*E + (c%G)*1024,
 *                                     stride = G*1024
 *                 c >= G*F (tail)   : base = c*E, stride = 1024
 *               so G = 1 makes every chunk a contiguous run of E elements, and
 *               G > 1 interleaves the G chunks of a group KiB by KiB: the
 *               pieces a wavefront touches back to back lie G KiB apart and
 *               the wavefronts of a workgroup fill the gaps (see group_chunks).
 *               Row-tiled layout (tile_rows = 16): with KC = cols / 4N chunks
 *               per block of 16 rows, chunk c = b*KC + kc holds rows
 *               16b .. 16b+15, columns 4N*kc .. 4N*(kc+1); the k-th symbol of
 *               lane l is the matrix element
 *                   row 16b + l%16,  column 4N*kc + 64*(k/16) + 16*(l/16) + k%16
 *               i.e. element index row*cols + column: in every decode step lane
 *               l holds 8 consecutive K-elements of row l%16, which is a lane's
 *               share of the B operand of v_mfma_f32_16x16x32_fp8_fp8.
 *               Symbols k < N/2 are written forward
 *               from bit S upwards (a codeword's first = most significant bit
 *               lowest), symbols k >= N/2 backward from bit S + lane_bits - 1
 *               downwards (first bit highest); the two runs meet exactly.
 *               Codes are the canonical code of code_len[] ordered by
 *               (length, symbol); zero padded to
 *               stream_bytes = roundup16(ceil(bits/8) + 8)
 *   plane     : nibbles q = sign<<3 | mantissa; element i lives in byte
 *               (i/8)*4 + (i%4), low nibble if (i%8) < 4 else high nibble;
 *               zero padded to n_chunks*32N bytes
 * A chunk is 64 lanes of N symbols: one wavefront decodes one chunk; in every
 * decode step the 64 lanes produce 64 adjacent 16-byte pieces of the output.
 */
#ifndef ECF8_H
#define ECF8_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ECF8_OK 0
#define ECF8_E_ARG (-1)      /* null pointer, zero size, unsupported option      */
#define ECF8_E_FORMAT (-2)   /* blob is not a valid container                    */
#define ECF8_E_CAPACITY (-3) /* an output buffer is too small                    */
#define ECF8_E_ALIGN (-4)    /* a device pointer is not 16-byte aligned          */
#define ECF8_E_HIP (-5)      /* the HIP runtime reported an error at launch      */
#define ECF8_E_NOMEM (-6)    /* host allocation failed                           */

#define ECF8_MAGIC 0x38464345u /* "ECF8" */
#define ECF8_VERSION 1u
#define ECF8_LANES 64u         /* lanes per chunk = wavefront width              */

/* The first 256 bytes of every blob. */
typedef struct ecf8_header {
    uint32_t magic;           /* ECF8_MAGIC                                      */
    uint32_t version;         /* ECF8_VERSION                                    */
    uint64_t total_size;      /* bytes of the whole blob                         */
    uint64_t n_elem;          /* rows * cols                                     */
    uint64_t rows, cols;
    uint32_t lane_syms;       /* N: symbols per lane, one of 32, 64, 128         */
    uint16_t table_bits;      /* 0: no embedded table; 14: table section present */
    uint8_t group_chunks;     /* G: chunks interleaved per group, a power of two */
                              /* <= 64.  HBM serves a wavefront's consecutive     */
                              /* 1 KiB accesses faster when they are >= 16 KiB    */
                              /* apart (measured: +15 % at G = 32 against G = 1)  */
    uint8_t tile_rows;        /* 0: linear layout (above); 16: row-tiled layout,  */
                              /* a chunk is a 16-row x 4N-column block of the     */
                              /* matrix, laid out as the FP8 matrix cores read    */
                              /* their B operand (see below); needs G == 1,       */
                              /* rows % 16 == 0, cols % 4N == 0                   */
    uint64_t n_chunks;        /* ceil(n_elem / (64 N))                           */
    uint64_t stream_bits;     /* sum over elements of their code length          */
    uint8_t code_len[16];     /* code length of exponent field x, 0 = absent     */
    uint64_t off_chunk_bit, off_lane_bits, off_stream, off_plane;
    uint64_t stream_bytes, plane_bytes;
    uint64_t freq[16];        /* exponent histogram p(x) * n_elem                */
} ecf8_header;

typedef struct ecf8_encode_opts {
    uint32_t lane_syms;  /* 0 = default (128; 64 when max_code_len is above 7);  */
                         /* 64 is what ecf8_gemm_fp8 needs                       */
    uint32_t n_threads;  /* host threads for encoding, 0 = all hardware threads  */
    uint32_t table_mode; /* 0 = embed the table when n_elem >= 2^22 (32 KiB is   */
                         /* then < 0.8 % of the tensor), 1 = always, 2 = never   */
    uint32_t group_chunks; /* 0 = default (32, or 1 in the row-tiled layout)       */
    uint32_t max_code_len; /* cap on the code length, 4..15; 0 = default (7 = half */
                           /* the decoder's table index, so that two codewords     */
                           /* always resolve in one lookup and the decode kernels  */
                           /* take their branch-free form).  Section 3.1 caps the  */
                           /* length too (at 16, by adjusting frequencies); here   */
                           /* the capped code is the cheapest one (package-merge). */
                           /* 15 never binds: plain Huffman                        */
    uint32_t tile_rows;    /* 0 = linear layout; 16 = row-tiled layout (what       */
                           /* ecf8_gemm_fp8 needs; group_chunks must be 0 or 1)    */
    uint32_t reserved[2];
} ecf8_encode_opts;

typedef struct ecf8_stats {
    double entropy_bits;    /* H of the exponent histogram                       */
    double avg_code_bits;   /* stream_bits / n_elem                              */
    double bits_per_weight; /* 8 * total_size / n_elem, metadata included        */
    double ratio;           /* total_size / n_elem                               */
    uint32_t max_code_len;
    uint32_t n_symbols;     /* distinct exponent fields present                  */
} ecf8_stats;

typedef struct ecf8_blob ecf8_blob; /* host object owning one encoded container   */

/*
 * ecf8_encode (Section 3.1, all three stages).  HOST ONLY.
 * Reads rows*cols raw E4M3 bytes (row-major; every byte value is legal: the
 * codec treats bits 6..3 as an opaque symbol, so zeros, subnormals and NaN
 * encodings round-trip), builds the histogram, an optimal prefix code
 * (lengths <= opts->max_code_len), the stream, the lane/chunk metadata and
 * the nibble plane.  *out receives a new blob the caller frees with
 * ecf8_blob_free.  rows*cols == 0 -> ECF8_E_ARG.
 */
int ecf8_encode(const uint8_t *fp8_host, uint64_t rows, uint64_t cols,
                const ecf8_encode_opts *opts, ecf8_blob **out);
void ecf8_blob_free(ecf8_blob *blob);
const void *ecf8_blob_data(const ecf8_blob *blob); /* host pointer, 256-byte aligned */
uint64_t ecf8_blob_size(const ecf8_blob *blob);

/*
 * ecf8_encode_gpu (Section 3.1 on the device: the paper's encoding pipeline runs
 * on the GPU).  d_fp8: DEVICE, rows*cols raw E4M3 bytes, 16-byte aligned;
 * d_blob: DEVICE buffer of blob_capacity bytes, 256-byte aligned, that receives
 * the container -- byte for byte the one ecf8_encode writes for the same input
 * and options (n_threads is ignored).  ecf8_encode_bound gives a capacity that
 * always suffices; ECF8_E_CAPACITY if the blob turns out larger than
 * blob_capacity (at least 256 bytes are needed in any case).  *hdr_out receives
 * the header.  The call synchronises `stream` ONCE (it reads the 16-bin
 * histogram back to build the code on the host), then queues the rest
 * asynchronously.  Uses no memory besides its input and output.
 */
int ecf8_encode_bound(uint64_t rows, uint64_t cols, const ecf8_encode_opts *opts, uint64_t *bytes);
int ecf8_encode_gpu(const void *d_fp8, uint64_t rows, uint64_t cols, const ecf8_encode_opts *opts,
                    void *d_blob, uint64_t blob_capacity, ecf8_header *hdr_out, void *stream);

/*
 * Header parse + structural checks of a container held in HOST memory
 * (sizes, offsets, alignment, code lengths satisfy Kraft).  Fills *hdr, which
 * is what the decode calls need on the host at launch time.
 */
int ecf8_blob_describe(const void *blob_host, uint64_t size, ecf8_header *hdr);

/*
 * Full metadata check of a HOST container before it is trusted on the device:
 * describe() plus chunk_bit monotone and consistent with lane_bits, lane_bits
 * <= 15 N, histogram consistent with stream_bits, zero padding, and an embedded
 * table equal to the one code_len[] defines.  The decode
 * calls do not read device memory from the host, so validate on the host
 * before uploading.
 */
int ecf8_blob_validate(const void *blob_host, uint64_t size);

int ecf8_blob_stats(const ecf8_header *hdr, ecf8_stats *stats);

/*
 * ecf8_decode (Section 3.2 / Algorithm 1: compressed buffers in, exact FP8
 * tensor out).  d_blob: DEVICE copy of the blob described by *hdr (16-byte
 * aligned).  d_out: DEVICE buffer of out_capacity >= n_elem bytes, 16-byte
 * aligned; exactly n_elem bytes are written.  Asynchronous on `stream`.
 */
int ecf8_decode(const ecf8_header *hdr, const void *d_blob, void *d_out,
                uint64_t out_capacity, void *stream);

/* One tensor of a batch as the kernel reads it from DEVICE memory. */
typedef struct ecf8_batch_item {
    uint64_t d_blob;       /* device address of the tensor's blob                */
    uint64_t d_out;        /* device address of its output buffer                */
    uint64_t n_elem;
    uint64_t n_chunks;
    uint64_t first_chunk;  /* chunks of all earlier items of the batch           */
    uint64_t off_chunk_bit, off_lane_bits, off_stream, off_plane;
    uint64_t stream_bytes;
    uint8_t code_len[16];
    uint64_t off_table;    /* 0 = the blob holds no table                        */
    uint64_t group_chunks; /* G of the tensor's header                           */
    uint64_t tile_cols;    /* 0: linear layout; else cols of a row-tiled tensor  */
    uint64_t reserved[1];
} ecf8_batch_item; /* 128 bytes */

/* What a batched launch needs to know on the host. */
typedef struct ecf8_batch_info {
    uint64_t total_chunks;  /* chunks of all tensors of the batch                 */
    uint32_t lane_syms;     /* N, shared by all tensors of the batch              */
    uint32_t max_code_len;  /* longest codeword of any tensor of the batch        */
    uint32_t max_workgroups; /* 0 = one workgroup per compute unit (fastest decode); */
                            /* else a cap, to leave compute units to kernels that   */
                            /* run beside the decode (a decode workgroup fills its  */
                            /* compute unit); batch_prepare sets 0                  */
    uint32_t row_tiled;     /* 1: every tensor of the batch is in the row-tiled layout */
                            /* (their chunks then leave the kernel as whole row       */
                            /* segments); batch_prepare sets it                       */
} ecf8_batch_info;

/*
 * ecf8_batch_prepare: HOST.  Fills items_host[0..n) from the headers and the
 * device addresses; the caller copies the array to device memory once and
 * keeps it, together with *info.  All tensors of a batch must share lane_syms.
 */
int ecf8_batch_prepare(const ecf8_header *hdrs, const void *const *d_blobs,
                       void *const *d_outs, const uint64_t *out_capacities,
                       uint32_t n_tensors, ecf8_batch_item *items_host,
                       ecf8_batch_info *info);

/*
 * ecf8_decode_batched: many tensors in ONE launch (the per-layer decode of
 * Section 3.3 collapsed over a layer's matrices / an MoE layer's experts).
 * d_items: DEVICE array written by ecf8_batch_prepare (16-byte aligned);
 * info: HOST, as filled by ecf8_batch_prepare for exactly these items.
 */
int ecf8_decode_batched(const ecf8_batch_item *d_items, uint32_t n_tensors,
                        const ecf8_batch_info *info, void *stream);

/*
 * ecf8_gemm_fp8: fused decode + FP8 GEMM for small batches.  The paper decodes a
 * layer into a buffer and lets the framework's GEMM read it back (Section 3.3);
 * here decoded weights go from the registers they are decoded into straight
 * into the FP8 matrix cores.
 *   Y[m][n] = sum_k X[m][k] * W[n][k]   (fp32 accumulate)
 * W: the rows x cols tensor held by the blob (hdr / d_blob as for ecf8_decode);
 * d_x: DEVICE, M x cols FP8 E4M3 bytes, row-major, 16-byte aligned, 1 <= M <= 64;
 * d_y: DEVICE, M x rows fp32, row-major.  Supported for now: cols a multiple of 256
 * (cols == 4096 keeps X in registers and is the fast case), rows a
 * multiple of 16, a blob in the row-tiled layout (tile_rows == 16) with
 * lane_syms == 64 and no codeword longer than 7 bits (the encoder's default
 * cap); ECF8_E_ARG otherwise.  Values are
 * used as stored (unit scales); NaN encodings propagate as NaN.
 * ecf8_gemm_fp8_raw: the same GEMM on uncompressed W (d_w: DEVICE, rows x cols
 * bytes, 16-byte aligned), the baseline the fused call is compared with.
 */
int ecf8_gemm_fp8(const ecf8_header *hdr, const void *d_blob, const void *d_x, uint32_t M,
                  float *d_y, void *stream);
int ecf8_gemm_fp8_raw(const void *d_w, uint64_t rows, uint64_t cols, const void *d_x, uint32_t M,
                      float *d_y, void *stream);

/*
 * The same two calls with the scales block-quantised FP8 checkpoints carry (the
 * paper's models store one scale per 128 x 128 block of W beside the FP8 bytes;
 * the codec itself never touches them, Section 3):
 *   Y[m][n] = sum_kb x_scale[m][kb] * w_scale[n/128][kb] * sum_{k in block kb} X[m][k] * W[n][k]
 * d_w_scale: DEVICE, fp32 [ceil(rows/128)][cols/128], row-major; d_x_scale: DEVICE,
 * fp32 [M][x_scale_cols], row-major, with x_scale_cols = 1 (one scale per row of X,
 * x_scale[m][kb] = x_scale[m]) or cols/128 (one per row and 128 columns, as
 * activations quantised in 1 x 128 groups carry them); NULL with x_scale_cols = 0 for
 * ones.  Each 128-wide slice of K is summed by the matrix cores on its own and enters
 * the fp32 sum through one multiply-add with its scale (the product of the two scales,
 * rounded to fp32, where X has one per slice); a single row scale multiplies the
 * finished sum.  Other arguments, limits and errors as above.  The raw twin takes the
 * same steps in the same order: the two agree bit for bit.
 */
int ecf8_gemm_fp8_scaled(const ecf8_header *hdr, const void *d_blob, const void *d_x, uint32_t M,
                         const float *d_w_scale, const float *d_x_scale, uint32_t x_scale_cols,
                         float *d_y, void *stream);
int ecf8_gemm_fp8_raw_scaled(const void *d_w, uint64_t rows, uint64_t cols, const void *d_x, uint32_t M,
                             const float *d_w_scale, const float *d_x_scale, uint32_t x_scale_cols,
                             float *d_y, void *stream);

/*
 * The same products on the F16 matrix cores, for callers who need the sum itself rather
 * than the FP8 matrix cores' version of it.  The FP8 cores (the calls above) align the
 * 8 products a lane contributes to a step to the largest of them and drop what lies more
 * than about 13 bits below it: an output can be off by up to 7 * 2^-13 * sum_k |x_k w_k|.
 * Here decoded weights and X are converted to halves in registers (exact: every E4M3
 * value is a half), so products are exact and sums are fp32 sums: outputs agree with the
 * sum in real numbers to fp32 rounding (tested to 1e-5 * sum_k |x_k w_k|, the tolerance of
 * the fused-GEMM configuration).  Same arguments, limits and errors as
 * ecf8_gemm_fp8_scaled / _raw_scaled; d_w_scale = d_x_scale = NULL and x_scale_cols = 0
 * give the unscaled product.  The fused call and its raw twin agree bit for bit.
 * Cost: two conversions per decoded dword and per dword of X; none of it in the decode.
 */
int ecf8_gemm_fp8_exact(const ecf8_header *hdr, const void *d_blob, const void *d_x, uint32_t M,
                        const float *d_w_scale, const float *d_x_scale, uint32_t x_scale_cols,
                        float *d_y, void *stream);
int ecf8_gemm_fp8_raw_exact(const void *d_w, uint64_t rows, uint64_t cols, const void *d_x, uint32_t M,
                            const float *d_w_scale, const float *d_x_scale, uint32_t x_scale_cols,
                            float *d_y, void *stream);

/*
 * Split K, for matrices of few rows and long K (rows / 16 well below the number
 * of compute units: low-rank projections, routers).  The calls above give a block
 * of 16 rows of W to one workgroup, so such a matrix would leave most of the chip
 * idle; here `slices` workgroups share a block, each takes an equal part of its
 * K / 256 chunks, writes its partial sums to the workspace, and the workgroup that
 * arrives last adds the parts up in slice order (the result does not depend on the
 * order of arrival; the raw twin takes the same steps and agrees bit for bit) and
 * writes Y.  No workgroup waits for another.  Same operation, arguments, limits
 * and errors as ecf8_gemm_fp8_scaled, with d_w_scale = d_x_scale = NULL and
 * x_scale_cols = 0 for the unscaled product.
 *   ecf8_gemm_splitk_plan             HOST: slices and workspace size for (rows, cols, M) on a
 *                                     device of `compute_units` compute units (0 = the current
 *                                     device; any other value needs no device); either output
 *                                     pointer may be NULL.  ECF8_E_ARG for a shape or M the
 *                                     calls do not take
 *   ecf8_gemm_splitk_slices           slices the calls will use for this shape on the
 *                                     current device: the largest divisor of cols / 256
 *                                     with rows / 16 * slices <= compute units (1 = the
 *                                     matrix has blocks enough and the calls fall through
 *                                     to the plain kernels; 0 = bad shape or no device)
 *   ecf8_gemm_splitk_workspace_bytes  size the calls need for (rows, cols, M) on the
 *                                     current device: 0 when slices <= 1, else
 *                                     4096 + rows / 16 * slices * 1024 * (1, 2 or 4 for M <= 16, 32, 64)
 *   ecf8_gemm_splitk_workspace_init   zeroes a workspace (a kernel on `stream`): once
 *                                     after allocating it
 * d_workspace: DEVICE, 16-byte aligned, caller-owned, workspace_bytes >= the size
 * above (ECF8_E_CAPACITY otherwise; may be NULL when that size is 0).  Its first
 * 4096 bytes are the arrival counters, which every call leaves at zero as it found them, so
 * one workspace serves any number of calls of any shapes it is large enough for,
 * one after the other; calls that overlap in time need a workspace each.  A call
 * that did not run to its end (a device error) leaves the counters undefined:
 * initialise again.
 */
int ecf8_gemm_splitk_plan(uint64_t rows, uint64_t cols, uint32_t M, uint32_t compute_units,
                          uint32_t *slices, uint64_t *workspace_bytes);
uint32_t ecf8_gemm_splitk_slices(uint64_t rows, uint64_t cols);
uint64_t ecf8_gemm_splitk_workspace_bytes(uint64_t rows, uint64_t cols, uint32_t M);
int ecf8_gemm_splitk_workspace_init(void *d_workspace, uint64_t workspace_bytes, void *stream);
int ecf8_gemm_fp8_splitk(const ecf8_header *hdr, const void *d_blob, const void *d_x, uint32_t M,
                         const float *d_w_scale, const float *d_x_scale, uint32_t x_scale_cols,
                         float *d_y, void *d_workspace, uint64_t workspace_bytes, void *stream);
int ecf8_gemm_fp8_raw_splitk(const void *d_w, uint64_t rows, uint64_t cols, const void *d_x, uint32_t M,
                             const float *d_w_scale, const float *d_x_scale, uint32_t x_scale_cols,
                             float *d_y, void *d_workspace, uint64_t workspace_bytes, void *stream);

/*
 * ecf8_gemm_fp8_splitk_static: ecf8_gemm_fp8_splitk for callers that cannot provide or
 * allocate a workspace (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc).  Same operation, arguments, results (bit for bit) and errors, without
 * the workspace arguments: counters and partial sums live in an array inside the library's
 * device code, 4096 + 256 * 4096 bytes = 1 052 672 bytes per GPU, held until the process
 * ends.  ECF8_E_CAPACITY when the shape would need more (only on devices of more than 256
 * compute units).  The call allocates nothing and synchronises nothing.  All calls on one
 * GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 * threads) race, issue them one after the other.  The first call on a GPU also clears the
 * counters with a small kernel on `stream`; every completed call leaves them at zero.
 */
int ecf8_gemm_fp8_splitk_static(const ecf8_header *hdr, const void *d_blob, const void *d_x, uint32_t M,
                                const float *d_w_scale, const float *d_x_scale, uint32_t x_scale_cols,
                                float *d_y, void *stream);

/*
 * A group of small products in ONE launch, each with its own W, X, M and Y: the
 * experts that a batch of tokens is routed to in a mixture-of-experts layer (the
 * largest model of the paper's Table 1 is one).  A launch per matrix is bound by
 * launches and leaves most of the chip idle (a 2048 x 7168 expert is 128 blocks
 * of rows); here the blocks of all matrices form one sequence, weighted by their
 * K / 256 chunks, which the workgroups share evenly.  Every product is computed
 * as ecf8_gemm_fp8 / _scaled (or the raw twins) compute it, under the same limits
 * on each matrix.  A group of compressed and the same group of uncompressed matrices
 * agree bit for bit.  Against the single calls a member agrees bit for bit when that
 * call runs workgroups of the group's shape (cols != 4096, and M on the same side of
 * 16 as the group's largest M: the shape follows the largest M, and with it the order
 * in which a block's chunk sums are added) and to a few fp32 roundings otherwise.
 *   ecf8_gemm_group_prepare  HOST: checks the n descriptions and fills items_host[n]
 *                            (copy them to DEVICE memory, 8-byte aligned, caller-
 *                            owned) and *info (stays on the host).  All matrices of
 *                            a group are compressed (hdr != NULL, d_w = the blob) or
 *                            all uncompressed (hdr == NULL, d_w = rows x cols bytes),
 *                            and carry the same kind of scales (none; d_w_scale with
 *                            no or one x scale per row; d_w_scale with x scales per
 *                            row and 128 columns), ECF8_E_ARG otherwise.  M may
 *                            differ from matrix to matrix (1 <= M <= 64).
 *   ecf8_gemm_fp8_grouped    DEVICE, asynchronous on `stream`; the items may be reused
 *                            for any number of launches while the buffers they
 *                            point to live.
 * Errors: prepare returns what the single call would return for the first member it
 * rejects (ECF8_E_ARG, _E_FORMAT, _E_ALIGN) and ECF8_E_ARG for a mixed group; it
 * writes nothing the caller can use in that case.  The launch checks *info
 * (ECF8_E_ARG), the alignment of d_items (ECF8_E_ALIGN) and the launch itself
 * (ECF8_E_HIP); it trusts the items, which only prepare writes.  Outputs of members
 * are independent: rows of Y beyond a member's M are never written.
 */
typedef struct ecf8_gemm_group_desc {
    const ecf8_header *hdr;   /* HOST; NULL for an uncompressed matrix              */
    const void *d_w;          /* DEVICE: the blob, or rows x cols FP8 bytes          */
    uint64_t rows, cols;      /* uncompressed matrices only (else taken from hdr)    */
    const void *d_x;          /* DEVICE: M x cols FP8 bytes                          */
    float *d_y;               /* DEVICE: M x rows fp32                               */
    const float *d_w_scale;   /* DEVICE or NULL, as for ecf8_gemm_fp8_scaled         */
    const float *d_x_scale;
    uint32_t x_scale_cols;
    uint32_t M;
} ecf8_gemm_group_desc;

typedef struct ecf8_gemm_group_item {
    uint64_t opaque[32];      /* the kernel's view of one matrix                     */
} ecf8_gemm_group_item;

typedef struct ecf8_gemm_group_info {
    uint64_t total_work;      /* chunks of 16 x 256 weights over all matrices        */
    uint32_t n_items;
    uint32_t max_M;
    uint32_t scale_mode;      /* 0 none, 1 W blocks (+ X rows), 2 W blocks + X groups */
    uint32_t raw;             /* 1: uncompressed matrices                            */
} ecf8_gemm_group_info;

int ecf8_gemm_group_prepare(const ecf8_gemm_group_desc *descs, uint32_t n,
                            ecf8_gemm_group_item *items_host, ecf8_gemm_group_info *info);
int ecf8_gemm_fp8_grouped(const ecf8_gemm_group_item *d_items, const ecf8_gemm_group_info *info,
                          void *stream);

/*
 * Just-in-time layer decode (Section 3.3: compressed layers stay resident, a
 * layer is decoded into a pre-allocated buffer right before its forward pass
 * and the buffer is reused by later layers).  The manager is host-side
 * bookkeeping around ecf8_decode_batched: it owns one decode stream and a few
 * events, no device memory.  Layer l uses buffer l % n_buffers; with two or
 * more buffers the decode of layer l+1 overlaps the compute of layer l.
 * Calls on one manager must come from one host thread at a time.
 *
 *   create        d_buffers: n_buffers DEVICE buffers of buffer_bytes each
 *                 (16-byte aligned, caller-owned, must outlive the manager)
 *   layer_prepare HOST: lays the layer's tensors out in its buffer (offsets[i]
 *                 = byte offset of tensor i, multiples of 256) and fills
 *                 items_host[0..n) for that placement; ECF8_E_CAPACITY if the
 *                 layer does not fit.  The caller copies items_host to device
 *                 memory and hands that copy over with layer_commit
 *   prefetch      launches the layer's decode on the manager's stream, after
 *                 the buffer's previous user has released it.  ECF8_E_ARG if
 *                 the buffer is still ready/acquired for another layer
 *   acquire       makes `stream` wait for the layer's decode; *d_base = the
 *                 buffer (tensor i is at d_base + offsets[i]).  Work queued
 *                 on `stream` after this call sees the decoded weights
 *   release       records on `stream` that the layer's weights are no longer
 *                 needed; the buffer's next prefetch waits for that point
 *   set_decode_workgroups  cap on the decode launches' workgroups (0 = one
 *                 per compute unit), to leave compute units to the consumer's
 *                 kernels while a decode runs beside them
 *   destroy       drains the decode stream and frees the host objects
 */
typedef struct ecf8_jit ecf8_jit;
int ecf8_jit_create(uint32_t n_layers, uint32_t n_buffers, void *const *d_buffers,
                    uint64_t buffer_bytes, ecf8_jit **out);
void ecf8_jit_destroy(ecf8_jit *jit);
int ecf8_jit_layer_prepare(ecf8_jit *jit, uint32_t layer, const ecf8_header *hdrs,
                           const void *const *d_blobs, uint32_t n_tensors,
                           ecf8_batch_item *items_host, uint64_t *offsets);
int ecf8_jit_layer_commit(ecf8_jit *jit, uint32_t layer, const ecf8_batch_item *d_items);
int ecf8_jit_set_decode_workgroups(ecf8_jit *jit, uint32_t max_workgroups);
int ecf8_jit_prefetch(ecf8_jit *jit, uint32_t layer);
int ecf8_jit_acquire(ecf8_jit *jit, uint32_t layer, void *stream, void **d_base);
int ecf8_jit_release(ecf8_jit *jit, uint32_t layer, void *stream);

const char *ecf8_strerror(int code);
uint32_t ecf8_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ECF8_H */
