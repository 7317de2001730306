// Internal (not part of the C ABI): what the CPU encoder and the GPU encoder share on the
// host -- option checks, the code built from a histogram, and the container layout.
#ifndef ECF8_PLAN_H
#define ECF8_PLAN_H

#include <cstdint>

#include "ecf8.h"

// A host blob: `data` comes from std::aligned_alloc(256, .) and is released by ecf8_blob_free.
struct ecf8_blob {
    uint8_t *data;
    uint64_t size;
};

namespace ecf8_internal {

struct Plan {
    ecf8_header hdr;              // complete header of the blob to be written
    uint32_t code[16];            // canonical codewords, first bit most significant
    uint32_t rcode[16];           // the same, bit-reversed (first bit = bit 0)
};

// Checks rows/cols/opts (ECF8_E_ARG) and returns the effective options.
int check_options(uint64_t rows, uint64_t cols, const ecf8_encode_opts *opts, uint32_t *lane_syms,
                  uint32_t *group_chunks, uint32_t *max_code_len, uint32_t *tile_rows, uint32_t *table_mode);

// From the exponent histogram of a rows x cols tensor: cheapest code under the cap, canonical
// codewords, section layout, header.  Same result for the same inputs on every path.
int plan_encode(const uint64_t freq[16], uint64_t rows, uint64_t cols, const ecf8_encode_opts *opts, Plan *out);

// Largest blob any rows x cols tensor can need under opts.
int encode_bound(uint64_t rows, uint64_t cols, const ecf8_encode_opts *opts, uint64_t *bytes);

// The decoder's pair table for a code (host builder; the kernels have their own).
void build_pair_table_host(const uint8_t len[16], uint16_t *tbl);

} // namespace ecf8_internal

#endif
