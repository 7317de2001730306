// Internal (not part of the C ABI): what the CPU encoder and the GPU encoder of the wide-alphabet
// codec share on the host -- option checks, the code built from a histogram, the container layout.
#ifndef ECFW_PLAN_H
#define ECFW_PLAN_H

#include <cstdint>

#include "ecfw.h"

namespace ecfw_internal {

struct WPlan {
    ecfw_header hdr;              // complete header of the blob to be written
    uint8_t len[256];             // code length of exponent field x, 0 = absent
    uint32_t code[256];           // canonical codewords, first bit most significant
    uint32_t rcode[256];          // the same, bit-reversed (first bit = bit 0)
};

// Checks rows/cols/opts (ECF8_E_ARG) and returns the effective options.
int check_options(const ecfw_encode_opts *opts, uint64_t rows, uint64_t cols, uint32_t *lane_syms,
                  uint32_t *group_chunks, uint32_t *max_code_len);

// From the exponent-field histogram of a rows x cols tensor: cheapest code under the cap, canonical
// codewords, section layout, header.  Same result for the same inputs on every path.
int plan_encode(const uint64_t *freq, uint32_t fmt, uint64_t rows, uint64_t cols, uint32_t lane_syms,
                uint32_t group_chunks, uint32_t max_code_len, WPlan *out);

// Largest blob any rows x cols tensor can need under the cap.
int encode_bound(uint32_t fmt, uint64_t rows, uint64_t cols, uint32_t lane_syms, uint32_t max_code_len, uint64_t *bytes);

} // namespace ecfw_internal

#endif
