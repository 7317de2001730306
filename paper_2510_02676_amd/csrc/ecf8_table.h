// Pair-table entry format shared by the host encoder (which may embed the table
// in the blob) and the decode kernel (which builds it in LDS when the blob holds
// none).  Product-internal; the public description is in include/ecf8.h.
#ifndef ECF8_TABLE_H
#define ECF8_TABLE_H
#include <stdint.h>

#if defined(__HIPCC__)
#define ECF8_HD __host__ __device__
#else
#define ECF8_HD
#endif

#define ECF8_TB 14                       /* table index bits */
#define ECF8_TBL_ENTRIES (1u << ECF8_TB)

// Entry for index bits b0 b1 ... (b0 = next stream bit in reading order), from the
// single-symbol facts (s1, l1) = first codeword spelled by the index bits, and
// (s2, l2) = the codeword that follows it; l = 0 means "needs more than ECF8_TB bits".
ECF8_HD static inline uint16_t ecf8_pair_entry(uint32_t s1, uint32_t l1, uint32_t s2, uint32_t l2)
{
    uint32_t e = 0;
    if (l1) {
        e = (s1 << 3) | (l1 & 7u) | ((l1 & 8u) << 12);
        if (l2 && l1 + l2 <= ECF8_TB) e |= (s2 << 11) | ((l1 + l2) << 7);
    }
    return (uint16_t)e;
}
#endif
