// Internal declarations shared by the translation units of libhikonv.so.
#ifndef HIKONV_INTERNAL_H
#define HIKONV_INTERNAL_H

#include "../../include/hikonv.h"

namespace hikonv {

// container width of the bit-dense format for b-bit values (0 = invalid b)
inline int container_bits(int bits)
{
    switch (bits) {
    case 1: return 1;
    case 2: return 2;
    case 3: case 4: return 4;
    case 5: case 6: case 7: case 8: return 8;
    default: return 0;
    }
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

} // namespace hikonv

#endif
