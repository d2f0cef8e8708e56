// Host-side helpers shared by the C ABI entry points: format codes, argument
// checks, status strings.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/positnn.h"

namespace pnn {

inline bool is_posit(int f) { return f >= PNN_POSIT8_0 && f <= PNN_POSIT12_2; }
inline bool is_standard(int f) { return (f >= PNN_POSIT8_0 && f <= PNN_POSIT32_2) || f == PNN_F32 || f == PNN_F64; }
inline bool is_float(int f) { return f == PNN_F32 || f == PNN_F64; }
inline size_t elem_size(int f) {
    switch (f) {
        case PNN_POSIT8_0: return 1;
        case PNN_POSIT16_1: return 2;
        case PNN_POSIT32_2: return 4;
        case PNN_POSIT8_1: case PNN_POSIT8_2: return 1;
        case PNN_POSIT10_1: case PNN_POSIT10_2: case PNN_POSIT12_1: case PNN_POSIT12_2: return 2;
        case PNN_F32: return 4;
        case PNN_F64: return 8;
    }
    return 0;
}
inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }
inline int hip_status(hipError_t e) { return e == hipSuccess ? PNN_OK : PNN_EHIP; }
// Entry points report their own launches through hipGetLastError(); an error left behind by an earlier, unrelated
// HIP call of this thread would otherwise be blamed on a call that launched fine.  Read (and so reset) it first.
inline void discard_stale_hip_error() { (void)hipGetLastError(); }

// Calls fn.template operator()<F>() ... with the format class of a posit code.
#define PNN_DISPATCH_POSIT(code, CALL)                    \
    switch (code) {                                        \
        case PNN_POSIT8_0: { typedef P8 F; CALL; } break;     \
        case PNN_POSIT16_1: { typedef P16 F; CALL; } break;   \
        case PNN_POSIT32_2: { typedef P32 F; CALL; } break;   \
        case PNN_POSIT8_1: { typedef P8_1 F; CALL; } break;   \
        case PNN_POSIT8_2: { typedef P8_2 F; CALL; } break;   \
        case PNN_POSIT10_1: { typedef P10_1 F; CALL; } break; \
        case PNN_POSIT10_2: { typedef P10_2 F; CALL; } break; \
        case PNN_POSIT12_1: { typedef P12_1 F; CALL; } break; \
        default: { typedef P12_2 F; CALL; } break;            \
    }

}  // namespace pnn
