// Host-side helpers shared by the C ABI entry points: format codes, argument
// checks, status strings.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/positnn.h"

namespace pnn {

inline bool is_posit(int f) { return f == PNN_POSIT8_0 || f == PNN_POSIT16_1 || f == PNN_POSIT32_2; }
inline bool is_float(int f) { return f == PNN_F32 || f == PNN_F64; }
inline size_t elem_size(int f) {
    switch (f) {
        case PNN_POSIT8_0: return 1;
        case PNN_POSIT16_1: return 2;
        case PNN_POSIT32_2: return 4;
        case PNN_F32: return 4;
        case PNN_F64: return 8;
    }
    return 0;
}
inline int quire_limbs(int f) { return f == PNN_POSIT8_0 ? 1 : f == PNN_POSIT16_1 ? 4 : 16; }
inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }
inline int hip_status(hipError_t e) { return e == hipSuccess ? PNN_OK : PNN_EHIP; }

}  // namespace pnn
