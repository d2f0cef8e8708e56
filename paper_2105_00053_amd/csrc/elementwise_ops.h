// Per-element operations of the bandwidth-bound entry points, written as
// functors over raw bit patterns: float -> posit (posit_round), posit -> posit
// and posit -> float (posit_convert; the paper's "convert PyTorch tensors" and
// "mixed precision tensor" utilities, Fig. 2), and the SGD update
// y <- round(y + alpha * x) (posit_axpy; Fig. 2 optimizer).  Every result is
// computed exactly and rounded once.
#pragma once

#include "posit_core.h"

namespace pnn {

template <class FD>
struct RoundF32 {
    PNN_HD uint64_t operator()(uint64_t bits) const {
        Real r;
        const int c = real_from_f32((uint32_t)bits, r);
        if (c == 0) return 0;
        if (c == 2) return FD::NAR;
        return encode<FD>(r);
    }
};

template <class FD>
struct RoundF64 {
    PNN_HD uint64_t operator()(uint64_t bits) const {
        Real r;
        const int c = real_from_f64(bits, r);
        if (c == 0) return 0;
        if (c == 2) return FD::NAR;
        return encode<FD>(r);
    }
};

template <class FS, class FD>
struct PositToPosit {
    PNN_HD uint64_t operator()(uint64_t p) const {
        const uint32_t q = (uint32_t)p & FS::MASK;
        if (q == 0) return 0;
        if (q == FS::NAR) return FD::NAR;
        return encode<FD>(decode_fields<FS>(q));
    }
};

template <class FS>
struct PositToF32 {
    PNN_HD uint64_t operator()(uint64_t p) const {
        const uint32_t q = (uint32_t)p & FS::MASK;
        if (q == 0) return 0;
        if (q == FS::NAR) return 0x7FC00000u;  // quiet NaN
        return real_to_f32_bits(decode_fields<FS>(q));
    }
};

template <class FS>
struct PositToF64 {
    PNN_HD uint64_t operator()(uint64_t p) const {
        const uint32_t q = (uint32_t)p & FS::MASK;
        if (q == 0) return 0;
        if (q == FS::NAR) return 0x7FF8000000000000ull;
        return real_to_f64_bits(decode_fields<FS>(q));
    }
};

// y_new = round_FY( y + alpha * x ), alpha given as a pattern of FY.
template <class FX, class FY>
struct Axpy {
    uint32_t alpha;
    PNN_HD uint32_t operator()(uint32_t x, uint32_t y) const {
        x &= FX::MASK;
        y &= FY::MASK;
        const uint32_t a = alpha & FY::MASK;
        if (a == FY::NAR || x == FX::NAR || y == FY::NAR) return FY::NAR;
        const bool t_zero = (a == 0) || (x == 0);
        if (t_zero) return y;  // y + 0 is y itself
        const Real t = real_mul(decode_fields<FY>(a), decode_fields<FX>(x));
        if (y == 0) return encode<FY>(t);
        Real s;
        if (!real_add(decode_fields<FY>(y), t, s)) return 0;
        return encode<FY>(s);
    }
};

}  // namespace pnn
