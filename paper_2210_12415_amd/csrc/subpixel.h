// The sub-pixel form of a transposed convolution, one axis at a time (host side).
// Output index o = q*stride + ph takes input indices i with o = i*stride - pad + r*dil, that is
// i = q + delta with delta = (ph + pad - r*dil) / stride for the taps r where that divides: each
// of the `stride` phases is a stride-1 convolution of the input itself.  Over the common range of
// offsets (extent delta_max - delta_min + 1, padding -delta_min) the phases share one window.
#pragma once

#include <cstdint>

namespace alt {

struct PhaseAxis {
    int32_t taps, pad;            // extent and padding of the merged filter along this axis
    int64_t outq;                 // outputs per phase
    bool ok;
};

inline PhaseAxis phase_axis(int64_t in, int64_t taps, int stride, int pad, int dil)
{
    PhaseAxis a{0, 0, 0, false};
    const int64_t out = (in - 1) * stride - 2 * (int64_t)pad + (int64_t)dil * (taps - 1) + 1;
    if (out < 1 || out % stride) return a;
    int64_t lo = 0, hi = 0;
    bool any = false;
    for (int ph = 0; ph < stride; ++ph)
        for (int64_t r = 0; r < taps; ++r) {
            const int64_t num = ph + pad - r * dil;
            if (((num % stride) + stride) % stride) continue;
            const int64_t delta = (num - (((num % stride) + stride) % stride)) / stride;
            lo = any ? (delta < lo ? delta : lo) : delta;
            hi = any ? (delta > hi ? delta : hi) : delta;
            any = true;
        }
    if (!any || lo > 0 || hi - lo + 1 > 64) return a;
    a.taps = (int32_t)(hi - lo + 1);
    a.pad = (int32_t)-lo;
    a.outq = out / stride;
    a.ok = in + 2 * (int64_t)a.pad - a.taps + 1 == a.outq;
    return a;
}

}  // namespace alt
