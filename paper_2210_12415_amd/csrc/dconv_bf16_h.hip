// Instantiations of the direct convolution kernel: 128 x 64 wave tiles (three operand reads per
// four MFMAs where the 64 x 64 wave tiles of the other lists take four), one wave per SIMD.
#include "dconv_reg.h"

namespace alt {
namespace {

ALT_DCONV(512, 64, 4, 1, 3);
ALT_DCONV(512, 64, 4, 1, 5);
ALT_DCONV(256, 128, 2, 2, 3);
ALT_DCONV(256, 128, 2, 2, 5);

}  // namespace
}  // namespace alt
