// Instantiations of the patch-resident direct convolution: 32-channel K steps with one K
// group (small weight rings, so several workgroups share a compute unit's LDS).
#include "dconv_reg.h"

namespace alt {
namespace {

ALT_DCONV_KW(128, 64, 4, 1, 1, 3, 32);
ALT_DCONV_KW(128, 64, 4, 1, 1, 4, 32);
ALT_DCONV_KW(128, 64, 2, 1, 1, 3, 32);
ALT_DCONV_KW(64, 64, 2, 1, 1, 3, 32);

}  // namespace
}  // namespace alt
