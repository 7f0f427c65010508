// Instantiations of the patch-resident direct convolution: K groups, 64-row tiles.
#include "dconv_reg.h"

namespace alt {
namespace {

ALT_DCONV_KW(64, 64, 1, 1, 8, 3, 32);
ALT_DCONV_KW(64, 64, 1, 1, 8, 3, 64);
ALT_DCONV_KW(64, 64, 1, 1, 4, 3, 64);
ALT_DCONV_KW(128, 32, 2, 1, 4, 3, 64);
ALT_DCONV_KW(128, 32, 2, 1, 4, 5, 64);
ALT_DCONV_KW(64, 32, 1, 1, 8, 3, 32);
ALT_DCONV_KW(64, 32, 1, 1, 8, 4, 32);
ALT_DCONV_KW(64, 32, 1, 1, 8, 3, 64);

}  // namespace
}  // namespace alt
