// Instantiations of the patch-resident direct convolution: K groups, 128- and 256-row tiles.
#include "dconv_reg.h"

namespace alt {
namespace {

ALT_DCONV_KW(128, 64, 2, 1, 4, 3, 64);
ALT_DCONV_KW(128, 64, 2, 1, 4, 3, 32);
ALT_DCONV_KW(128, 64, 2, 1, 2, 3, 64);
ALT_DCONV_KW(256, 64, 4, 1, 2, 3, 64);
ALT_DCONV_KW(128, 128, 2, 2, 2, 3, 64);
ALT_DCONV_KW(256, 64, 4, 1, 2, 3, 32);
ALT_DCONV_KW(256, 64, 4, 1, 2, 5, 32);
ALT_DCONV_KW(128, 64, 2, 1, 2, 5, 32);

}  // namespace
}  // namespace alt
