// Instantiations of the patch-resident direct convolution: 256-row tiles.
#include "dconv.h"

namespace alt {
namespace {

#include "dconv_reg.h"

ALT_DCONV(256, 64, 4, 1, 3);
ALT_DCONV(256, 64, 4, 1, 5);
ALT_DCONV(256, 64, 8, 1, 3);
ALT_DCONV(256, 64, 8, 1, 5);
ALT_DCONV(256, 128, 4, 2, 3);
ALT_DCONV(256, 128, 4, 2, 5);

}  // namespace
}  // namespace alt
