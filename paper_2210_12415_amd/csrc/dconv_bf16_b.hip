// Instantiations of the patch-resident direct convolution: 128x64 tiles.
#include "dconv.h"

namespace alt {
namespace {

#include "dconv_reg.h"

ALT_DCONV(128, 64, 2, 1, 3);
ALT_DCONV(128, 64, 2, 1, 5);
ALT_DCONV(128, 64, 4, 1, 3);
ALT_DCONV(128, 64, 4, 1, 5);
ALT_DCONV(128, 64, 4, 2, 3);
ALT_DCONV(128, 64, 4, 2, 5);

}  // namespace
}  // namespace alt
