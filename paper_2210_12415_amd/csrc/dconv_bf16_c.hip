// Instantiations of the patch-resident direct convolution: 128x128 tiles.
#include "dconv.h"

namespace alt {
namespace {

#include "dconv_reg.h"

ALT_DCONV(128, 128, 2, 2, 3);
ALT_DCONV(128, 128, 2, 2, 5);
ALT_DCONV(128, 128, 4, 2, 3);
ALT_DCONV(128, 128, 4, 2, 5);
ALT_DCONV(64, 128, 1, 2, 3);
ALT_DCONV(64, 128, 1, 2, 5);

}  // namespace
}  // namespace alt
