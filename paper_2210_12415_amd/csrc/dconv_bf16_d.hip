// Instantiations of the patch-resident direct convolution: 64x64 tiles.
#include "dconv.h"

namespace alt {
namespace {

#include "dconv_reg.h"

ALT_DCONV(64, 64, 1, 1, 3);
ALT_DCONV(64, 64, 1, 1, 5);
ALT_DCONV(64, 64, 2, 2, 3);
ALT_DCONV(64, 64, 2, 2, 5);
ALT_DCONV(64, 64, 2, 1, 3);
ALT_DCONV(64, 64, 2, 1, 5);

}  // namespace
}  // namespace alt
