// Instantiations of the channel-planar direct convolution (NCHW / OIHW / NCHW).
#include "dplanar.h"

namespace alt {
namespace {

#include "dconv_reg.h"

ALT_DPLANAR(256, 64, 4, 2, 1);
ALT_DPLANAR(128, 64, 4, 2, 1);
ALT_DPLANAR(128, 64, 2, 2, 2);
ALT_DPLANAR(128, 32, 4, 1, 2);
ALT_DPLANAR(64, 64, 2, 2, 2);
ALT_DPLANAR(64, 32, 2, 1, 4);
ALT_DPLANAR(64, 32, 2, 1, 2);

}  // namespace
}  // namespace alt
