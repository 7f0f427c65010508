// Instantiations of the register-weights direct convolution (NHWC or blocked activations, OHWI weights).
#include "dregw.h"
#include "dstream.h"

namespace alt {
namespace {

#include "dconv_reg.h"

ALT_DREGW();

}  // namespace
}  // namespace alt
