// Instantiations of the streaming GEMM kernel: small tiles and K groups.
#include "dconv_reg.h"

namespace alt {
namespace {

ALT_DSTREAM(128, 64, 2, 1, 1, 4, 64);
ALT_DSTREAM(128, 64, 4, 1, 1, 4, 64);
ALT_DSTREAM(128, 64, 4, 1, 1, 8, 32);
ALT_DSTREAM(128, 64, 2, 1, 2, 3, 64);
ALT_DSTREAM(128, 64, 2, 1, 2, 6, 32);
ALT_DSTREAM(64, 128, 1, 2, 2, 3, 64);
ALT_DSTREAM(64, 64, 2, 2, 1, 4, 64);
ALT_DSTREAM(64, 64, 2, 2, 1, 8, 32);
ALT_DSTREAM(256, 64, 8, 1, 1, 3, 64);
ALT_DSTREAM(256, 64, 8, 1, 1, 4, 64);

}  // namespace
}  // namespace alt
