// Instantiations of the streaming GEMM kernel for row-major B ([K][N]: the GMM's default layout), read
// through the LDS transpose reads of gfx950.
#include "dstream.h"

namespace alt {
namespace {

#include "dconv_reg.h"

ALT_DSTREAM_KN(128, 64, 4, 1, 1, 4, 64);
ALT_DSTREAM_KN(128, 64, 2, 1, 2, 3, 64);
ALT_DSTREAM_KN(64, 64, 2, 2, 1, 4, 64);
ALT_DSTREAM_KN(128, 128, 4, 2, 1, 4, 64);
ALT_DSTREAM_KN(256, 64, 8, 1, 1, 3, 64);
ALT_DSTREAM_KN(256, 128, 2, 2, 1, 3, 64);
ALT_DSTREAM_KN(256, 128, 4, 2, 1, 3, 64);
ALT_DSTREAM_KN(128, 256, 2, 4, 1, 6, 32);
ALT_DSTREAM_KN(256, 256, 2, 4, 1, 4, 32);

}  // namespace
}  // namespace alt
