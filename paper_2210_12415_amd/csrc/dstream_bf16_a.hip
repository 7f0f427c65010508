// Instantiations of the streaming GEMM kernel: large tiles.
#include "dconv_reg.h"

namespace alt {
namespace {

ALT_DSTREAM(256, 128, 4, 2, 1, 3, 64);
ALT_DSTREAM(256, 128, 2, 2, 1, 3, 64);
ALT_DSTREAM(128, 256, 2, 2, 1, 3, 64);
ALT_DSTREAM(256, 128, 4, 2, 1, 6, 32);
ALT_DSTREAM(128, 256, 2, 4, 1, 6, 32);
ALT_DSTREAM(128, 128, 2, 2, 1, 4, 64);
ALT_DSTREAM(128, 128, 4, 2, 1, 4, 64);
ALT_DSTREAM(128, 128, 4, 2, 1, 8, 32);
ALT_DSTREAM(256, 64, 4, 1, 1, 4, 64);
ALT_DSTREAM(256, 64, 4, 1, 1, 8, 32);
// 128 x 128 per wave: half the operand reads per MFMA of the 64 x 64 wave tiles above; the 256
// accumulator registers live in the second half of the register file (one wave per SIMD)
ALT_DSTREAM(256, 256, 2, 2, 1, 4, 32);
ALT_DSTREAM(256, 256, 4, 2, 1, 4, 32);
ALT_DSTREAM(256, 256, 2, 4, 1, 4, 32);

}  // namespace
}  // namespace alt
