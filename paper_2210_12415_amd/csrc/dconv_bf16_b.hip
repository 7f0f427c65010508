// Instantiations of the patch-resident direct convolution: smaller wavefront tiles.
#include "dconv.h"

namespace alt {
namespace {

#define ALT_DCONV(BM, BN, WGM, WGN, NS)                                                                          \
    const bool reg_dconv_##BM##x##BN##_w##WGM##x##WGN##_s##NS =                                                  \
        (igemm_register(IgemmLaunch{"bf16_" #BM "x" #BN "x64_direct_w" #WGM "x" #WGN "_s" #NS, ALT_BF16, BM, BN,  \
                                    64, LOAD_VEC, LOAD_VEC, NS - 1, 1, 0, nullptr,                               \
                                    &dconv_launch<BM, BN, WGM, WGN, NS>}),                                       \
         true)

ALT_DCONV(128, 64, 4, 1, 2);
ALT_DCONV(128, 64, 4, 1, 3);
ALT_DCONV(128, 64, 4, 1, 4);
ALT_DCONV(256, 64, 8, 1, 2);
ALT_DCONV(256, 64, 8, 1, 3);
ALT_DCONV(256, 64, 8, 1, 4);
ALT_DCONV(64, 64, 2, 2, 2);
ALT_DCONV(64, 64, 2, 2, 3);
ALT_DCONV(64, 64, 2, 2, 4);
ALT_DCONV(128, 64, 4, 2, 2);
ALT_DCONV(128, 64, 4, 2, 3);
ALT_DCONV(128, 64, 4, 2, 4);
ALT_DCONV(64, 64, 2, 1, 2);
ALT_DCONV(64, 64, 2, 1, 3);
ALT_DCONV(64, 64, 2, 1, 4);
ALT_DCONV(128, 128, 4, 2, 2);
ALT_DCONV(128, 128, 4, 2, 3);
ALT_DCONV(128, 128, 4, 2, 4);

}  // namespace
}  // namespace alt
