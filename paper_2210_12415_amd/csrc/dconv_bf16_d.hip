// Instantiations of the patch-resident direct convolution: 64x64 tiles.
#include "dconv.h"

namespace alt {
namespace {

#define ALT_DCONV(BM, BN, WGM, WGN, NS)                                                                          \
    const bool reg_dconv_##BM##x##BN##_w##WGM##x##WGN##_s##NS =                                                  \
        (igemm_register(IgemmLaunch{"bf16_" #BM "x" #BN "x64_direct_w" #WGM "x" #WGN "_s" #NS, ALT_BF16, BM, BN,  \
                                    64, LOAD_VEC, LOAD_VEC, NS - 1, 1, 0, nullptr,                               \
                                    &dconv_launch<BM, BN, WGM, WGN, NS>, WGM, WGN}),                             \
         true)

ALT_DCONV(64, 64, 1, 1, 3);
ALT_DCONV(64, 64, 1, 1, 5);
ALT_DCONV(64, 64, 2, 2, 3);
ALT_DCONV(64, 64, 2, 2, 5);
ALT_DCONV(64, 64, 2, 1, 3);
ALT_DCONV(64, 64, 2, 1, 5);

}  // namespace
}  // namespace alt
