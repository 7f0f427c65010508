// Instantiations of the implicit-GEMM kernel: bf16, both operands channel-contiguous, large tiles.
#include "igemm.h"

namespace alt {
namespace {

#define ALT_IGEMM(T, TNAME, DT, BM, BN, BK, WGM, WGN, AM, BMD, MODES)                                   \
    const bool reg_##TNAME##_##BM##x##BN##x##BK##_##MODES =                                             \
        (igemm_register(IgemmLaunch{#TNAME "_" #BM "x" #BN "x" #BK "_" #MODES, DT, BM, BN, BK, AM, BMD, \
                                    igemm_lds_bytes<T, BM, BN, BK>(),                                   \
                                    &igemm_launch<T, BM, BN, BK, WGM, WGN, AM, BMD>}),                  \
         true)

ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 128, 128, 32, 2, 2, LOAD_VEC, LOAD_VEC, vv);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 128, 128, 64, 2, 2, LOAD_VEC, LOAD_VEC, vv);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 256, 128, 32, 2, 2, LOAD_VEC, LOAD_VEC, vv);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 256, 128, 64, 2, 2, LOAD_VEC, LOAD_VEC, vv);

}  // namespace
}  // namespace alt
