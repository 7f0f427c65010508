// Instantiations of the implicit-GEMM kernel: bf16, both operands channel-contiguous, medium tiles.
#include "igemm.h"

namespace alt {
namespace {

#define ALT_IGEMM(T, TNAME, DT, BM, BN, BK, WGM, WGN, AM, BMD, MODES)                                   \
    const bool reg_##TNAME##_##BM##x##BN##x##BK##_##MODES =                                             \
        (igemm_register(IgemmLaunch{#TNAME "_" #BM "x" #BN "x" #BK "_" #MODES, DT, BM, BN, BK, AM, BMD, \
                                    igemm_lds_bytes<T, BM, BN, BK>(),                                   \
                                    &igemm_launch<T, BM, BN, BK, WGM, WGN, AM, BMD>}),                  \
         true)

ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 128, 64, 32, 2, 2, LOAD_VEC, LOAD_VEC, vv);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 128, 64, 64, 2, 2, LOAD_VEC, LOAD_VEC, vv);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 256, 64, 32, 4, 1, LOAD_VEC, LOAD_VEC, vv);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 256, 64, 64, 4, 1, LOAD_VEC, LOAD_VEC, vv);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 64, 128, 32, 1, 4, LOAD_VEC, LOAD_VEC, vv);

}  // namespace
}  // namespace alt
