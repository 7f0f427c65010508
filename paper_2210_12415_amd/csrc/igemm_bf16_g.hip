// Instantiations of the implicit-GEMM kernel: bf16, element-gather loaders (NCHW / OIHW and other layouts).
#include "igemm.h"

namespace alt {
namespace {

#define ALT_IGEMM(T, TNAME, DT, BM, BN, BK, WGM, WGN, AM, BMD, MODES)                                   \
    const bool reg_##TNAME##_##BM##x##BN##x##BK##_##MODES =                                             \
        (igemm_register(IgemmLaunch{#TNAME "_" #BM "x" #BN "x" #BK "_" #MODES, DT, BM, BN, BK, AM, BMD, \
                                    igemm_lds_bytes<T, BM, BN, BK>(),                                   \
                                    &igemm_launch<T, BM, BN, BK, WGM, WGN, AM, BMD>}),                  \
         true)

ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 128, 128, 32, 2, 2, LOAD_GATHER, LOAD_VEC, gv);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 128, 64, 32, 2, 2, LOAD_GATHER, LOAD_VEC, gv);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 64, 64, 32, 2, 2, LOAD_GATHER, LOAD_VEC, gv);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 128, 128, 32, 2, 2, LOAD_GATHER, LOAD_GATHER, gg);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 128, 64, 32, 2, 2, LOAD_GATHER, LOAD_GATHER, gg);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 64, 64, 32, 2, 2, LOAD_GATHER, LOAD_GATHER, gg);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 64, 64, 16, 2, 2, LOAD_GATHER, LOAD_GATHER, gg);
ALT_IGEMM(bf16_tag, bf16, ALT_BF16, 64, 64, 32, 2, 2, LOAD_VEC, LOAD_GATHER, vg);

}  // namespace
}  // namespace alt
