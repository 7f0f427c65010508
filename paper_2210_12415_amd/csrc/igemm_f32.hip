// Instantiations of the implicit-GEMM kernel: fp32 (fp32 MFMA, true fp32 products).
#include "igemm.h"

namespace alt {
namespace {

#define ALT_IGEMM(T, TNAME, DT, BM, BN, BK, WGM, WGN, AM, BMD, MODES)                                   \
    const bool reg_##TNAME##_##BM##x##BN##x##BK##_##MODES =                                             \
        (igemm_register(IgemmLaunch{#TNAME "_" #BM "x" #BN "x" #BK "_" #MODES, DT, BM, BN, BK, AM, BMD, \
                                    igemm_lds_bytes<T, BM, BN, BK>(),                                   \
                                    &igemm_launch<T, BM, BN, BK, WGM, WGN, AM, BMD>}),                  \
         true)

ALT_IGEMM(float, f32, ALT_F32, 64, 64, 16, 2, 2, LOAD_VEC, LOAD_VEC, vv);
ALT_IGEMM(float, f32, ALT_F32, 128, 64, 16, 2, 2, LOAD_VEC, LOAD_VEC, vv);
ALT_IGEMM(float, f32, ALT_F32, 128, 128, 16, 2, 2, LOAD_VEC, LOAD_VEC, vv);
ALT_IGEMM(float, f32, ALT_F32, 64, 64, 32, 2, 2, LOAD_VEC, LOAD_VEC, vv);
ALT_IGEMM(float, f32, ALT_F32, 64, 64, 16, 2, 2, LOAD_GATHER, LOAD_VEC, gv);
ALT_IGEMM(float, f32, ALT_F32, 128, 64, 16, 2, 2, LOAD_GATHER, LOAD_VEC, gv);
ALT_IGEMM(float, f32, ALT_F32, 64, 64, 16, 2, 2, LOAD_GATHER, LOAD_GATHER, gg);
ALT_IGEMM(float, f32, ALT_F32, 64, 64, 8, 2, 2, LOAD_GATHER, LOAD_GATHER, gg);
ALT_IGEMM(float, f32, ALT_F32, 128, 64, 16, 2, 2, LOAD_GATHER, LOAD_GATHER, gg);
ALT_IGEMM(float, f32, ALT_F32, 64, 64, 16, 2, 2, LOAD_VEC, LOAD_GATHER, vg);
ALT_IGEMM(float, f32, ALT_F32, 64, 64, 16, 2, 2, LOAD_VEC, LOAD_TRANS, vt);
ALT_IGEMM(float, f32, ALT_F32, 128, 128, 16, 2, 2, LOAD_VEC, LOAD_TRANS, vt);
ALT_IGEMM(float, f32, ALT_F32, 64, 64, 16, 2, 2, LOAD_TRANS, LOAD_TRANS, tt);
ALT_IGEMM(float, f32, ALT_F32, 64, 64, 16, 2, 2, LOAD_TRANS, LOAD_VEC, tv);

}  // namespace
}  // namespace alt
