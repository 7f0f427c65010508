// Registration of one direct-convolution tile configuration with the kernel table.
#pragma once
#include "dstream.h"

// BM x BN output tile, WGM x WGN waves, NS weight stages
#define ALT_DCONV(BM, BN, WGM, WGN, NS)                                                                          \
    const bool reg_dconv_##BM##x##BN##_w##WGM##x##WGN##_s##NS =                                                  \
        (igemm_register(IgemmLaunch{"bf16_" #BM "x" #BN "x64_direct_w" #WGM "x" #WGN "_s" #NS, ALT_BF16, BM, BN,  \
                                    64, LOAD_VEC, LOAD_VEC, NS - 1, 1, 0, nullptr,                               \
                                    &dconv_launch<BM, BN, WGM, WGN, 1, NS, 64>, WGM, WGN, 1}),                   \
         true)

// the same with KW K groups of WGM x WGN waves each and K steps of BK channels
#define ALT_DCONV_KW(BM, BN, WGM, WGN, KW, NS, BK)                                                               \
    const bool reg_dconv_##BM##x##BN##_w##WGM##x##WGN##x##KW##_s##NS##_b##BK =                                   \
        (igemm_register(IgemmLaunch{"bf16_" #BM "x" #BN "x" #BK "_direct_w" #WGM "x" #WGN "x" #KW "_s" #NS,       \
                                    ALT_BF16, BM, BN, BK, LOAD_VEC, LOAD_VEC, NS - 1, 1, 0, nullptr,             \
                                    &dconv_launch<BM, BN, WGM, WGN, KW, NS, BK>, WGM, WGN, KW}),                 \
         true)

// streaming kernel (dstream.h): BM x BN tile, KW K groups of WGM x WGN waves, NS stages of BK channels
#define ALT_DSTREAM(BM, BN, WGM, WGN, KW, NS, BK)                                                                \
    const bool reg_dstream_##BM##x##BN##x##BK##_w##WGM##x##WGN##x##KW##_s##NS =                                  \
        (igemm_register(IgemmLaunch{"bf16_" #BM "x" #BN "x" #BK "_stream_w" #WGM "x" #WGN "x" #KW "_s" #NS,       \
                                    ALT_BF16, BM, BN, BK, LOAD_VEC, LOAD_VEC, NS - 1, 1, 0, nullptr,             \
                                    &dstream_launch<BM, BN, WGM, WGN, KW, NS, BK>, WGM, WGN, KW, 1}),            \
         true)

// channel-planar kernel (dplanar.h): BM x BN tile, KW K groups of WGM x WGN waves
#define ALT_DPLANAR(BM, BN, WGM, WGN, KW)                                                                        \
    const bool reg_dplanar_##BM##x##BN##_w##WGM##x##WGN##x##KW =                                                 \
        (igemm_register(IgemmLaunch{"bf16_" #BM "x" #BN "x64_planar_w" #WGM "x" #WGN "x" #KW, ALT_BF16, BM, BN,   \
                                    64, LOAD_VEC, LOAD_VEC, 0, 0, 0, nullptr,                                    \
                                    &dplanar_launch<BM, BN, WGM, WGN, KW>, WGM, WGN, KW, 2}),                    \
         true)

// the streaming kernel for B stored [K][N] (row-major): the same tiles, B read through LDS transpose reads
#define ALT_DSTREAM_KN(BM, BN, WGM, WGN, KW, NS, BK)                                                             \
    const bool reg_dstream_kn_##BM##x##BN##x##BK##_w##WGM##x##WGN##x##KW##_s##NS =                               \
        (igemm_register(IgemmLaunch{"bf16_" #BM "x" #BN "x" #BK "_streamkn_w" #WGM "x" #WGN "x" #KW "_s" #NS,     \
                                    ALT_BF16, BM, BN, BK, LOAD_VEC, LOAD_VEC, NS - 1, 1, 0, nullptr,             \
                                    &dstream_launch<BM, BN, WGM, WGN, KW, NS, BK, true>, WGM, WGN, KW, 1, 1}),   \
         true)
