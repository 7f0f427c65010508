"""Seeded synthetic inputs and workload shapes shared by the tests, the smoke
check and the benchmark.  Nothing in here performs any of the method's
arithmetic (no layout index maps, no convolution, no matrix product): it only
draws numbers and lists shapes."""
from .inputs import (uniform_f32, normal_f32, small_ints_f32, f32_to_bf16_bits,
                     bf16_bits_to_f32, special_bit_patterns)
from .configs import (SMALL_CONV, RESNET_LAYERS, TRANSFORM_SHAPES, BERT_GEMMS,
                      BERT_QKT, CHAIN_LAYERS, conv_out_hw, conv_flops)
