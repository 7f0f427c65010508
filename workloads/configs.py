"""Shapes of the synthetic workloads (stand-ins for the networks the paper
evaluates: ResNet-style convolution layers, BERT-base-style matrix products,
and the conversion operator on their activation tensors)."""

# Single small fp32 convolution (parity case the CPU oracle finishes at once).
SMALL_CONV = dict(N=1, C=16, H=14, W=14, K=16, R=3, S=3, stride=1, pad=1)

# ResNet-50-style layers, run at batch 1 and 16, bf16 in / fp32 accumulate.
RESNET_LAYERS = [
    dict(name="c64_56_3x3", C=64, H=56, W=56, K=64, R=3, S=3, stride=1, pad=1),
    dict(name="c128_28_3x3", C=128, H=28, W=28, K=128, R=3, S=3, stride=1, pad=1),
    dict(name="c256_14_3x3", C=256, H=14, W=14, K=256, R=3, S=3, stride=1, pad=1),
    dict(name="c512_7_3x3", C=512, H=7, W=7, K=512, R=3, S=3, stride=1, pad=1),
    dict(name="c256_56_1x1", C=256, H=56, W=56, K=64, R=1, S=1, stride=1, pad=0),
]

# Activation tensors the conversion operator is measured on (N, C, H, W).
TRANSFORM_SHAPES = [(16, 64, 56, 56), (16, 256, 14, 14), (64, 512, 7, 7)]

# BERT-base-shaped products: M = batch 16 x 128 tokens.
BERT_GEMMS = [
    dict(name="proj", batch=1, M=2048, K=768, N=768),
    dict(name="ffn_up", batch=1, M=2048, K=768, N=3072),
    dict(name="ffn_down", batch=1, M=2048, K=3072, N=768),
]
# Attention scores: 16 sequences x 12 heads, Q (128x64) times K^T (64x128).
BERT_QKT = dict(name="qkt", batch=192, M=128, K=64, N=128)

# Three-layer chain at N=16: conv3x3+bias+ReLU -> conv3x3 stride 2 -> conv1x1.
CHAIN_LAYERS = [
    dict(C=64, H=56, W=56, K=64, R=3, S=3, stride=1, pad=1, bias=True, relu=True),
    dict(C=64, H=56, W=56, K=128, R=3, S=3, stride=2, pad=1, bias=False, relu=False),
    dict(C=128, H=28, W=28, K=256, R=1, S=1, stride=1, pad=0, bias=False, relu=False),
]


def conv_out_hw(H, W, R, S, stride, pad, dil=1):
    oh = (H + 2 * pad - dil * (R - 1) - 1) // stride + 1
    ow = (W + 2 * pad - dil * (S - 1) - 1) // stride + 1
    return oh, ow


def conv_flops(N, C, H, W, K, R, S, stride, pad, **_):
    oh, ow = conv_out_hw(H, W, R, S, stride, pad)
    return 2 * N * K * oh * ow * C * R * S
