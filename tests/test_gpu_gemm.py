"""GPU parity: alt_gemm against the oracle's triple loop."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_12415_amd as alt
from workloads import BERT_GEMMS, BERT_QKT, f32_to_bf16_bits, normal_f32, small_ints_f32

from gpu_util import TOL, applicable_variants, canary_dev, canary_ok, dev, from_layout, host, rel_err, to_layout

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def h():
    return alt.Handle()


def run_gemm(h, A, B, al, bl, cl, in_dtype, out_dtype=alt.F32, variant=-1):
    """A (batch,M,K), B (batch,K,N) logical.  Returns logical (batch,M,N)."""
    batch, M, K = A.shape
    N = B.shape[2]
    d = alt.gemm_desc(M, N, K, batch=batch, in_dtype=in_dtype, out_dtype=out_dtype, variant=variant,
                      a_layout="MK->" + al, b_layout="KN->" + bl, c_layout="MN->" + cl)
    Ap = np.concatenate([to_layout(A[b], "MK", al) for b in range(batch)])
    Bp = np.concatenate([to_layout(B[b], "KN", bl) for b in range(batch)])
    cdt = np.float32 if out_dtype == alt.F32 else np.uint16
    whole, Cd = canary_dev(batch * M * N, cdt)
    ws_bytes = 36 * batch * M * N * 4
    ws = torch.empty(ws_bytes // 4, dtype=torch.float32, device="cuda")
    h.gemm(d, dev(Ap), dev(Bp), Cd, workspace=ws, ws_bytes=ws_bytes)
    got = host(Cd, cdt)
    assert canary_ok(whole, batch * M * N)
    return np.stack([from_layout(got[b * M * N:(b + 1) * M * N], (M, N), "MN", cl) for b in range(batch)]), d


GEMM_LAYOUTS = [("MK", "KN", "MN"), ("MK", "NK", "MN"), ("KM", "KN", "MN"), ("KM", "NK", "NM"),
                ("MK32m16k", "NK32n16k", "MN"), ("MK", "KN16k32n", "MN16m8n"), ("MK", "NK64n32k", "MN")]


@pytest.mark.parametrize("layouts", GEMM_LAYOUTS)
@pytest.mark.parametrize("in_dtype", [alt.BF16, alt.F32])
def test_exact_integers_every_variant(h, layouts, in_dtype):
    al, bl, cl = layouts
    batch, M, K, N = 2, 160, 96, 192
    A = small_ints_f32(61, (batch, M, K))
    B = small_ints_f32(62, (batch, K, N))
    ref = oracle.gemm(A, B)
    if in_dtype == alt.BF16:
        A, B = f32_to_bf16_bits(A), f32_to_bf16_bits(B)
    d0 = alt.gemm_desc(M, N, K, batch=batch, in_dtype=in_dtype, a_layout="MK->" + al, b_layout="KN->" + bl,
                       c_layout="MN->" + cl)
    variants = applicable_variants(h, d0, "gemm")
    assert variants
    for v, name in variants:
        got, _ = run_gemm(h, A, B, al, bl, cl, in_dtype, variant=v)
        assert np.array_equal(got, ref), name


@pytest.mark.parametrize("shape", [(2, 160, 256, 192), (1, 300, 768, 200), (3, 128, 64, 128), (1, 70, 1536, 36),
                                   (1, 70, 1536, 40), (2, 260, 320, 264)],
                         ids=lambda s: "b%d_%dx%dx%d" % s)
@pytest.mark.parametrize("bl", ["NK", "KN"])
def test_streaming_kernels_exact_integers(h, shape, bl):
    """The streaming kernels (A as MK, B as NK or, read through LDS transpose reads, as KN; K a multiple of
    64): every tile shape, K-group count and split factor, bit for bit; batched, ragged M and N, deep K."""
    batch, M, K, N = shape
    if bl == "KN" and N % 8:
        pytest.skip("row-major B is loaded eight columns at a time")
    A = small_ints_f32(71, (batch, M, K), -3, 3)
    B = small_ints_f32(72, (batch, K, N), -3, 3)
    ref = oracle.gemm(A, B)
    Ab, Bb = f32_to_bf16_bits(A), f32_to_bf16_bits(B)
    d0 = alt.gemm_desc(M, N, K, batch=batch, in_dtype=alt.BF16, a_layout="MK->MK", b_layout="KN->" + bl, c_layout="MN->MN")
    variants = [(v, n) for v, n in applicable_variants(h, d0, "gemm") if "stream" in n]
    assert all(("streamkn" in n) == (bl == "KN") for _, n in variants)
    assert len(variants) >= 6, "streaming kernels should cover this case"
    assert batch > 1 or K < 128 or any(not n.endswith("_k1") for _, n in variants)
    for v, name in variants:
        print(name, flush=True)
        got, _ = run_gemm(h, Ab, Bb, "MK", bl, "MN", alt.BF16, variant=v)
        assert np.array_equal(got, ref), name
    picks = [variants[0], variants[-1]] + [vn for vn in variants if not vn[1].endswith("_k1")][:2]
    for v, name in picks:
        got16, _ = run_gemm(h, Ab, Bb, "MK", bl, "MN", alt.BF16, out_dtype=alt.BF16, variant=v)
        assert np.array_equal(got16[0], f32_to_bf16_bits(ref[0])), name


def test_ragged_sizes(h):
    for (M, K, N) in [(1, 8, 8), (37, 40, 24), (130, 72, 200), (64, 4608, 64)]:
        A = small_ints_f32(63, (1, M, K), -2, 2)
        B = small_ints_f32(64, (1, K, N), -2, 2)
        ref = oracle.gemm(A, B)
        for al, bl in [("MK", "KN"), ("MK", "NK")]:
            got, _ = run_gemm(h, f32_to_bf16_bits(A), f32_to_bf16_bits(B), al, bl, "MN", alt.BF16)
            assert np.array_equal(got, ref), (M, K, N, al, bl)
    # K not a multiple of 8: only the gather loaders can run it
    A = small_ints_f32(65, (1, 20, 13))
    B = small_ints_f32(66, (1, 13, 9))
    got, _ = run_gemm(h, f32_to_bf16_bits(A), f32_to_bf16_bits(B), "MK", "KN", "MN", alt.BF16)
    assert np.array_equal(got, oracle.gemm(A, B))


def test_tolerance_fp32_and_bf16_out(h):
    A = normal_f32(67, (1, 256, 768), std=0.02)
    B = normal_f32(68, (1, 768, 192), std=0.02)
    ref = oracle.gemm(A, B)
    got, _ = run_gemm(h, A, B, "MK", "KN", "MN", alt.F32)
    assert rel_err(got, ref) <= TOL[alt.F32]
    Ab, Bb = f32_to_bf16_bits(A), f32_to_bf16_bits(B)
    ref = oracle.gemm(Ab, Bb)
    got, _ = run_gemm(h, Ab, Bb, "MK", "NK", "MN", alt.BF16)
    assert rel_err(got, ref) <= 1e-4
    got16, _ = run_gemm(h, Ab, Bb, "MK", "NK", "MN", alt.BF16, out_dtype=alt.BF16)
    ref16 = oracle.gemm(Ab, Bb, out_bf16=True)
    diff = np.abs(got16.astype(np.int32) - ref16.astype(np.int32))
    assert diff.max() <= 1 and (diff != 0).mean() < 0.02


@pytest.mark.parametrize("g", BERT_GEMMS + [BERT_QKT], ids=[g["name"] for g in BERT_GEMMS + [BERT_QKT]])
def test_bert_shapes_sampled(h, g):
    batch, M, K, N = g["batch"], g["M"], g["K"], g["N"]
    A = f32_to_bf16_bits(normal_f32(0xA17 + 4, (batch, M, K), std=0.02))
    B = f32_to_bf16_bits(normal_f32(0xA17 + 104, (batch, K, N), std=0.02))
    rng = np.random.RandomState(9)
    flat = np.unique(np.concatenate([rng.randint(0, batch * M * N, 3000), [0, batch * M * N - 1]]))
    ref = oracle.gemm_at(A, B, flat)
    rms = float(np.sqrt(np.mean(ref * ref)))
    for bl in ["KN", "NK"]:
        d = alt.gemm_desc(M, N, K, batch=batch, b_layout="KN->" + bl)
        Bp = B if bl == "KN" else np.ascontiguousarray(B.transpose(0, 2, 1))
        Cd = torch.empty(batch * M * N, dtype=torch.float32, device="cuda")
        ws_bytes = h.gemm_workspace_size(d)
        ws = torch.empty(max(ws_bytes, 4) // 4, dtype=torch.float32, device="cuda")
        h.gemm(d, dev(A.reshape(-1)), dev(Bp.reshape(-1)), Cd, workspace=ws, ws_bytes=ws_bytes)
        got = host(Cd, np.float32)[flat].astype(np.float64)
        err = float(np.max(np.abs(got - ref) / (np.abs(ref) + rms)))
        assert err <= 1e-4, (bl, err)


@pytest.mark.parametrize("b_layout", ["NK", "KN"])
def test_operand_of_2_gib_and_more(h, b_layout):
    """Maximum sizes: A just over 2 GiB (1,050,000 x 1024 bf16), beyond the 32-bit buffer offsets of the fast
    loaders: the product must still be the oracle's, bit for bit on integers, on sampled rows that include
    both ends of A and the rows around the 2 GiB boundary."""
    M, K, N = 1050000, 1024, 64
    assert M * K * 2 > 2 ** 31
    lut = f32_to_bf16_bits(np.array([-3, -2, -1, 0, 1, 2, 3, 0], dtype=np.float32))      # a hash of the offset picks the value
    A = np.empty(M * K, dtype=np.uint16)
    step = 1 << 26
    for a in range(0, M * K, step):
        e = min(M * K, a + step)
        i = np.arange(a, e, dtype=np.uint32)
        A[a:e] = lut[((i * np.uint32(2654435761)) >> np.uint32(13)) & np.uint32(7)]
    A = A.reshape(M, K)
    B = f32_to_bf16_bits(small_ints_f32(1401, (K, N), -3, 3))
    d = alt.gemm_desc(M, N, K, in_dtype=alt.BF16, out_dtype=alt.F32, a_layout="MK->MK", b_layout="KN->" + b_layout, c_layout="MN->MN")
    whole, Cd = canary_dev(M * N, np.float32)
    h.gemm(d, torch.from_numpy(A.reshape(-1).view(np.int16)).cuda(), dev(to_layout(B, "KN", b_layout)), Cd)
    torch.cuda.synchronize()
    assert canary_ok(whole, M * N)
    rng = np.random.default_rng(1402)
    rows = np.unique(np.concatenate([np.arange(0, 300), np.arange(M - 300, M), np.arange(2 ** 20 - 150, 2 ** 20 + 150),
                                     rng.integers(0, M, 1500)]))
    ref = oracle.gemm(A[rows], B)
    got = Cd.view(M, N)[torch.from_numpy(rows).cuda()].cpu().numpy()
    assert np.array_equal(got, ref)



@pytest.mark.parametrize("bl", ["NK", "KN"])
def test_streaming_kernels_every_step_count(h, bl):
    """Every number of K steps from 1 to 12, and 16, 17, 24 (whole and partial rounds over rings of 3 to 8 stages,
    with and without K groups and split-K), on every streaming variant: the fragment reads of these kernels
    complete behind the compiler's back, and a register copy the compiler places at a branch while such a
    read is in flight would show as a wrong sum for exactly some step counts."""
    M, N = 96, 136
    for steps in list(range(1, 13)) + [16, 17, 24]:
        K = 64 * steps
        A = small_ints_f32(131 + steps, (1, M, K), -3, 3)
        B = small_ints_f32(231 + steps, (1, K, N), -3, 3)
        ref = oracle.gemm(A, B)
        Ab, Bb = f32_to_bf16_bits(A), f32_to_bf16_bits(B)
        d0 = alt.gemm_desc(M, N, K, in_dtype=alt.BF16, a_layout="MK->MK", b_layout="KN->" + bl, c_layout="MN->MN")
        variants = [(v, n) for v, n in applicable_variants(h, d0, "gemm") if "stream" in n]
        assert len(variants) >= 9
        for v, name in variants:
            got, _ = run_gemm(h, Ab, Bb, "MK", bl, "MN", alt.BF16, variant=v)
            assert np.array_equal(got, ref), (name, steps)
