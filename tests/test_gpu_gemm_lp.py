"""GPU parity of the 16-bit-input Gemm, MatMul and Conv (IEEE half / bfloat16 inputs, fp32
accumulation) against the CPU oracle evaluated on the fp32 values the 16-bit inputs denote."""
import numpy as np
import pytest

import oracle
import workloads
from util import REL_TOL, rel_err, within_rounding_bound

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TORCH_T = {"f16": torch.float16, "bf16": torch.bfloat16}
PRECISION = {"f16": 11, "bf16": 8}          # significand bits: round-to-nearest relative error <= 2^-p


@pytest.fixture(scope="module")
def lib():
    import paper_2008_08272_amd as p
    assert torch.cuda.is_available(), "these tests need the GPU"
    return p


def bits_to_dev(bits, kind):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(TORCH_T[kind])


def lp_to_host(t, kind):
    torch.cuda.synchronize()
    b = t.view(torch.int16).cpu().numpy().view(np.uint16)
    return workloads.from_bf16_bits(b) if kind == "bf16" else b.view(np.float16).astype(np.float32)


def announce(*what):
    print("CASE", *what, flush=True)


SHAPES = [(64, 64, 64), (32, 32, 8), (1, 1, 8), (130, 70, 96), (257, 383, 128), (512, 512, 1024), (1000, 1000, 40),
          (1, 1000, 2048), (32, 1000, 2048), (300, 520, 72), (768, 1280, 256), (1024, 1024, 1024)]


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_16bit_matches_oracle(lib, M, N, K, kind):
    announce("gemm_lp", kind, M, N, K)
    c = workloads.gemm_case_16bit(N, kind, m=M, k=K)
    A, B, C = bits_to_dev(c["A_bits"], kind), bits_to_dev(c["B_bits"], kind), torch.from_numpy(c["C"]).cuda()
    ref, S = oracle.gemm(c["A"], c["B"], c["C"], 1.0, 1.0, 0, 1, relu=False, want_scale=True)
    got = lib.onnx_gemm_lp(A, B, C, out_dtype=torch.float32)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    assert got.shape == ref.shape
    assert rel_err(got, ref) <= REL_TOL
    assert within_rounding_bound(got, ref, S, K + 2)
    # result stored in the inputs' type: the fp32 value rounded once more, to nearest
    ref2 = oracle.gemm(c["A"], c["B"], c["C"], 0.5, 2.0, 0, 1, relu=True)
    got2 = lp_to_host(lib.onnx_gemm_lp(A, B, C, alpha=0.5, beta=2.0, act=1), kind)
    u = 2.0 ** -PRECISION[kind]
    assert (np.abs(got2 - ref2) <= u * np.abs(ref2) + (K + 5) * 2.0 ** -24 * (0.5 * S + 2.0) + 1e-7).all()
    assert (got2 >= 0).all()


@pytest.mark.parametrize("kind", ["f16", "bf16"])
def test_gemm_16bit_small_integers_bit_exact(lib, kind):
    announce("gemm_lp integers", kind)
    rng = np.random.default_rng(21)
    for (M, N, K) in [(257, 130, 64), (512, 384, 256), (64, 1000, 8)]:
        a = rng.integers(-8, 9, (M, K)).astype(np.float32)        # exactly representable in both formats
        b = rng.integers(-8, 9, (N, K)).astype(np.float32)
        cb = rng.integers(-100, 100, (M, N)).astype(np.float32)   # full-matrix bias
        enc = (lambda x: workloads.to_bf16_bits(x)) if kind == "bf16" else (lambda x: x.astype(np.float16).view(np.uint16))
        A, B = bits_to_dev(enc(a), kind), bits_to_dev(enc(b), kind)
        ref = oracle.gemm(a, b, cb, 1.0, 1.0, 0, 1)
        got = lib.onnx_gemm_lp(A, B, torch.from_numpy(cb).cuda(), out_dtype=torch.float32)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), ref.astype(np.float32))
        # stored in 16 bits: exactly the nearest-even rounding of the exact result
        col = rng.integers(-3, 4, (M, 1)).astype(np.float32)       # per-row bias
        ref = oracle.gemm(a, b, col, 1.0, 1.0, 0, 1).astype(np.float32)
        want = workloads.from_bf16_bits(workloads.to_bf16_bits(ref)) if kind == "bf16" else ref.astype(np.float16).astype(np.float32)
        got = lp_to_host(lib.onnx_gemm_lp(A, B, torch.from_numpy(col).cuda()), kind)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("n", [2048, 4096])
def test_gemm_16bit_full_size_whole_output(lib, n, kind):
    """2048^3 and 4096^3 in the configuration the benchmark times, every output element compared."""
    announce("gemm_lp full", n, kind)
    c = workloads.gemm_case_16bit(n, kind)
    A, B, C = bits_to_dev(c["A_bits"], kind), bits_to_dev(c["B_bits"], kind), torch.from_numpy(c["C"]).cuda()
    got = lib.onnx_gemm_lp(A, B, C, out_dtype=torch.float32)
    torch.cuda.synchronize()
    want = "gemm_lp 256x256x64" if n == 4096 else "gemm_lp 128x128x64"
    assert lib.onnx_last_launch().startswith(want), lib.onnx_last_launch()
    ref, S = oracle.gemm(c["A"], c["B"], c["C"], 1.0, 1.0, 0, 1, relu=False, want_scale=True)
    g = got.cpu().numpy()
    assert rel_err(g, ref) <= REL_TOL
    assert within_rounding_bound(g, ref, S, n + 2)
    # the same launch with the result stored in the inputs' type
    got2 = lp_to_host(lib.onnx_gemm_lp(A, B, C), kind)
    assert lib.onnx_last_launch().startswith(want), lib.onnx_last_launch()
    u = 2.0 ** -PRECISION[kind]
    assert (np.abs(got2 - ref) <= u * np.abs(ref) + (n + 5) * 2.0 ** -24 * (S + 2.0) + 1e-7).all()


@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_matmul_16bit_large_whole_output(lib, kind):
    """B stored [K][N]: the 256 x 256 and 128 x 128 tiles with the row-contiguous loader in chunks of 8 and
    of 4 columns, every output element compared (4096 x 768 x 3072 is the shape the benchmark times)."""
    for (M, K, N, want, chunk) in ((4096, 512, 4096, "gemm_lp 256x256x64", 8), (4096, 768, 3072, "gemm_lp 128x128x64", 8),
                                   (4096, 136, 3844, "gemm_lp 256x256x64", 4), (2048, 136, 2052, "gemm_lp 128x128x64", 4)):
        announce("matmul_lp large", kind, M, K, N)
        rng = np.random.default_rng([M, K, N])
        ab, av = encode(rng.uniform(-1, 1, (M, K)).astype(np.float32), kind)
        bb, bv = encode(rng.uniform(-1, 1, (K, N)).astype(np.float32), kind)
        got = lib.onnx_matmul_lp(bits_to_dev(ab, kind), bits_to_dev(bb, kind), out_dtype=torch.float32)
        torch.cuda.synchronize()
        launch = lib.onnx_last_launch()
        assert launch.startswith(want) and "B=RC/%d" % chunk in launch, launch
        ref, S = oracle.matmul(av, bv, want_scale=True)
        g = got.cpu().numpy()
        assert rel_err(g, ref) <= REL_TOL
        assert within_rounding_bound(g, ref, S, K + 2)
        got2 = lp_to_host(lib.onnx_matmul_lp(bits_to_dev(ab, kind), bits_to_dev(bb, kind)), kind)
        u = 2.0 ** -PRECISION[kind]
        assert (np.abs(got2 - ref) <= u * np.abs(ref) + (K + 5) * 2.0 ** -24 * (S + 1.0) + 1e-7).all()


def encode(x, kind):
    """fp32 array -> (16-bit storage, the fp32 values it denotes)."""
    if kind == "bf16":
        b = workloads.to_bf16_bits(x)
        return b, workloads.from_bf16_bits(b)
    hh = x.astype(np.float16)
    return hh.view(np.uint16), hh.astype(np.float32)


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("transA,transB", [(0, 0), (1, 0), (1, 1), (0, 1)])
@pytest.mark.parametrize("M,N,K", [(70, 90, 50), (130, 257, 129), (64, 64, 32), (300, 200, 7), (1, 1, 1), (130, 264, 136),
                                   (70, 92, 48), (257, 200, 64)])
def test_gemm_16bit_every_layout_and_ragged_k(lib, M, N, K, transA, transB, kind):
    """The tuned kernel takes transA = 0 with K a multiple of 8 and B either K-contiguous (transB = 1)
    or row-contiguous with N a multiple of 4 (chunks of 8 columns when N is a multiple of 8, else
    of 4); every other layout, K and N goes through the general kernel."""
    announce("gemm_lp layouts", kind, M, N, K, transA, transB)
    rng = np.random.default_rng([M, N, K, transA, transB])
    ab, av = encode(rng.uniform(-1, 1, (K, M) if transA else (M, K)).astype(np.float32), kind)
    bb, bv = encode(rng.uniform(-1, 1, (N, K) if transB else (K, N)).astype(np.float32), kind)
    cshape = [(1, N), (M, 1), (M, N), (N,)][(M + K + transA) % 4]
    C = rng.uniform(-1, 1, cshape).astype(np.float32)
    ref, S = oracle.gemm(av, bv, C, 0.75, -1.25, transA, transB, relu=False, want_scale=True)
    got = lib.onnx_gemm_lp(bits_to_dev(ab, kind), bits_to_dev(bb, kind), torch.from_numpy(C).cuda(), alpha=0.75, beta=-1.25,
                           transA=transA, transB=transB, out_dtype=torch.float32)
    torch.cuda.synchronize()
    fast = transA == 0 and K % 8 == 0 and (transB == 1 or N % 4 == 0)
    launch = lib.onnx_last_launch()
    assert launch.startswith("gemm_lp" if fast else "lp_generic"), launch
    if fast:
        assert ("B=KC/8" if transB else "B=RC/%d" % (8 if N % 8 == 0 else 4)) in launch, launch
    g = got.cpu().numpy()
    assert rel_err(g, ref) <= REL_TOL
    assert within_rounding_bound(g, ref, S, K + 2)
    # stored in the inputs' type, with Relu
    ref2 = oracle.gemm(av, bv, C, 0.75, -1.25, transA, transB, relu=True)
    got2 = lp_to_host(lib.onnx_gemm_lp(bits_to_dev(ab, kind), bits_to_dev(bb, kind), torch.from_numpy(C).cuda(), alpha=0.75,
                                       beta=-1.25, transA=transA, transB=transB, act=1), kind)
    u = 2.0 ** -PRECISION[kind]
    assert (np.abs(got2 - ref2) <= u * np.abs(ref2) + (K + 5) * 2.0 ** -24 * (S + 2.0) + 1e-7).all()


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("sa,sb", [((5, 4), (4, 6)), ((3, 2, 50, 40), (2, 40, 60)), ((2, 70, 33), (3, 1, 33, 65)), ((40,), (40, 6)),
                                   ((50, 40), (40,)), ((2, 3, 130, 36), (36, 200)), ((8, 12, 128, 64), (8, 12, 64, 128)),
                                   ((4, 130, 72), (72, 264)), ((2, 3, 100, 64), (3, 64, 136)), ((2, 300, 48), (2, 48, 140))])
def test_matmul_16bit_matches_oracle(lib, sa, sb, kind):
    announce("matmul_lp", kind, sa, sb)
    rng = np.random.default_rng(len(sa) * 100 + len(sb))
    ab, av = encode(rng.uniform(-1, 1, sa).astype(np.float32), kind)
    bb, bv = encode(rng.uniform(-1, 1, sb).astype(np.float32), kind)
    ref, S = oracle.matmul(av, bv, want_scale=True)
    got = lib.onnx_matmul_lp(bits_to_dev(ab, kind), bits_to_dev(bb, kind), out_dtype=torch.float32)
    torch.cuda.synchronize()
    # the tuned kernel takes K a multiple of 8 with N a multiple of 4 (batch entries then start aligned)
    n_cols = sb[-1] if len(sb) > 1 else 1
    fast = len(sa) > 1 and sa[-1] % 8 == 0 and n_cols % 4 == 0
    launch = lib.onnx_last_launch()
    assert launch.startswith("gemm_lp" if fast else "lp_generic"), launch
    if fast:
        assert "B=RC/%d" % (8 if n_cols % 8 == 0 else 4) in launch, launch
    g = got.cpu().numpy()
    assert g.shape == ref.shape
    assert rel_err(g, ref) <= REL_TOL
    assert within_rounding_bound(g, ref, S, sa[-1] + 2)
    got2 = lp_to_host(lib.onnx_matmul_lp(bits_to_dev(ab, kind), bits_to_dev(bb, kind)), kind)
    u = 2.0 ** -PRECISION[kind]
    assert (np.abs(got2 - ref) <= u * np.abs(ref) + (sa[-1] + 5) * 2.0 ** -24 * (S + 1.0) + 1e-7).all()


@pytest.mark.parametrize("kind", ["f16", "bf16"])
def test_gemm_16bit_misaligned_operands(lib, kind):
    """Operands that do not start on a 16-byte boundary: the tuned kernel is taken only as far as its wide
    loads allow (B [K][N] 8 bytes off: chunks of 4 columns; A or a K-contiguous B off: the general kernel)."""
    announce("gemm_lp misaligned", kind)
    M, N, K = 96, 136, 72
    rng = np.random.default_rng(77)
    ab, av = encode(rng.uniform(-1, 1, (M, K)).astype(np.float32), kind)
    b0, b0v = encode(rng.uniform(-1, 1, (K, N)).astype(np.float32), kind)       # transB = 0
    b1, b1v = encode(rng.uniform(-1, 1, (N, K)).astype(np.float32), kind)       # transB = 1

    def shifted(bits, elems):
        flat = torch.zeros(bits.size + 16, dtype=torch.int16, device="cuda")
        flat[elems:elems + bits.size] = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16).ravel()).cuda()
        t = flat[elems:elems + bits.size].view(bits.shape).view(TORCH_T[kind])
        assert t.data_ptr() % 16 == (2 * elems) % 16
        return t

    for a_shift, b_shift, transB, want in ((0, 4, 0, "B=RC/4"), (0, 1, 0, "lp_generic"), (1, 0, 0, "lp_generic"), (0, 4, 1, "lp_generic"),
                                           (0, 0, 0, "B=RC/8"), (0, 0, 1, "B=KC/8")):
        A = shifted(ab, a_shift)
        Bt = shifted(b1 if transB else b0, b_shift)
        ref, S = oracle.gemm(av, b1v if transB else b0v, None, 1.0, 1.0, 0, transB, relu=False, want_scale=True)
        got = lib.onnx_gemm_lp(A, Bt, None, transA=0, transB=transB, out_dtype=torch.float32)
        torch.cuda.synchronize()
        assert want in lib.onnx_last_launch(), (a_shift, b_shift, transB, lib.onnx_last_launch())
        g = got.cpu().numpy()
        assert rel_err(g, ref) <= REL_TOL
        assert within_rounding_bound(g, ref, S, K + 2)


def test_16bit_tuned_kernel_random_sweep(lib):
    """Seeded random shapes through the row-contiguous loader of the tuned kernel: MatMul with batch
    broadcasting and 1x1 convolutions whose tiles span many small images, both types, both output types."""
    rng = np.random.default_rng(20080827)
    for it in range(36):
        kind = ("f16", "bf16")[it % 2]
        u = 2.0 ** -PRECISION[kind]
        if it % 3 != 2:
            M = int(rng.integers(1, 200)); K = 8 * int(rng.integers(1, 30)); N = 4 * int(rng.integers(1, 60))
            batch = [(), (3,), (2, 2)][int(rng.integers(0, 3))]
            sa = batch + (M, K)
            sb = [(K, N), batch + (K, N), batch[-1:] + (K, N)][int(rng.integers(0, 3))]
            announce("lp sweep matmul", it, kind, sa, sb)
            ab, av = encode(rng.uniform(-1, 1, sa).astype(np.float32), kind)
            bb, bv = encode(rng.uniform(-1, 1, sb).astype(np.float32), kind)
            ref, S = oracle.matmul(av, bv, want_scale=True)
            got = lib.onnx_matmul_lp(bits_to_dev(ab, kind), bits_to_dev(bb, kind), out_dtype=torch.float32)
            torch.cuda.synchronize()
            assert lib.onnx_last_launch().startswith("gemm_lp") and "B=RC/" in lib.onnx_last_launch(), lib.onnx_last_launch()
            g = got.cpu().numpy()
            assert g.shape == ref.shape and rel_err(g, ref) <= REL_TOL and within_rounding_bound(g, ref, S, K + 2)
            got2 = lp_to_host(lib.onnx_matmul_lp(bits_to_dev(ab, kind), bits_to_dev(bb, kind)), kind)
            assert (np.abs(got2 - ref) <= u * np.abs(ref) + (K + 5) * 2.0 ** -24 * (S + 1.0) + 1e-7).all()
        else:
            n = int(rng.integers(1, 40)); g_ = (1, 1, 2, 4)[int(rng.integers(0, 4))]
            C = 8 * g_ * int(rng.integers(1, 12)); Mo = g_ * int(rng.integers(1, 50))
            H, W = [(2, 2), (4, 4), (2, 6), (6, 6), (3, 4), (10, 10), (8, 5)][int(rng.integers(0, 7))]
            announce("lp sweep conv1x1", it, kind, n, C, H, W, Mo, g_)
            xb, xv = encode(rng.uniform(-1, 1, (n, C, H, W)).astype(np.float32), kind)
            wb, wv = encode(rng.uniform(-1, 1, (Mo, C // g_, 1, 1)).astype(np.float32), kind)
            Bv = rng.uniform(-1, 1, (Mo,)).astype(np.float32)
            rb, rv = encode(rng.uniform(-1, 1, (n, Mo, H, W)).astype(np.float32), kind)
            z4, o2 = (0, 0, 0, 0), (1, 1)
            ref, S = oracle.conv(xv, wv, Bv, z4, o2, o2, g_, want_scale=True)
            X, Wt = bits_to_dev(xb, kind), bits_to_dev(wb, kind)
            got = lib.onnx_conv_lp(X, Wt, torch.from_numpy(Bv).cuda(), z4, o2, o2, g_, out_dtype=torch.float32)
            torch.cuda.synchronize()
            assert lib.onnx_last_launch().startswith("gemm_lp") and "B=RC/" in lib.onnx_last_launch(), lib.onnx_last_launch()
            gth = got.cpu().numpy()
            K = C // g_
            assert rel_err(gth, ref) <= REL_TOL and within_rounding_bound(gth, ref, S, K + 1)
            ref2, S2 = oracle.conv(xv, wv, Bv, z4, o2, o2, g_, residual=rv, relu=False, want_scale=True)
            got2 = lp_to_host(lib.onnx_conv_lp(X, Wt, torch.from_numpy(Bv).cuda(), z4, o2, o2, g_, residual=bits_to_dev(rb, kind), act=1), kind)
            want = np.maximum(ref2, 0)
            assert (np.abs(got2 - want) <= u * np.abs(want) + (K + 5) * 2.0 ** -24 * (S2 + 1.0) + 1e-7).all()


CONV_LP_CASES = [
    # N, C, H, W, M, kH, kW, pads, strides, dilations, group
    (2, 16, 19, 23, 40, 3, 3, (1, 1, 1, 1), (1, 1), (1, 1), 1),
    (2, 3, 37, 41, 48, 7, 7, (3, 3, 3, 3), (2, 2), (1, 1), 1),            # 48 filters: not the stem kernel (64)
    (2, 32, 20, 20, 48, 3, 3, (2, 0, 1, 3), (2, 3), (2, 1), 2),
    (2, 64, 12, 12, 96, 1, 1, (0, 0, 0, 0), (1, 1), (1, 1), 1),          # pointwise: row-contiguous input, chunks of 8 positions
    (2, 64, 9, 7, 96, 1, 1, (0, 0, 0, 0), (1, 1), (1, 1), 1),            # pointwise, 63 positions per image: general kernel
    (5, 72, 14, 14, 200, 1, 1, (0, 0, 0, 0), (1, 1), (1, 1), 1),         # pointwise, 196 positions: chunks of 4, tiles span images
    (3, 64, 12, 12, 96, 1, 1, (0, 0, 0, 0), (1, 1), (1, 1), 2),          # pointwise with two groups
    (2, 36, 12, 12, 96, 1, 1, (0, 0, 0, 0), (1, 1), (1, 1), 1),          # pointwise, K = 36: general kernel
    (8, 64, 28, 28, 512, 1, 1, (0, 0, 0, 0), (1, 1), (1, 1), 1),         # pointwise, 196 tiles of 128 x 128
    (2, 64, 12, 12, 96, 1, 1, (0, 0, 0, 0), (2, 2), (1, 1), 1),          # strided 1x1
    (4, 6, 10, 10, 6, 3, 3, (1, 1, 1, 1), (1, 1), (1, 1), 6),            # depthwise
    (1, 1, 28, 28, 8, 5, 5, (2, 2, 2, 2), (1, 1), (1, 1), 1),
    (3, 128, 14, 14, 128, 3, 3, (1, 1, 1, 1), (1, 1), (1, 1), 1),        # K = 1152
]


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("case", CONV_LP_CASES)
def test_conv_16bit_matches_oracle(lib, case, kind):
    announce("conv_lp", kind, case)
    N, C, H, W, M, kH, kW, pads, st, dl, g = case
    rng = np.random.default_rng(list(case[:7]) + [g])
    xb, xv = encode(rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32), kind)
    wb, wv = encode(rng.uniform(-1, 1, (M, C // g, kH, kW)).astype(np.float32), kind)
    Bv = rng.uniform(-1, 1, (M,)).astype(np.float32)
    K = (C // g) * kH * kW
    ref, S = oracle.conv(xv, wv, Bv, pads, st, dl, g, want_scale=True)
    X, Wt = bits_to_dev(xb, kind), bits_to_dev(wb, kind)
    got = lib.onnx_conv_lp(X, Wt, torch.from_numpy(Bv).cuda(), pads, st, dl, g, out_dtype=torch.float32)
    torch.cuda.synchronize()
    # 1x1, stride 1, no padding, K a multiple of 8 and 4 | H*W: the tuned kernel on the input as a [C][H*W] matrix
    fast = kH == 1 and kW == 1 and st == (1, 1) and pads == (0, 0, 0, 0) and K % 8 == 0 and (H * W) % 4 == 0
    launch = lib.onnx_last_launch()
    assert launch.startswith("gemm_lp" if fast else "lp_generic"), launch
    if fast:
        assert "B=RC/%d" % (8 if (H * W) % 8 == 0 else 4) in launch, launch
    gth = got.cpu().numpy()
    assert gth.shape == ref.shape
    assert rel_err(gth, ref) <= REL_TOL
    assert within_rounding_bound(gth, ref, S, K + 1)
    # 16-bit result with a 16-bit residual and Relu: one more rounding on top of the fp32 result
    rb, rv = encode(rng.uniform(-1, 1, ref.shape).astype(np.float32), kind)
    ref2, S2 = oracle.conv(xv, wv, None, pads, st, dl, g, residual=rv, relu=False, want_scale=True)
    got2 = lp_to_host(lib.onnx_conv_lp(X, Wt, None, pads, st, dl, g, residual=bits_to_dev(rb, kind), act=1), kind)
    u = 2.0 ** -PRECISION[kind]
    want = np.maximum(ref2, 0)
    assert (np.abs(got2 - want) <= u * np.abs(want) + (K + 5) * 2.0 ** -24 * (S2 + 1.0) + 1e-7).all()
    assert (got2 >= 0).all()


CONV3X3_LP_CASES = [
    # N, C, H, W, M, pads, strides, dilations, group, expected "tile B=IM2COL/columns-per-unit npb"
    (2, 16, 7, 7, 40, (1, 1, 1, 1), (2, 1), (1, 1), 1, "64x64x144 1 2"),          # odd row length: one column per unit
    (2, 16, 7, 7, 40, (1, 1, 1, 1), (2, 1), (1, 3), 1, "64x64x144 1 4"),
    (2, 16, 7, 7, 40, (1, 1, 1, 1), (2, 2), (1, 3), 1, "64x64x144 1 8"),
    (2, 16, 12, 12, 40, (1, 1, 1, 1), (2, 1), (1, 1), 1, "64x64x144 2 1"),        # even row length: pairs of columns
    (2, 16, 14, 14, 40, (1, 1, 1, 1), (2, 2), (1, 3), 1, "64x64x144 2 2"),
    (2, 16, 12, 12, 40, (1, 1, 1, 1), (2, 2), (1, 3), 1, "64x64x144 2 4"),
    (3, 64, 19, 23, 72, (2, 0, 1, 3), (1, 1), (1, 1), 2, "64x64x144 1 2"),        # two groups, asymmetric pads, ragged M and N
    (3, 64, 18, 22, 72, (0, 2, 1, 1), (1, 2), (2, 1), 2, "64x64x144 2 2"),        # even left pad: no column shift
    (5, 32, 28, 28, 200, (1, 1, 1, 1), (1, 1), (1, 1), 1, "64x64x144 2 1"),       # tiles that span images
    (3, 128, 14, 14, 128, (1, 1, 1, 1), (1, 1), (1, 1), 1, "64x64x144 2 1"),      # K = 1152: eight steps
    (40, 16, 30, 31, 128, (1, 1, 1, 1), (1, 1), (1, 3), 1, "128x128x144 1 2"),    # enough tiles for the 128 x 128 tile
    (40, 16, 25, 51, 128, (1, 1, 1, 1), (2, 1), (2, 2), 1, "128x128x144 1 4"),
    (210, 16, 7, 7, 256, (1, 1, 1, 1), (1, 1), (1, 1), 1, "128x128x144 1 2"),     # tiles that span three or four images
    (160, 16, 10, 10, 256, (0, 0, 0, 0), (1, 1), (1, 1), 1, "128x128x144 2 1"),
    (40, 16, 20, 20, 256, (1, 1, 1, 1), (1, 1), (1, 3), 1, "128x128x144 2 1"),
    (40, 16, 24, 50, 128, (1, 1, 1, 1), (2, 1), (2, 2), 1, "128x128x144 2 2"),
    (70, 32, 14, 14, 300, (1, 1, 1, 1), (1, 1), (1, 1), 2, "64x128x144 2 2"),     # two groups of 150 filters: a ragged third row of tiles
    (2, 512, 7, 7, 72, (1, 1, 1, 1), (1, 1), (1, 1), 1, "64x64x144 1 2 split"),   # 4 tiles, 32 channel steps: K split, finishing kernel
    (1, 256, 50, 100, 128, (1, 1, 1, 1), (1, 1), (1, 1), 1, "128x128x144 2 2 split"),  # rows wider than 64: 40 tiles of 128 x 128, K split
    (700, 16, 9, 9, 40, (1, 1, 1, 1), (1, 1), (1, 1), 1, "64x128x144 1 2"),       # few filters, many positions: the 64 x 128 tile
    (80, 16, 30, 31, 40, (1, 1, 1, 1), (1, 1), (1, 1), 1, "64x128x144 1 4"),
    (80, 16, 25, 51, 40, (1, 1, 1, 1), (1, 1), (2, 2), 1, "64x128x144 1 8"),
    (1200, 16, 10, 10, 40, (0, 0, 0, 0), (1, 1), (1, 1), 1, "64x128x144 2 1"),
    (80, 16, 24, 50, 40, (1, 1, 1, 1), (1, 1), (2, 2), 1, "64x128x144 2 4"),
]


@pytest.fixture(autouse=True)
def no_inherited_workspace(lib):
    """The workspace is one process-wide setting (a GraphRunner of an earlier test file may have left its own):
    the tests here start without one, so that the kernel each of them expects is the one that runs."""
    lib.onnx_set_workspace(None)
    yield


@pytest.fixture
def lp_workspace(lib, no_inherited_workspace):
    ws = torch.empty(16 << 20, dtype=torch.uint8, device="cuda")
    lib.onnx_set_workspace(ws)
    try:
        yield ws
    finally:
        torch.cuda.synchronize()
        lib.onnx_set_workspace(None)


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("case", CONV3X3_LP_CASES)
def test_conv3x3_16bit_lds_patch_matches_oracle(lib, lp_workspace, case, kind):
    """With a workspace (it holds the rewritten filter bank) 3x3 convolutions whose channel count per group is
    a multiple of 16 run the LDS-patch kernel: every instance, against the oracle."""
    N, C, H, W, M, pads, st, dl, g, expect = case
    announce("conv_lp 3x3", kind, case)
    rng = np.random.default_rng([N, C, H, W, M, g])
    xb, xv = encode(rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32), kind)
    wb, wv = encode(rng.uniform(-1, 1, (M, C // g, 3, 3)).astype(np.float32), kind)
    Bv = rng.uniform(-1, 1, (M,)).astype(np.float32)
    K = (C // g) * 9
    ref, S = oracle.conv(xv, wv, Bv, pads, st, dl, g, want_scale=True)
    X, Wt = bits_to_dev(xb, kind), bits_to_dev(wb, kind)
    got = lib.onnx_conv_lp(X, Wt, torch.from_numpy(Bv).cuda(), pads, st, dl, g, out_dtype=torch.float32)
    torch.cuda.synchronize()
    tile, cols, npb = expect.split()[:3]
    launch = lib.onnx_last_launch()
    assert launch.startswith("conv_window_lp " + tile) and "B=IM2COL/%s npb=%s " % (cols, npb) in launch, launch
    assert ("ksplit=1 " not in launch) == expect.endswith("split"), launch
    gth = got.cpu().numpy()
    assert gth.shape == ref.shape
    assert rel_err(gth, ref) <= REL_TOL
    assert within_rounding_bound(gth, ref, S, K + 1)
    # 16-bit result with a 16-bit residual and Relu: one more rounding on top of the fp32 result
    rb, rv = encode(rng.uniform(-1, 1, ref.shape).astype(np.float32), kind)
    ref2, S2 = oracle.conv(xv, wv, None, pads, st, dl, g, residual=rv, relu=False, want_scale=True)
    got2 = lp_to_host(lib.onnx_conv_lp(X, Wt, None, pads, st, dl, g, residual=bits_to_dev(rb, kind), act=1), kind)
    assert lib.onnx_last_launch().startswith("conv_window_lp " + tile)
    u = 2.0 ** -PRECISION[kind]
    want = np.maximum(ref2, 0)
    assert (np.abs(got2 - want) <= u * np.abs(want) + (K + 5) * 2.0 ** -24 * (S2 + 1.0) + 1e-7).all()
    assert (got2 >= 0).all()
    # small integers: every product and partial sum exact, so the bits must agree
    Xi = rng.integers(-4, 5, (N, C, H, W)).astype(np.float32)
    Wi = rng.integers(-4, 5, (M, C // g, 3, 3)).astype(np.float32)
    refi = oracle.conv(Xi, Wi, None, pads, st, dl, g)
    goti = lib.onnx_conv_lp(bits_to_dev(encode(Xi, kind)[0], kind), bits_to_dev(encode(Wi, kind)[0], kind), None, pads, st, dl, g,
                            out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert np.array_equal(goti.cpu().numpy().astype(np.float64), refi)


def test_conv3x3_16bit_lds_patch_operands_off_alignment(lib, lp_workspace):
    """X two bytes off a 4-byte boundary: single-column loads although the rows have even length.  W at any
    2-byte offset: the filter bank is rewritten with 2-byte loads.  Same results."""
    announce("conv_lp 3x3 misaligned")
    rng = np.random.default_rng(5)
    N, C, H, W, M = 3, 32, 12, 12, 72
    pads, st, dl = (1, 1, 1, 1), (1, 1), (1, 1)
    for kind in ("f16", "bf16"):
        xb, xv = encode(rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32), kind)
        wb, wv = encode(rng.uniform(-1, 1, (M, C, 3, 3)).astype(np.float32), kind)
        ref, S = oracle.conv(xv, wv, None, pads, st, dl, 1, want_scale=True)
        for x_off, w_off, cols in ((1, 0, 1), (0, 1, 2), (1, 3, 1), (2, 8, 2)):
            def shifted(bits, off):
                flat = bits_to_dev(bits, kind).reshape(-1)
                buf = torch.empty(flat.numel() + 16, dtype=flat.dtype, device="cuda")
                buf[off:off + flat.numel()].copy_(flat)
                return buf[off:off + flat.numel()].view(bits.shape)
            X, Wt = shifted(xb, x_off), shifted(wb, w_off)
            assert X.data_ptr() % 4 == (2 * x_off) % 4 and Wt.data_ptr() % 16 == (2 * w_off) % 16
            got = lib.onnx_conv_lp(X, Wt, None, pads, st, dl, 1, out_dtype=torch.float32)
            torch.cuda.synchronize()
            launch = lib.onnx_last_launch()
            assert launch.startswith("conv_window_lp 64x64x144") and "B=IM2COL/%d " % cols in launch, launch
            gth = got.cpu().numpy()
            assert rel_err(gth, ref) <= REL_TOL and within_rounding_bound(gth, ref, S, C * 9 + 1)


STEM_LP_CASES = [
    # N, H, W, runs the stem kernel
    (2, 32, 32, True),        # 16 x 16 outputs: one tile of 16 rows per image
    (1, 224, 224, True),      # ResNet50's: 112 x 112 outputs, tiles of two rows
    (3, 30, 34, True),        # 15 x 17 outputs: rows that end inside a wavefront, a last tile with fewer rows
    (2, 17, 23, True),        # odd extents: the last window column lies past the image
    (1, 9, 300, True),        # 150 outputs per row: one row per tile, five wavefronts, three idle
    (1, 20, 80, True),        # 40 outputs per row: patch rows of two 64-column pieces
    (2, 12, 150, True),       # 75 outputs per row: three pieces
    (1, 7, 520, False),       # 260 outputs per row: more than a tile holds, the general kernel
]


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("case", STEM_LP_CASES)
def test_conv_stem_16bit_matches_oracle(lib, case, kind):
    """The 7x7 stride-2 convolution of 3 channels into 64 feature maps (ResNet50's first layer, Section 4.2) on 16-bit
    tensors: its own kernel, with and without bias and Relu, fp32 and 16-bit results; other 7x7 shapes keep the
    general kernel."""
    N, H, W, stem = case
    announce("conv_lp stem", kind, case)
    rng = np.random.default_rng([N, H, W])
    pads, st, dl = (3, 3, 3, 3), (2, 2), (1, 1)
    xb, xv = encode(rng.uniform(-1, 1, (N, 3, H, W)).astype(np.float32), kind)
    wb, wv = encode(rng.uniform(-1, 1, (64, 3, 7, 7)).astype(np.float32), kind)
    Bv = rng.uniform(-1, 1, (64,)).astype(np.float32)
    K = 147
    X, Wt = bits_to_dev(xb, kind), bits_to_dev(wb, kind)
    family = "conv_stem_lp" if stem else "lp_generic"
    ref, S = oracle.conv(xv, wv, Bv, pads, st, dl, 1, want_scale=True)
    got = lib.onnx_conv_lp(X, Wt, torch.from_numpy(Bv).cuda(), pads, st, dl, 1, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert lib.onnx_last_launch().startswith(family), lib.onnx_last_launch()
    gth = got.cpu().numpy()
    assert gth.shape == ref.shape
    assert rel_err(gth, ref) <= REL_TOL
    assert within_rounding_bound(gth, ref, S, K + 1)
    # 16-bit result, no bias, Relu
    ref2, S2 = oracle.conv(xv, wv, None, pads, st, dl, 1, relu=False, want_scale=True)
    got2 = lp_to_host(lib.onnx_conv_lp(X, Wt, None, pads, st, dl, 1, act=1), kind)
    assert lib.onnx_last_launch().startswith(family)
    u = 2.0 ** -PRECISION[kind]
    want = np.maximum(ref2, 0)
    assert (np.abs(got2 - want) <= u * np.abs(want) + (K + 5) * 2.0 ** -24 * (S2 + 1.0) + 1e-7).all()
    assert (got2 >= 0).all()
    # small integers: every product and partial sum exact, so the bits must agree; an infinity in one pixel must reach
    # exactly the windows that contain it (the zero taps that pad K see neighbouring pixels)
    Xi = rng.integers(-4, 5, (N, 3, H, W)).astype(np.float32)
    Wi = rng.integers(-4, 5, (64, 3, 7, 7)).astype(np.float32)
    refi = oracle.conv(Xi, Wi, None, pads, st, dl, 1)
    Xd, Wd = bits_to_dev(encode(Xi, kind)[0], kind), bits_to_dev(encode(Wi, kind)[0], kind)
    goti = lib.onnx_conv_lp(Xd, Wd, None, pads, st, dl, 1, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert np.array_equal(goti.cpu().numpy().astype(np.float64), refi)
    Wpos = np.abs(Wi) + 1
    Xinf = Xi.copy()
    Xinf[0, 1, H // 2, W // 2] = np.inf
    gotf = lib.onnx_conv_lp(bits_to_dev(encode(Xinf, kind)[0], kind), bits_to_dev(encode(Wpos, kind)[0], kind), None, pads, st, dl, 1,
                            out_dtype=torch.float32).cpu().numpy()
    hit = np.zeros(gotf.shape[2:], dtype=bool)
    for oh in range(gotf.shape[2]):
        for ow in range(gotf.shape[3]):
            hit[oh, ow] = 0 <= H // 2 - (2 * oh - 3) < 7 and 0 <= W // 2 - (2 * ow - 3) < 7
    assert np.isposinf(gotf[0][:, hit]).all() and np.isfinite(gotf[0][:, ~hit]).all() and np.isfinite(gotf[1:]).all()
    # a residual, another filter count or other pads: not this kernel
    res = torch.zeros(got.shape, dtype=TORCH_T[kind], device="cuda")
    lib.onnx_conv_lp(X, Wt, None, pads, st, dl, 1, residual=res)
    assert lib.onnx_last_launch().startswith("lp_generic")
    lib.onnx_conv_lp(X, Wt[:32].contiguous(), None, pads, st, dl, 1)
    assert lib.onnx_last_launch().startswith("lp_generic")
    if H >= 9:
        lib.onnx_conv_lp(X, Wt, None, (2, 3, 3, 3), st, dl, 1)
        assert lib.onnx_last_launch().startswith("lp_generic")
    torch.cuda.synchronize()


CONV1X1_LAYOUT_CASES = [
    # N, C, H, W, M, strides, group, expected B loader of the tuned kernel
    (3, 64, 12, 12, 96, (2, 2), 1, "B=RC/4"),       # strided: the 6 x 6 positions it reads are copied, then chunks of 4 columns
    (2, 32, 17, 16, 40, (1, 2), 1, "B=RC/8"),       # stride along the row only: 17 x 8 positions, chunks of 8
    (5, 64, 14, 14, 200, (2, 2), 2, "B=KC/8"),      # strided into 7 x 7 = 49 positions: copied, then one row per position; two groups
    (4, 128, 7, 7, 130, (1, 1), 1, "B=KC/8"),       # pointwise on 49 positions per image
    (2, 72, 9, 7, 96, (1, 1), 3, "B=KC/8"),         # 63 positions, three groups of 24 channels
    (33, 256, 7, 7, 512, (1, 1), 1, "B=KC/8"),      # several 128 x 128 tiles, each spanning three images
    (3, 24, 13, 11, 20, (3, 2), 1, "B=KC/8"),       # strided into 5 x 6 = 30 positions
]


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("case", CONV1X1_LAYOUT_CASES)
def test_conv1x1_16bit_through_layout_passes(lib, lp_workspace, case, kind):
    """With a workspace, 1x1 convolutions the tuned kernel cannot read in place go through it after a layout pass:
    strided ones on a dense copy of the positions they read, planes without aligned column chunks as one
    K-contiguous row per position."""
    N, C, H, W, M, st, g, loader = case
    announce("conv_lp 1x1 layouts", kind, case)
    rng = np.random.default_rng([N, C, H, W, M, g])
    xb, xv = encode(rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32), kind)
    wb, wv = encode(rng.uniform(-1, 1, (M, C // g, 1, 1)).astype(np.float32), kind)
    Bv = rng.uniform(-1, 1, (M,)).astype(np.float32)
    z4, o2 = (0, 0, 0, 0), (1, 1)
    K = C // g
    ref, S = oracle.conv(xv, wv, Bv, z4, st, o2, g, want_scale=True)
    X, Wt = bits_to_dev(xb, kind), bits_to_dev(wb, kind)
    got = lib.onnx_conv_lp(X, Wt, torch.from_numpy(Bv).cuda(), z4, st, o2, g, out_dtype=torch.float32)
    torch.cuda.synchronize()
    launch = lib.onnx_last_launch()
    assert launch.startswith("gemm_lp") and loader in launch, launch
    gth = got.cpu().numpy()
    assert gth.shape == ref.shape
    assert rel_err(gth, ref) <= REL_TOL and within_rounding_bound(gth, ref, S, K + 1)
    rb, rv = encode(rng.uniform(-1, 1, ref.shape).astype(np.float32), kind)
    ref2, S2 = oracle.conv(xv, wv, None, z4, st, o2, g, residual=rv, relu=False, want_scale=True)
    got2 = lp_to_host(lib.onnx_conv_lp(X, Wt, None, z4, st, o2, g, residual=bits_to_dev(rb, kind), act=1), kind)
    u = 2.0 ** -PRECISION[kind]
    want = np.maximum(ref2, 0)
    assert (np.abs(got2 - want) <= u * np.abs(want) + (K + 5) * 2.0 ** -24 * (S2 + 1.0) + 1e-7).all()
    Xi = rng.integers(-4, 5, (N, C, H, W)).astype(np.float32)
    Wi = rng.integers(-4, 5, (M, C // g, 1, 1)).astype(np.float32)
    goti = lib.onnx_conv_lp(bits_to_dev(encode(Xi, kind)[0], kind), bits_to_dev(encode(Wi, kind)[0], kind), None, z4, st, o2, g,
                            out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert np.array_equal(goti.cpu().numpy().astype(np.float64), oracle.conv(Xi, Wi, None, z4, st, o2, g))


def test_conv3x3_16bit_filters_rewritten_once(lib):
    """onnx_conv_lp_filter_taps + onnx_conv_lp_taps: the filter bank rewritten once, no workspace; bit for bit the
    result of onnx_conv_lp with a workspace (same kernel, same operands), and within the budget of the oracle."""
    announce("conv_lp taps")
    rng = np.random.default_rng(21)
    for kind in ("f16", "bf16"):
        for (N, C, H, W, M, pads, st, dl, g) in [(3, 64, 19, 23, 72, (2, 0, 1, 3), (1, 1), (1, 1), 2), (40, 16, 20, 20, 256, (1, 1, 1, 1), (1, 1), (1, 3), 1),
                                                 (2, 32, 14, 14, 40, (1, 1, 1, 1), (2, 2), (1, 1), 1)]:
            xb, xv = encode(rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32), kind)
            wb, wv = encode(rng.uniform(-1, 1, (M, C // g, 3, 3)).astype(np.float32), kind)
            Bv = rng.uniform(-1, 1, (M,)).astype(np.float32)
            X, Wt, Bd = bits_to_dev(xb, kind), bits_to_dev(wb, kind), torch.from_numpy(Bv).cuda()
            taps = lib.onnx_conv_lp_filter_taps(Wt)
            got = lib.onnx_conv_lp_taps(X, taps, Bd, pads, st, dl, g, act=1)
            torch.cuda.synchronize()
            assert lib.onnx_last_launch().startswith("conv_window_lp"), lib.onnx_last_launch()
            ws = torch.empty(16 << 20, dtype=torch.uint8, device="cuda")
            lib.onnx_set_workspace(ws)
            try:
                same = lib.onnx_conv_lp(X, Wt, Bd, pads, st, dl, g, act=1)
                torch.cuda.synchronize()
            finally:
                lib.onnx_set_workspace(None)
            assert torch.equal(got.view(torch.int16), same.view(torch.int16))
            ref, S = oracle.conv(xv, wv, Bv, pads, st, dl, g, relu=False, want_scale=True)
            want = np.maximum(ref, 0)
            u = 2.0 ** -PRECISION[kind]
            assert (np.abs(lp_to_host(got, kind) - want) <= u * np.abs(want) + (C // g * 9 + 5) * 2.0 ** -24 * (S + 1.0) + 1e-7).all()
    # shapes the kernel does not take are refused before any launch
    x = torch.zeros((1, 16, 300, 300), dtype=torch.bfloat16, device="cuda")            # rows longer than the widest tile
    w = torch.zeros((8, 16, 3, 3), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(lib.OnnxHipError) as e:
        lib.onnx_conv_lp_taps(x, lib.onnx_conv_lp_filter_taps(w), None, (1, 1, 1, 1))
    assert e.value.status == 5
    with pytest.raises(lib.OnnxHipError):
        lib.onnx_conv_lp_filter_taps(torch.zeros((8, 24, 3, 3), dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(lib.OnnxHipError):
        lib.onnx_conv_lp_filter_taps(torch.zeros((8, 16, 5, 5), dtype=torch.bfloat16, device="cuda"))


@pytest.mark.parametrize("kind", ["f16", "bf16"])
def test_16bit_split_k_with_a_workspace(lib, lp_workspace, kind):
    """Few tiles and a long K: with a workspace the 64 x 64 tile of the tuned kernel splits its K range over several
    workgroups per tile and a finishing kernel adds the shares; Gemm (both B layouts), MatMul and a 1x1 convolution,
    fp32 and 16-bit results."""
    announce("lp split k", kind)
    rng = np.random.default_rng(31)
    u = 2.0 ** -PRECISION[kind]
    for (M, N, K, transB) in [(64, 64, 4096, 1), (130, 70, 2048, 1), (200, 136, 1024, 0), (33, 260, 1536, 0)]:
        ab, av = encode(rng.uniform(-1, 1, (M, K)).astype(np.float32), kind)
        bb, bv = encode(rng.uniform(-1, 1, (N, K) if transB else (K, N)).astype(np.float32), kind)
        Cv = rng.uniform(-1, 1, (1, N)).astype(np.float32)
        A, Bm, C = bits_to_dev(ab, kind), bits_to_dev(bb, kind), torch.from_numpy(Cv).cuda()
        ref, S = oracle.gemm(av, bv, Cv, 1.0, 1.0, 0, transB, relu=False, want_scale=True)
        got = lib.onnx_gemm_lp(A, Bm, C, transB=transB, out_dtype=torch.float32)
        torch.cuda.synchronize()
        launch = lib.onnx_last_launch()
        assert launch.startswith("gemm_lp 64x64") and "ksplit=1 " not in launch, launch
        g = got.cpu().numpy()
        assert rel_err(g, ref) <= REL_TOL and within_rounding_bound(g, ref, S, K + 2)
        got2 = lp_to_host(lib.onnx_gemm_lp(A, Bm, C, transB=transB, act=1), kind)
        assert "ksplit=1 " not in lib.onnx_last_launch()
        want = np.maximum(ref, 0)
        assert (np.abs(got2 - want) <= u * np.abs(want) + (K + 5) * 2.0 ** -24 * (S + 1.0) + 1e-7).all()
    # MatMul with a batch, small integers: every partial sum exact, so the shares must add up bit for bit
    a = rng.integers(-4, 5, (3, 70, 1024)).astype(np.float32)
    b = rng.integers(-4, 5, (1024, 72)).astype(np.float32)
    got = lib.onnx_matmul_lp(bits_to_dev(encode(a, kind)[0], kind), bits_to_dev(encode(b, kind)[0], kind), out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert "ksplit=1 " not in lib.onnx_last_launch(), lib.onnx_last_launch()
    assert np.array_equal(got.cpu().numpy().astype(np.float64), oracle.matmul(a, b))
    # 1x1 convolution on one image with a residual: 16-bit result from the finishing kernel
    xb, xv = encode(rng.uniform(-1, 1, (1, 1024, 14, 14)).astype(np.float32), kind)
    wb, wv = encode(rng.uniform(-1, 1, (256, 1024, 1, 1)).astype(np.float32), kind)
    rb, rv = encode(rng.uniform(-1, 1, (1, 256, 14, 14)).astype(np.float32), kind)
    z4, o2 = (0, 0, 0, 0), (1, 1)
    ref, S = oracle.conv(xv, wv, None, z4, o2, o2, 1, residual=rv, relu=False, want_scale=True)
    got = lp_to_host(lib.onnx_conv_lp(bits_to_dev(xb, kind), bits_to_dev(wb, kind), None, z4, o2, o2, 1, residual=bits_to_dev(rb, kind), act=1), kind)
    assert "ksplit=1 " not in lib.onnx_last_launch(), lib.onnx_last_launch()
    want = np.maximum(ref, 0)
    assert (np.abs(got - want) <= u * np.abs(want) + (1024 + 5) * 2.0 ** -24 * (S + 1.0) + 1e-7).all()


def test_conv3x3_16bit_workspace_too_small_or_channels_not_16(lib, lp_workspace):
    """The LDS-patch kernel needs room for the rewritten filter bank and 16 | channels per group; otherwise the
    general kernel runs, with the same result up to summation order."""
    announce("conv_lp 3x3 fallbacks")
    rng = np.random.default_rng(77)
    for C, M in ((24, 32), (64, 1024 * 16)):
        N, H, W = (2, 10, 10) if C == 24 else (1, 4, 4)
        xb, xv = encode(rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32), "bf16")
        wb, wv = encode(rng.uniform(-1, 1, (M, C, 3, 3)).astype(np.float32), "bf16")
        ref, S = oracle.conv(xv, wv, None, (1, 1, 1, 1), (1, 1), (1, 1), 1, want_scale=True)
        got = lib.onnx_conv_lp(bits_to_dev(xb, "bf16"), bits_to_dev(wb, "bf16"), None, (1, 1, 1, 1), (1, 1), (1, 1), 1,
                               out_dtype=torch.float32)
        torch.cuda.synchronize()
        # 24 channels; 16384 x 64 x 9 values = 18 MiB of filters against a 16 MiB workspace
        assert lib.onnx_last_launch().startswith("lp_generic"), lib.onnx_last_launch()
        gth = got.cpu().numpy()
        assert rel_err(gth, ref) <= REL_TOL and within_rounding_bound(gth, ref, S, C * 9 + 1)


def test_conv_16bit_small_integers_bit_exact(lib):
    announce("conv_lp integers")
    rng = np.random.default_rng(8)
    X = rng.integers(-4, 5, (3, 48, 17, 19)).astype(np.float32)
    Wt = rng.integers(-4, 5, (72, 48, 3, 3)).astype(np.float32)
    Bv = rng.integers(-4, 5, (72,)).astype(np.float32)
    for kind in ("f16", "bf16"):
        xb, _ = encode(X, kind)
        wb, _ = encode(Wt, kind)
        for pads, st, dl in [((1, 1, 1, 1), (1, 1), (1, 1)), ((0, 2, 1, 0), (2, 1), (1, 2))]:
            ref = oracle.conv(X, Wt, Bv, pads, st, dl)
            got = lib.onnx_conv_lp(bits_to_dev(xb, kind), bits_to_dev(wb, kind), torch.from_numpy(Bv).cuda(), pads, st, dl,
                                   out_dtype=torch.float32)
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy().astype(np.float64), ref)


POOL_LP_CASES = [
    # N, C, H, W, kernel, pads, strides, dilations, ceil_mode
    (2, 3, 9, 8, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0),
    (1, 2, 10, 7, (2, 3), (0, 1, 0, 1), (2, 1), (1, 1), 0),
    (2, 2, 11, 11, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 1),
    (1, 3, 12, 9, (3, 2), (0, 0, 0, 0), (3, 2), (2, 2), 0),
    (2, 5, 13, 10, (3, 2), (2, 0, 1, 1), (1, 2), (1, 1), 0),
    (3, 64, 56, 56, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0),      # 3 columns, stride 2, left pad 1, rows of 56: four outputs per thread
    (1, 2, 9, 10, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0),        # the same with an odd number of output columns
    (2, 4, 17, 24, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0),       # rows a multiple of 8 long: four outputs per thread from 16-byte loads
    (1, 3, 10, 16, (2, 3), (0, 1, 0, 1), (1, 2), (1, 1), 0),       # the same with two rows per window at vertical stride 1
    (1, 2, 11, 16, (3, 3), (2, 1, 2, 1), (3, 2), (2, 1), 0),       # the same with vertical dilation, stride 3 and pads of 2
    (2, 2, 9, 20, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0),        # rows of 20: even but not a multiple of 8, two outputs per thread
    (1, 2, 12, 10, (2, 3), (0, 1, 0, 1), (1, 2), (1, 1), 0),       # two rows per window, vertical stride 1
    (2, 2, 9, 12, (3, 3), (1, 1, 0, 0), (2, 2), (1, 1), 1),        # ceil_mode: a last window past the row, one output per thread
    (4, 1, 1, 1, (1, 1), (0, 0, 0, 0), (1, 1), (1, 1), 0),
    (5, 13, 7, 7, (2, 2), (0, 0, 0, 0), (1, 1), (1, 1), 0),        # 65 planes of 49 values: the global mean takes eight planes per wavefront, one left over
    (4, 16, 8, 8, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0),        # 64 planes of 64 values
    (0, 3, 8, 8, (2, 2), (0, 0, 0, 0), (2, 2), (1, 1), 0),
]


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("case", POOL_LP_CASES)
def test_pools_16bit_match_oracle(lib, case, kind):
    """MaxPool on 16-bit tensors returns one of its inputs: bit-exact against the oracle on the values the bits
    denote.  AveragePool sums in fp32 and rounds once: within one rounding of the type of the oracle's fp64 mean."""
    N, C, H, W, k, pads, st, dl, ceil = case
    announce("pool_lp", kind, case)
    rng = np.random.default_rng([N, C, H, W, k[0], k[1]])
    xb, xv = encode(rng.uniform(-2, 2, (N, C, H, W)).astype(np.float32), kind)
    X = bits_to_dev(xb, kind) if N else torch.empty((0, C, H, W), dtype=TORCH_T[kind], device="cuda")
    got = lib.onnx_maxpool_lp(X, k, pads, st, dl, ceil)
    assert got.dtype == TORCH_T[kind]
    if N == 0:
        assert got.shape[0] == 0
        return
    ref = oracle.maxpool(xv, k, pads, st, dl, ceil, want_indices=False)
    assert np.array_equal(lp_to_host(got, kind), ref)
    # the same tensor two bytes off a 4-byte boundary (no 4-byte loads then)
    buf = torch.empty(X.numel() + 8, dtype=X.dtype, device="cuda")
    buf[1:1 + X.numel()].copy_(X.reshape(-1))
    assert np.array_equal(lp_to_host(lib.onnx_maxpool_lp(buf[1:1 + X.numel()].view(X.shape), k, pads, st, dl, ceil), kind), ref)
    u = 2.0 ** -PRECISION[kind]
    if dl == (1, 1):
        for cip in (0, 1):
            want = oracle.avgpool(xv, k, pads, st, ceil, cip)
            g = lp_to_host(lib.onnx_avgpool_lp(X, k, pads, st, ceil, cip), kind)
            assert g.shape == want.shape
            # one rounding to the type plus the fp32 sum of at most k0*k1 values of magnitude <= 2
            assert (np.abs(g - want) <= u * np.abs(want) + k[0] * k[1] * 2.0 ** -22).all()
    want = oracle.avgpool(xv, None)
    g = lp_to_host(lib.onnx_avgpool_lp(X), kind)
    assert g.shape == (N, C, 1, 1)
    assert (np.abs(g - want) <= u * np.abs(want) + H * W * 2.0 ** -22).all()


@pytest.mark.parametrize("kind", ["f16", "bf16"])
def test_leakyrelu_16bit_bit_exact(lib, kind):
    """LeakyRelu on 16-bit tensors (the paper's operator definition lists F16): x >= 0 keeps its bits, otherwise the
    fp32 product alpha * x rounded to the type.  Both sides round the same way, so kept elements agree bit for bit and
    products value for value (a zero product may carry either sign): 16-byte and element-wise forms, special values,
    and through the runner's 16-bit mode behind a convolution."""
    announce("leakyrelu_lp", kind)
    rng = np.random.default_rng(17)
    special = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-40, -1e-40, -6e-8, 6e-8, -65504.0, 65504.0, -1.0, 1.0], dtype=np.float32)
    for count, off in ((8192, 0), (8200, 0), (1003, 0), (8192, 1), (13, 0), (0, 0)):
        x = rng.standard_normal(count).astype(np.float32) * 3
        x[:min(count, special.size)] = special[:min(count, special.size)]
        xb, xv = encode(x, kind)
        buf = torch.empty(count + 16, dtype=TORCH_T[kind], device="cuda")
        X = buf[off:off + count]
        if count:
            X.copy_(bits_to_dev(xb, kind))
        for alpha in (0.0, 0.01, 0.3, -1.5):
            got = lib.onnx_leakyrelu_lp(X, alpha)
            torch.cuda.synchronize()
            assert got.dtype == TORCH_T[kind] and got.shape == (count,)
            if count == 0:
                continue
            with np.errstate(all="ignore"):
                want64 = np.where(xv.astype(np.float64) >= 0.0, xv.astype(np.float64), float(np.float32(alpha)) * xv.astype(np.float64))
                _, wv = encode(want64.astype(np.float32), kind)
            gb = got.view(torch.int16).cpu().numpy().view(np.uint16)
            gv = lp_to_host(got, kind)
            keep = xv >= 0                                  # kept elements carry the input's bits
            nan = np.isnan(xv)
            assert np.array_equal(gb[keep], xb[keep]), (count, off, alpha)
            # the products: equal values (a zero product may carry either sign)
            assert np.array_equal(gv[~keep & ~nan], wv[~keep & ~nan], equal_nan=True), (count, off, alpha)
            assert np.isnan(gv[nan]).all()
    # through the runner: Conv -> LeakyRelu -> Relu on 16-bit tensors
    from paper_2008_08272_amd.runner import GraphRunner
    conv = dict(op="conv", x="x", w="w", b="b", pads=(1, 1, 1, 1), strides=(1, 1), dilations=(1, 1), group=1, residual=None,
                relu=False, y="c")
    m = dict(inputs={"x": rng.standard_normal((2, 16, 9, 9)).astype(np.float32)},
             weights={"w": (rng.standard_normal((24, 16, 3, 3)) * 0.1).astype(np.float32), "b": rng.standard_normal(24).astype(np.float32)},
             graph=[conv, dict(op="leakyrelu", x="c", alpha=0.2, y="l"), dict(op="relu", x="l", y="r")], output="r")
    r = GraphRunner(m, dtype=TORCH_T[kind])
    r.run()
    torch.cuda.synchronize()
    c = r.t["c"].float().cpu().numpy().astype(np.float64)
    want_l = encode(np.where(c >= 0, c, float(np.float32(0.2)) * c).astype(np.float32), kind)[1]
    assert np.array_equal(r.t["l"].float().cpu().numpy(), want_l)
    assert np.array_equal(r.t["r"].float().cpu().numpy(), np.maximum(want_l, 0))
    with pytest.raises(NotImplementedError):
        GraphRunner(dict(m, graph=[conv, dict(op="batchnorm", x="c", y="r")]), dtype=TORCH_T[kind])


ADD_LP_CASES = [((4, 24, 14, 16), (4, 24, 14, 16), 0), ((4, 24, 14, 16), (24, 1, 1), 0), ((2, 3, 7, 40), (40,), 0), ((5, 1, 48), (1, 9, 1), 0),
                ((3, 5, 7), (3, 5, 7), 0), ((6, 33), (1,), 0), ((6, 32), (6, 1), 0), ((2, 16, 8), (2, 16, 8), 1), ((4, 8), (8,), 3),
                ((1,), (7, 3, 8), 0), ((0, 5), (5,), 0), ((2, 2, 2, 2, 2, 3, 8), (2, 1, 2, 1, 2, 1, 8), 0)]


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("sa,sb,off", ADD_LP_CASES)
def test_add_abs_16bit_bit_exact(lib, sa, sb, off, kind):
    """Add on 16-bit tensors (Section 3's running example in the type Section 3.1 also lists): the fp32 sum of two 16-bit
    values rounded to the type is the correctly rounded sum, so the result equals the oracle's value for value (zeros
    with their sign, NaN where infinities cancel): same-shape, per-channel, row, column, scalar and two-sided
    broadcasts, element-wise forms for misaligned views and short rows, an empty tensor.  Abs: the sign bit cleared."""
    announce("add_lp", kind, sa, sb, off)
    from oracle import elementwise as ew
    rng = np.random.default_rng(abs(hash((sa, sb, off))) % 1000)
    special = np.array([0.0, -0.0, np.inf, -np.inf, 65504.0, -65504.0, 6e-8, -6e-8, 1e-40, 40000.0, 40000.0, 1.0], dtype=np.float32)

    def operand(shape):
        n = int(np.prod(shape))
        x = (rng.standard_normal(n) * 10.0 ** rng.integers(-3, 3, n)).astype(np.float32)
        k = min(n, special.size)
        x[:k] = rng.permutation(special)[:k]
        bits, vals = encode(x, kind)
        buf = torch.empty(n + 16, dtype=TORCH_T[kind], device="cuda")
        t = buf[off:off + n]
        if n:
            t.copy_(bits_to_dev(bits, kind))
        return t.view(shape), vals.reshape(shape).astype(np.float64)

    A, av = operand(sa)
    B, bv = operand(sb)
    got = lib.onnx_add_lp(A, B)
    torch.cuda.synchronize()
    with np.errstate(all="ignore"):
        want = ew.add_16bit(av, bv, kind)
    assert got.dtype == TORCH_T[kind] and tuple(got.shape) == want.shape
    g = lp_to_host(got, kind).astype(np.float64).reshape(want.shape)
    assert np.array_equal(g, want, equal_nan=True)
    assert np.array_equal(np.signbit(g)[want == 0], np.signbit(want)[want == 0])
    # Abs of the first operand: the same bits without the sign
    ab = lib.onnx_abs_lp(A)
    torch.cuda.synchronize()
    assert np.array_equal(ab.view(torch.int16).cpu().numpy().view(np.uint16), A.contiguous().view(torch.int16).cpu().numpy().view(np.uint16) & 0x7fff)
    assert np.array_equal(lp_to_host(ab, kind).astype(np.float64), ew.absolute(av.astype(np.float32)), equal_nan=True)


def test_add_abs_16bit_errors_and_runner(lib):
    announce("add_lp errors and runner nodes")
    x = torch.zeros((4, 8), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(TypeError):
        lib.onnx_add_lp(x, x.half())
    with pytest.raises(lib.OnnxHipError):
        lib.onnx_add_lp(x, torch.zeros((3,), dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(lib.OnnxHipError):
        lib.onnx_add_lp(x, x, out=x)                               # the result may not overlap an input
    with pytest.raises(lib.OnnxHipError):
        lib.onnx_abs_lp(x, out=x)
    # through the runner's 16-bit mode: Conv -> Add (with the input, unfused) -> Abs
    from oracle import elementwise as ew
    from paper_2008_08272_amd.runner import GraphRunner
    rng = np.random.default_rng(5)
    conv = dict(op="conv", x="x", w="w", b="b", pads=(1, 1, 1, 1), strides=(1, 1), dilations=(1, 1), group=1, residual=None,
                relu=False, y="c")
    m = dict(inputs={"x": rng.standard_normal((2, 16, 9, 9)).astype(np.float32)},
             weights={"w": (rng.standard_normal((16, 16, 3, 3)) * 0.1).astype(np.float32), "b": rng.standard_normal(16).astype(np.float32)},
             graph=[conv, dict(op="add", a="c", b="x", y="s"), dict(op="abs", x="s", y="r")], output="r")
    for kind in ("f16", "bf16"):
        r = GraphRunner(m, dtype=TORCH_T[kind])
        r.run()
        torch.cuda.synchronize()
        c, xin = r.t["c"].double().cpu().numpy(), r.t["x"].double().cpu().numpy()
        want = ew.add_16bit(c, xin, kind)
        assert np.array_equal(r.t["s"].double().cpu().numpy(), want)
        assert np.array_equal(r.t["r"].double().cpu().numpy(), np.abs(want))


REDUCE_LP_CASES = [((4, 6, 10, 12), [2, 3], 1), ((4, 6, 10, 12), [1], 0), ((3, 70000), [1], 1), ((5, 7, 9), None, 0), ((64, 33), [0], 1),
                   ((9, 1, 40), [0, 2], 0), ((2, 100003), [1], 0), ((3, 5, 4099), [2], 1), ((0, 4), [0], 0), ((1, 300000), None, 1)]


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("use_ws", [False, True])
@pytest.mark.parametrize("shape,axes,keep", REDUCE_LP_CASES)
def test_reducesum_16bit_matches_oracle(lib, shape, axes, keep, use_ws, kind):
    """ReduceSum on 16-bit tensors: fp32 partial sums in an unspecified order, one rounding to the type at the end.
    Small integers (every partial sum exact, the result a value of the type) must come out exactly; for random data
    the result is within (count + 2) 2^-24 sum|x| of the exact sum, plus half a unit of the type in the last place."""
    announce("reducesum_lp", kind, shape, axes, keep, use_ws)
    from oracle import elementwise as ew
    ws = torch.empty(8 << 20, dtype=torch.uint8, device="cuda") if use_ws else None
    lib.onnx_set_workspace(ws)
    try:
        rng = np.random.default_rng(31)
        u = 2.0 ** -11 if kind == "f16" else 2.0 ** -8
        tiny = 2.0 ** -25 if kind == "f16" else 2.0 ** -134
        n = int(np.prod(shape))
        # values in {-1, 0, 1}: partial sums are small integers, and so is every result for the short sums; the long ones
        # are bounded by the tolerance test below
        x = rng.integers(-1, 2, shape).astype(np.float32)
        bits, vals = encode(x, kind)
        X = bits_to_dev(bits.reshape(-1), kind).view(shape) if n else torch.empty(shape, dtype=TORCH_T[kind], device="cuda")
        Y = lib.onnx_reducesum_lp(X, axes, keep)
        ref = ew.reducesum(vals, axes, keep)
        assert tuple(Y.shape) == ref.shape and Y.dtype == TORCH_T[kind]
        got = lp_to_host(Y.reshape(-1), kind).astype(np.float64).reshape(ref.shape)
        assert np.array_equal(got, ew.round_to_16bit(ref, kind))
        if n == 0:
            return
        x = (rng.standard_normal(shape) * 4).astype(np.float32)
        bits, vals = encode(x, kind)
        X = bits_to_dev(bits.reshape(-1), kind).view(shape)
        got = lp_to_host(lib.onnx_reducesum_lp(X, axes, keep).reshape(-1), kind).astype(np.float64)
        ref = ew.reducesum(vals, axes, keep).reshape(-1)
        scale = ew.reducel1(vals, axes, keep).reshape(-1)
        count = n // max(ref.size, 1)
        assert (np.abs(got - ref) <= (count + 2) * 2.0 ** -24 * scale * (1 + u) + u * np.abs(ref) + tiny).all()
    finally:
        torch.cuda.synchronize()
        lib.onnx_set_workspace(None)


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("shape,axis", [((1, 5), 1), ((32, 1000), 1), ((32, 1000), 0), ((7, 1025), -1), ((3, 5000), 1), ((4, 9, 6), 1),
                                        ((2, 3, 4, 5), 2), ((513,), 0), ((6, 1), 1), ((0, 7), 1)])
def test_softmax_16bit_matches_oracle(lib, shape, axis, kind):
    """Softmax on 16-bit tensors: the fp32 kernel's arithmetic on the 16-bit values (the bound of the fp32 test), then one
    rounding to the type."""
    announce("softmax_lp", kind, shape, axis)
    from oracle import elementwise as ew
    rng = np.random.default_rng(32)
    u = 2.0 ** -11 if kind == "f16" else 2.0 ** -8
    tiny = 2.0 ** -25 if kind == "f16" else 2.0 ** -134
    for scale in (1.0, 8.0):
        x = (rng.standard_normal(shape) * scale).astype(np.float32)
        bits, vals = encode(x, kind)
        if x.size == 0:
            assert lib.onnx_softmax_lp(torch.empty(shape, dtype=TORCH_T[kind], device="cuda"), axis).shape == shape
            continue
        X = bits_to_dev(bits.reshape(-1), kind).view(shape)
        got = lp_to_host(lib.onnx_softmax_lp(X, axis), kind).astype(np.float64)
        ref = ew.softmax(vals, axis)
        assert got.shape == ref.shape
        depth = np.abs(vals.astype(np.float64) - vals.astype(np.float64).max(axis=axis, keepdims=True))
        assert (np.abs(got - ref) <= ((depth * 2.0 ** -23 + 4e-6) * (1 + u) + u) * ref + tiny).all()
    big = bits_to_dev(encode(np.array([1000.0, 1000.0, -1000.0], np.float32), kind)[0], kind).view(1, 3)
    assert lp_to_host(lib.onnx_softmax_lp(big, 1), kind).tolist() == [[0.5, 0.5, 0.0]]
    with pytest.raises(lib.OnnxHipError):
        lib.onnx_softmax_lp(big, 2)
    with pytest.raises(lib.OnnxHipError):
        lib.onnx_reducesum_lp(big, [3])


def test_pools_16bit_errors(lib):
    announce("pool_lp errors")
    import ctypes
    B = lib
    x = torch.zeros((1, 1, 4, 4), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(TypeError):
        lib.onnx_maxpool_lp(torch.zeros((1, 1, 4, 4), device="cuda"), (2, 2))
    with pytest.raises(lib.OnnxHipError):
        lib.onnx_maxpool_lp(x, (2, 2), pads=(2, 2, 2, 2))           # pads as large as the window
    with pytest.raises(lib.OnnxHipError):
        lib.onnx_avgpool_lp(x, (5, 5))                              # window larger than the image
    y = torch.zeros((1, 1, 2, 2), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(lib.OnnxHipError):
        lib.onnx_maxpool_lp(x, (2, 2), out=y)                       # y_dims do not match the inferred shape


@pytest.mark.parametrize("kind", ["f16", "bf16"])
def test_resnet50_16bit_every_layer_from_its_own_inputs(lib, kind):
    """ResNet-50 through the runner in a 16-bit type (batch 2: tiles span both images).  Every node is checked as
    an operator: the oracle gets the very tensors the node read on the GPU (16-bit activations and weights decoded,
    fp32 biases) and the node's result must lie within the operator's budget of the fp64 value: exact for MaxPool,
    one rounding of the type plus the fp32 accumulation bound otherwise.  The fp32 logits are also compared with
    the fp32 network's, as a sanity bound on what 54 roundings of the activations add up to."""
    announce("resnet50 16-bit", kind)
    from paper_2008_08272_amd.runner import GraphRunner
    from oracle import chain
    m = workloads.resnet50(2)
    r = GraphRunner(m, dtype=TORCH_T[kind])
    out = r.run()
    torch.cuda.synchronize()
    assert out.dtype == torch.float32 and out.shape == (2, 1000)
    u = 2.0 ** -PRECISION[kind]
    val = lambda name: r.t[name].float().cpu().numpy()
    tuned3x3 = 0
    for nd in m["graph"]:
        op = nd["op"]
        if op == "reshape":
            continue
        got = val(nd["y"]).astype(np.float64)
        last = nd["y"] == m["output"]
        ulp = 0.0 if last else u
        if op == "conv":
            x, w = val(nd["x"]), val(nd["w"])
            res = val(nd["residual"]) if nd["residual"] else None
            ref, S = oracle.conv(x, w, val(nd["b"]) if nd["b"] else None, nd["pads"], nd["strides"], nd["dilations"], nd["group"],
                                 residual=res, relu=False, want_scale=True)
            if nd["relu"]:
                ref = np.maximum(ref, 0)
            K = w.shape[1] * w.shape[2] * w.shape[3]
            bound = ulp * np.abs(ref) + (K + 5) * 2.0 ** -24 * (S + 1.0) + 1e-7
        elif op == "gemm":
            a, b = val(nd["a"]), val(nd["b"])
            ref, S = oracle.gemm(a, b, val(nd["c"]) if nd["c"] else None, nd["alpha"], nd["beta"], nd["transA"], nd["transB"],
                                 relu=nd["relu"], want_scale=True)
            bound = ulp * np.abs(ref) + (a.shape[1] + 5) * 2.0 ** -24 * (S + 1.0) + 1e-7
        elif op == "maxpool":
            ref = oracle.maxpool(val(nd["x"]), nd["kernel"], nd["pads"], nd["strides"], nd["dilations"], nd["ceil_mode"],
                                 want_indices=False).astype(np.float64)
            bound = np.zeros_like(ref)
        else:
            assert op == "avgpool"
            x = val(nd["x"])
            ref = oracle.avgpool(x, nd["kernel"], nd["pads"], nd["strides"], nd["ceil_mode"], nd["count_include_pad"])
            bound = u * np.abs(ref) + x.shape[2] * x.shape[3] * 2.0 ** -22 * np.abs(x).max()
        assert got.shape == ref.shape, nd["y"]
        assert (np.abs(got - ref) <= bound).all(), (nd["y"], op, float(np.abs(got - ref).max()))
    _, exact = chain.run(m, keep=())
    e = rel_err(out.cpu().numpy(), exact["logits"])
    print("resnet50 %s logits against the fp32 network: %.4f" % (kind, e), flush=True)
    assert e <= (0.1 if kind == "bf16" else 0.02)


def test_gemm_16bit_errors(lib):
    announce("gemm_lp errors")
    a = torch.zeros((16, 16), dtype=torch.bfloat16, device="cuda")
    b = torch.zeros((16, 16), dtype=torch.bfloat16, device="cuda")
    assert lib.onnx_gemm_lp(a, b, transB=0).shape == (16, 16)            # every layout is taken
    assert lib.onnx_gemm_lp(torch.zeros((16, 12), dtype=torch.bfloat16, device="cuda"),
                            torch.zeros((16, 12), dtype=torch.bfloat16, device="cuda")).shape == (16, 16)
    with pytest.raises(lib.OnnxHipError) as e:
        lib.onnx_gemm_lp(a, torch.zeros((16, 24), dtype=torch.bfloat16, device="cuda"))
    assert e.value.status == 3
    assert lib.onnx_gemm_lp(torch.zeros((0, 16), dtype=torch.float16, device="cuda"),
                            torch.zeros((8, 16), dtype=torch.float16, device="cuda")).shape == (0, 8)
