"""GPU parity of the 16-bit-input Gemm (IEEE half / bfloat16 inputs, fp32 accumulation) against the
CPU oracle evaluated on the fp32 values the 16-bit inputs denote."""
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


def test_gemm_16bit_full_size_sampled_rows(lib):
    """4096^3 in the configuration the benchmark times, checked on sampled rows."""
    announce("gemm_lp 4096 sampled")
    for kind in ("bf16", "f16"):
        c = workloads.gemm_case_16bit(4096, kind)
        A, B, C = bits_to_dev(c["A_bits"], kind), bits_to_dev(c["B_bits"], kind), torch.from_numpy(c["C"]).cuda()
        got = lib.onnx_gemm_lp(A, B, C, out_dtype=torch.float32)
        torch.cuda.synchronize()
        rows = np.array([0, 1, 255, 256, 257, 1023, 2048, 3071, 4094, 4095])
        ref, S = oracle.gemm(c["A"][rows], c["B"], c["C"], 1.0, 1.0, 0, 1, relu=False, want_scale=True)
        g = got[torch.from_numpy(rows).cuda()].cpu().numpy()
        assert rel_err(g, ref) <= REL_TOL
        assert within_rounding_bound(g, ref, S, 4096 + 2)


def test_gemm_16bit_errors(lib):
    announce("gemm_lp errors")
    a = torch.zeros((16, 16), dtype=torch.bfloat16, device="cuda")
    b = torch.zeros((16, 16), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(lib.OnnxHipError) as e:
        lib.onnx_gemm_lp(a, b, transB=0)
    assert e.value.status == 5
    with pytest.raises(lib.OnnxHipError) as e:
        lib.onnx_gemm_lp(torch.zeros((16, 12), dtype=torch.bfloat16, device="cuda"),
                         torch.zeros((16, 12), dtype=torch.bfloat16, device="cuda"))
    assert e.value.status == 5
    with pytest.raises(lib.OnnxHipError) as e:
        lib.onnx_gemm_lp(a, torch.zeros((16, 24), dtype=torch.bfloat16, device="cuda"))
    assert e.value.status == 3
    assert lib.onnx_gemm_lp(torch.zeros((0, 16), dtype=torch.float16, device="cuda"),
                            torch.zeros((8, 16), dtype=torch.float16, device="cuda")).shape == (0, 8)
