"""GPU parity of the single-launch chain (onnx_chain: a linear chain of Conv / pool / Gemm operators
run by one workgroup per image with everything in LDS) against the CPU oracle applied operator by
operator.  Every operator's result is requested (its Y pointer set), so each layer is compared,
not only the last.  Floating outputs: rel. error <= 1e-4 against the fp64 oracle; MaxPool of exact
inputs and small-integer data: bit-exact.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from util import REL_TOL, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2008_08272_amd as p
    assert torch.cuda.is_available(), "these tests need the GPU"
    return p


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def oracle_chain(X, ops):
    """The chain by the operators' definitions, one oracle call per operator, each fed the fp32
    rounding of its predecessor's exact result (what the device hands on is fp32 too)."""
    outs = []
    cur = np.asarray(X, dtype=np.float32)
    for o in ops:
        k = o["op"]
        if k == "conv":
            y = oracle.conv(cur, o["W"], o.get("B"), o.get("pads", (0, 0, 0, 0)), o.get("strides", (1, 1)),
                            o.get("dilations", (1, 1)), 1, relu=bool(o.get("act", 0)))
        elif k == "maxpool":
            y = oracle.maxpool(cur, o["kernel"], o.get("pads", (0, 0, 0, 0)), o.get("strides", (1, 1)),
                               o.get("dilations", (1, 1)), o.get("ceil_mode", 0), want_indices=False)
        elif k == "avgpool":
            y = oracle.avgpool(cur, o.get("kernel"), o.get("pads", (0, 0, 0, 0)), o.get("strides", (1, 1)),
                               o.get("ceil_mode", 0), o.get("count_include_pad", 0))
        else:
            flat = cur.reshape(cur.shape[0], -1)
            y = oracle.gemm(flat, o["W"], o.get("B"), o.get("alpha", 1.0), o.get("beta", 1.0), 0, o.get("transB", 0),
                            relu=bool(o.get("act", 0)))
        outs.append(np.asarray(y, dtype=np.float64))
        cur = np.asarray(y, dtype=np.float32)
        if k == "gemm":
            cur = cur.reshape(cur.shape[0], cur.shape[1], 1, 1)
    return outs


def device_ops(ops):
    return [{k: (dev(v) if k in ("W", "B") and v is not None else v) for k, v in o.items()} for o in ops]


def run_and_compare(lib, X, ops, exact_ints=False):
    ref = oracle_chain(X, ops)
    got = lib.onnx_chain(dev(X), device_ops(ops), keep=True)
    torch.cuda.synchronize()
    for i, (g, r) in enumerate(zip(got, ref)):
        g = g.cpu().numpy()
        assert g.reshape(r.shape).shape == r.shape
        g = g.reshape(r.shape)
        if exact_ints:
            assert np.array_equal(g.astype(np.float64), r), (i, ops[i]["op"])
        else:
            assert rel_err(g, r) <= REL_TOL, (i, ops[i]["op"], rel_err(g, r))
    # only the last result requested: the same values
    last = lib.onnx_chain(dev(X), device_ops(ops))
    torch.cuda.synchronize()
    assert torch.equal(last, got[-1])


def small_cnn_ops(m):
    w = m["weights"]
    return [dict(op="conv", W=w["w1"], B=w["b1"], pads=(2, 2, 2, 2), act=1),
            dict(op="maxpool", kernel=(2, 2), strides=(2, 2)),
            dict(op="conv", W=w["w2"], B=w["b2"], pads=(2, 2, 2, 2), act=1),
            dict(op="maxpool", kernel=(3, 3), strides=(3, 3)),
            dict(op="gemm", W=w["wg"], B=w["bg"].reshape(-1))]


@pytest.mark.parametrize("batch", [1, 3, 70])
def test_small_cnn_every_layer(lib, batch):
    """The MNIST-shaped network of Section 4.2, one workgroup per image."""
    print("CASE chain small cnn batch", batch, flush=True)
    m = workloads.small_cnn()
    rng = np.random.default_rng(batch)
    X = rng.uniform(0, 1, (batch, 1, 28, 28)).astype(np.float32)
    X[0] = m["inputs"]["x"][0]
    run_and_compare(lib, X, small_cnn_ops(m))


def _rand(rng, shape, scale=1.0):
    return (rng.uniform(-1, 1, shape) * scale).astype(np.float32)


def chain_cases():
    rng = np.random.default_rng(2024)
    cases = {}
    # strides, asymmetric pads, a ceil_mode average pool that counts the padding, a 1x1 Conv, the global
    # pool, a transposed Gemm with alpha / beta / Relu
    cases["strided_avg_global"] = ((2, 3, 17, 19), [
        dict(op="conv", W=_rand(rng, (5, 3, 3, 3)), B=_rand(rng, (5,)), pads=(1, 0, 2, 1), strides=(2, 2), act=1),
        dict(op="avgpool", kernel=(2, 2), strides=(2, 2), pads=(1, 1, 0, 0), ceil_mode=1, count_include_pad=1),
        dict(op="conv", W=_rand(rng, (20, 5, 1, 1)), B=None),
        dict(op="avgpool", kernel=None),
        dict(op="gemm", W=_rand(rng, (7, 20)), B=_rand(rng, (7,)), transB=1, alpha=0.5, beta=2.0, act=1)])
    # dilated Conv with a non-square window, a dilated padded MaxPool, then Conv feeding Conv (padded
    # buffer written by a Conv), 40 output channels (three channel blocks, the last half empty)
    cases["dilated_conv_conv"] = ((3, 2, 21, 16), [
        dict(op="conv", W=_rand(rng, (6, 2, 3, 2)), B=_rand(rng, (6,)), pads=(2, 1, 2, 2), dilations=(2, 3)),
        dict(op="maxpool", kernel=(2, 3), pads=(1, 1, 0, 1), strides=(1, 2), dilations=(2, 1)),
        dict(op="conv", W=_rand(rng, (40, 6, 3, 3), 0.3), B=_rand(rng, (40,)), pads=(1, 1, 1, 1), act=1),
        dict(op="conv", W=_rand(rng, (9, 40, 2, 2), 0.2), B=None, pads=(0, 1, 1, 0), strides=(2, 1), act=1),
        dict(op="avgpool", kernel=(3, 3), strides=(2, 2), pads=(1, 1, 1, 1), count_include_pad=0)])
    # a multi-layer perceptron: Gemm after Gemm, both weight layouts, no bias
    cases["mlp"] = ((5, 300, 1, 1), [
        dict(op="gemm", W=_rand(rng, (300, 33), 0.1), B=_rand(rng, (33,)), act=1),
        dict(op="gemm", W=_rand(rng, (17, 33), 0.3), B=None, transB=1, act=1),
        dict(op="gemm", W=_rand(rng, (17, 4)), B=_rand(rng, (4,)), alpha=-1.5)])
    # the limits: an activation of exactly ONNX_CHAIN_MAX_ACTIVATION floats, a Conv with K = C*kH*kW =
    # ONNX_CHAIN_MAX_CONV_K whose 6 filter rows (2052 floats each in LDS) almost fill the weight arena
    cases["at_the_limits"] = ((2, 128, 8, 10), [
        dict(op="conv", W=_rand(rng, (6, 128, 4, 4), 0.05), B=_rand(rng, (6,)), act=1),
        dict(op="maxpool", kernel=(2, 2), strides=(1, 1), pads=(1, 1, 1, 1)),
        dict(op="gemm", W=_rand(rng, (6 * 6 * 8, 3)), B=None)])
    # at most 8 output channels and a short K: the one-thread-per-position Conv, with strides, pads and dilation,
    # feeding a padded Conv on the matrix cores
    cases["direct_conv"] = ((3, 2, 23, 19), [
        dict(op="conv", W=_rand(rng, (7, 2, 3, 3)), B=_rand(rng, (7,)), pads=(2, 0, 1, 3), strides=(2, 3), dilations=(1, 2), act=1),
        dict(op="conv", W=_rand(rng, (8, 7, 2, 2), 0.4), B=None, pads=(1, 1, 0, 0)),
        dict(op="conv", W=_rand(rng, (12, 8, 3, 3), 0.3), B=_rand(rng, (12,)), pads=(1, 1, 1, 1), act=1),
        dict(op="avgpool", kernel=None)])
    # a single operator of each kind
    cases["one_conv"] = ((1, 4, 9, 9), [dict(op="conv", W=_rand(rng, (3, 4, 3, 3)), B=None, pads=(1, 1, 1, 1))])
    cases["one_pool"] = ((4, 6, 11, 13), [dict(op="maxpool", kernel=(3, 3), strides=(2, 2), pads=(1, 1, 1, 1), ceil_mode=1)])
    cases["one_gemm"] = ((2, 3, 5, 7), [dict(op="gemm", W=_rand(rng, (105, 19)), B=_rand(rng, (19,)))])
    return cases


CASES = chain_cases()


@pytest.mark.parametrize("name", sorted(CASES))
def test_chain_attribute_cases(lib, name):
    print("CASE chain", name, flush=True)
    shape, ops = CASES[name]
    rng = np.random.default_rng(len(name))
    run_and_compare(lib, _rand(rng, shape), ops)


def random_chain(rng):
    """A random chain of up to 6 operators on a small image; None when shape inference refuses it."""
    import paper_2008_08272_amd as lib
    n, c, h, w = int(rng.integers(1, 5)), int(rng.integers(1, 7)), int(rng.integers(5, 25)), int(rng.integers(5, 25))
    shape = (n, c, h, w)
    ops = []
    cur = shape
    for _ in range(int(rng.integers(1, 7))):
        flat = cur[2] == 1 and cur[3] == 1
        kind = "gemm" if (flat and ops) or rng.random() < 0.15 else ("conv", "conv", "maxpool", "avgpool")[int(rng.integers(0, 4))]
        pick = lambda lo, hi: int(rng.integers(lo, hi + 1))
        if kind == "gemm":
            k = cur[1] * cur[2] * cur[3]
            outs = pick(1, 40)
            tb = pick(0, 1)
            op = dict(op="gemm", W=_rand(rng, (outs, k) if tb else (k, outs), 0.3), B=_rand(rng, (outs,)) if pick(0, 1) else None,
                      transB=tb, alpha=float(rng.uniform(-1.5, 1.5)), beta=float(rng.uniform(-1.5, 1.5)), act=pick(0, 1))
        elif kind == "conv":
            m, kh, kw = pick(1, 24), pick(1, 4), pick(1, 4)
            op = dict(op="conv", W=_rand(rng, (m, cur[1], kh, kw), 0.4), B=_rand(rng, (m,)) if pick(0, 1) else None,
                      pads=tuple(pick(0, 2) for _ in range(4)), strides=(pick(1, 2), pick(1, 2)), dilations=(pick(1, 2), pick(1, 2)),
                      act=pick(0, 1))
        elif kind == "maxpool":
            kh, kw = pick(1, 3), pick(1, 3)
            op = dict(op="maxpool", kernel=(kh, kw), strides=(pick(1, 3), pick(1, 3)), dilations=(pick(1, 2), pick(1, 2)),
                      pads=(pick(0, (kh - 1) // 2), pick(0, (kw - 1) // 2), pick(0, (kh - 1) // 2), pick(0, (kw - 1) // 2)), ceil_mode=pick(0, 1))
        else:
            if rng.random() < 0.2:
                op = dict(op="avgpool", kernel=None)
            else:
                kh, kw = pick(1, 3), pick(1, 3)
                op = dict(op="avgpool", kernel=(kh, kw), strides=(pick(1, 3), pick(1, 3)),
                          pads=(pick(0, (kh - 1) // 2), pick(0, (kw - 1) // 2), pick(0, (kh - 1) // 2), pick(0, (kw - 1) // 2)),
                          ceil_mode=pick(0, 1), count_include_pad=pick(0, 1))
        try:
            cur = lib.chain_shapes(cur, [op])[0]
        except lib.OnnxHipError:
            return None
        if min(cur) < 1:
            return None
        ops.append(op)
    return shape, ops


def test_chain_random_sweep(lib):
    """Seeded random chains (every operator kind, random attributes, both Conv forms, every layer compared);
    chains that do not fit the kernel's LDS budget must be refused with ONNX_ERR_UNSUPPORTED and are skipped."""
    rng = np.random.default_rng(20080827)
    ran = refused = 0
    while ran < 40:
        c = random_chain(rng)
        if c is None:
            continue
        shape, ops = c
        print("CASE chain sweep", ran, shape, [(o["op"], tuple(o["W"].shape) if "W" in o else o.get("kernel")) for o in ops], flush=True)
        X = _rand(rng, shape)
        try:
            run_and_compare(lib, X, ops)
        except lib.OnnxHipError as e:
            assert e.status == 5, (e.status, str(e))
            refused += 1
            assert refused < 200
            continue
        ran += 1


def test_chain_small_integers_bit_exact(lib):
    """Integer-valued inputs and weights: every product and partial sum is exact in fp32, so the
    result must equal the oracle's bit for bit whatever the order of the K steps."""
    print("CASE chain integers", flush=True)
    rng = np.random.default_rng(11)
    ints = lambda shape, lo=-3, hi=4: rng.integers(lo, hi, shape).astype(np.float32)
    ops = [dict(op="conv", W=ints((8, 3, 5, 5)), B=ints((8,)), pads=(2, 2, 2, 2), act=1),
           dict(op="maxpool", kernel=(2, 2), strides=(2, 2)),
           dict(op="conv", W=ints((16, 8, 3, 3), -2, 3), B=ints((16,)), pads=(1, 1, 1, 1), strides=(2, 2), act=1),
           dict(op="gemm", W=ints((16 * 5 * 5, 10), -1, 2), B=ints((10,)))]
    run_and_compare(lib, ints((3, 3, 20, 20)), ops, exact_ints=True)


def test_chain_refuses_what_does_not_fit(lib):
    """Too large for LDS: ONNX_ERR_UNSUPPORTED, nothing launched, outputs untouched."""
    print("CASE chain limits", flush=True)
    rng = np.random.default_rng(3)
    X = dev(_rand(rng, (1, 3, 64, 64)))                       # 12288 floats > 10240
    with pytest.raises(lib.OnnxHipError) as e:
        lib.onnx_chain(X, [dict(op="maxpool", kernel=(2, 2), strides=(2, 2))])
    assert e.value.status == 5
    X = dev(_rand(rng, (1, 8, 30, 30)))                       # 7200 floats, but 8 x 36 x 36 = 10368 with the Conv's padding
    with pytest.raises(lib.OnnxHipError) as e:
        lib.onnx_chain(X, [dict(op="conv", W=dev(_rand(rng, (4, 8, 7, 7))), pads=(3, 3, 3, 3))])
    assert e.value.status == 5
    X = dev(_rand(rng, (1, 64, 8, 8)))                        # weights 64 rows of 580 floats > 14336
    with pytest.raises(lib.OnnxHipError) as e:
        lib.onnx_chain(X, [dict(op="conv", W=dev(_rand(rng, (64, 64, 3, 3))), pads=(1, 1, 1, 1))])
    assert e.value.status == 5
    X = dev(_rand(rng, (1, 240, 4, 4)))                       # K = 240*9 = 2160 > 2048
    with pytest.raises(lib.OnnxHipError) as e:
        lib.onnx_chain(X, [dict(op="conv", W=dev(_rand(rng, (2, 240, 3, 3))), pads=(1, 1, 1, 1))])
    assert e.value.status == 5
    out = torch.full((1, 3, 32, 32), 7.0, device="cuda")
    with pytest.raises(lib.OnnxHipError):
        lib.onnx_chain(dev(_rand(rng, (1, 3, 64, 64))), [dict(op="maxpool", kernel=(2, 2), strides=(2, 2))], outs=[out])
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())


def test_runner_uses_the_chain_for_the_small_cnn(lib):
    """The graph runner recognises the MNIST-shaped model as a chain and runs it as one launch; with
    the chain switched off the same model runs as one call per node; both match the oracle's chain
    on every layer."""
    print("CASE chain runner", flush=True)
    from oracle import chain
    from paper_2008_08272_amd.runner import GraphRunner
    m = workloads.small_cnn()
    _, exact = chain.run(m)
    for fuse in (True, False):
        r = GraphRunner(m, fuse_chain=fuse, keep_intermediates=True)
        assert (r.chain is not None) == fuse
        out = r.run()
        torch.cuda.synchronize()
        assert rel_err(out.cpu().numpy(), exact["logits"]) <= REL_TOL
        for name in ("c1", "p1", "c2", "p2"):
            assert rel_err(r.t[name].cpu().numpy(), exact[name]) <= REL_TOL, (fuse, name)
    # a model that is no chain (ResNet's shortcuts) or too large keeps the per-node calls
    assert GraphRunner(workloads.resnet50(1)).chain is None
    # the chain under HIP graph capture: every replay equals the eager result
    r = GraphRunner(m)
    eager = r.run().clone()
    torch.cuda.synchronize()
    r.capture()
    for i in range(3):
        r.output.zero_()
        torch.cuda.synchronize()
        assert torch.equal(r.replay(), eager), i
