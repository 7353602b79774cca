"""Pins for the oracle's operator definitions: brute force on tiny inputs, closed
forms, invariants, and special cases that reduce to a library routine."""
import math
import numpy as np
import pytest
from oracle import ops as O
from oracle import executor
from workloads import inception_block, random_small_dag

RNG = np.random.default_rng(1234)

# every (kernel, stride, pad) combination the five configs use
CONV_CASES = [((1, 1), (1, 1), (0, 0)), ((3, 3), (1, 1), (1, 1)), ((5, 5), (1, 1), (2, 2)),
              ((7, 7), (2, 2), (3, 3)), ((3, 3), (2, 2), (0, 0)), ((3, 3), (1, 1), (0, 0)),
              ((1, 7), (1, 1), (0, 3)), ((7, 1), (1, 1), (3, 0)), ((1, 3), (1, 1), (0, 1)),
              ((3, 1), (1, 1), (1, 0))]


def conv_brute(x, w, b, stride, pad, relu):
    cin, h, wd = x.shape
    cout, _, kh, kw = w.shape
    ho = (h + 2 * pad[0] - kh) // stride[0] + 1
    wo = (wd + 2 * pad[1] - kw) // stride[1] + 1
    y = np.zeros((cout, ho, wo))
    for co in range(cout):
        for oh in range(ho):
            for ow in range(wo):
                acc = b[co]
                for ci in range(cin):
                    for i in range(kh):
                        for j in range(kw):
                            ih, iw = oh * stride[0] + i - pad[0], ow * stride[1] + j - pad[1]
                            if 0 <= ih < h and 0 <= iw < wd:
                                acc += x[ci, ih, iw] * w[co, ci, i, j]
                y[co, oh, ow] = max(acc, 0.0) if relu else acc
    return y


@pytest.mark.parametrize("k,s,p", CONV_CASES)
@pytest.mark.parametrize("relu", [False, True])
def test_conv_brute_force(k, s, p, relu):
    x = RNG.standard_normal((3, 9, 8))
    w = RNG.standard_normal((4, 3, k[0], k[1]))
    b = RNG.standard_normal(4)
    np.testing.assert_allclose(O.conv2d(x, w, b, s, p, relu), conv_brute(x, w, b, s, p, relu),
                               rtol=1e-12, atol=1e-12)


def test_conv_1x1_is_matmul():
    x = RNG.standard_normal((5, 6, 7))
    w = RNG.standard_normal((4, 5, 1, 1))
    y = O.conv2d(x, w, np.zeros(4), (1, 1), (0, 0), False)
    ref = (x.reshape(5, -1).T @ w[:, :, 0, 0].T).T.reshape(4, 6, 7)
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-13)


def test_conv_delta_and_box():
    x = RNG.standard_normal((2, 6, 6))
    w = np.zeros((2, 2, 3, 3))
    w[0, 0, 1, 1] = w[1, 1, 1, 1] = 1.0       # centre tap, identity over channels
    np.testing.assert_array_equal(O.conv2d(x, w, np.zeros(2), (1, 1), (1, 1), False), x)
    # off-centre tap shifts: no kernel flip (cross-correlation)
    w2 = np.zeros((1, 1, 3, 3)); w2[0, 0, 0, 2] = 1.0
    y = O.conv2d(x[:1], w2, np.zeros(1), (1, 1), (1, 1), False)
    np.testing.assert_array_equal(y[0, 1:, :-1], x[0, :-1, 1:])
    ones = np.ones((1, 1, 3, 3))
    box = O.conv2d(np.ones((1, 5, 5)), ones, np.zeros(1), (1, 1), (1, 1), False)
    assert box[0, 0, 0] == 4 and box[0, 0, 2] == 6 and box[0, 2, 2] == 9


def test_conv_bias_and_relu():
    x = np.zeros((1, 3, 3))
    y = O.conv2d(x, np.ones((2, 1, 1, 1)), np.array([-1.5, 2.5]), (1, 1), (0, 0), True)
    assert (y[0] == 0).all() and (y[1] == 2.5).all()


def test_gemm_three_loops():
    m, k, n = 5, 7, 4
    x, w, b, e = RNG.standard_normal((m, k)), RNG.standard_normal((k, n)), RNG.standard_normal(n), RNG.standard_normal((m, n))
    ref = np.zeros((m, n))
    for i in range(m):
        for j in range(n):
            acc = b[j] + e[i, j]
            for t in range(k):
                acc += x[i, t] * w[t, j]
            ref[i, j] = acc
    np.testing.assert_allclose(O.gemm(x, w, b, [e]), ref, rtol=1e-12, atol=1e-12)
    # a transposed weight must not pass
    assert not np.allclose(O.gemm(x[:, :4], w[:4, :], b), x[:, :4] @ w[:4, :].T + b)


def test_bgemm_loops():
    heads, s, d = 3, 4, 2
    q, k, v = (RNG.standard_normal((s, heads * d)) for _ in range(3))
    sc = O.bgemm_qk(q, k, heads, 0.5)
    for h in range(heads):
        for i in range(s):
            for j in range(s):
                ref = 0.5 * sum(q[i, h * d + t] * k[j, h * d + t] for t in range(d))
                assert abs(sc[h, i, j] - ref) < 1e-12
    p = RNG.standard_normal((heads, s, s))
    ctx = O.bgemm_pv(p, v, heads)
    for h in range(heads):
        for i in range(s):
            for t in range(d):
                ref = sum(p[h, i, j] * v[j, h * d + t] for j in range(s))
                assert abs(ctx[i, h * d + t] - ref) < 1e-12


def pool_brute(x, k, s, p, kind):
    c, h, w = x.shape
    ho, wo = (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1
    y = np.zeros((c, ho, wo))
    for ch in range(c):
        for oh in range(ho):
            for ow in range(wo):
                vals = []
                for i in range(k):
                    for j in range(k):
                        ih, iw = oh * s + i - p, ow * s + j - p
                        if 0 <= ih < h and 0 <= iw < w:
                            vals.append(x[ch, ih, iw])
                y[ch, oh, ow] = max(vals) if kind == "max" else sum(vals) / (k * k)
    return y


@pytest.mark.parametrize("k,s,p", [(3, 1, 1), (3, 2, 1), (3, 2, 0)])
def test_pools_brute_force(k, s, p):
    x = RNG.standard_normal((3, 9, 10))
    np.testing.assert_array_equal(O.maxpool(x, (k, k), (s, s), (p, p)), pool_brute(x, k, s, p, "max"))
    np.testing.assert_allclose(O.avgpool(x, (k, k), (s, s), (p, p)), pool_brute(x, k, s, p, "avg"), rtol=1e-13, atol=1e-15)


def test_pool_invariants():
    x = RNG.standard_normal((2, 7, 7))
    assert (O.maxpool(x, (3, 3), (1, 1), (1, 1)) >= x).all()
    c = np.full((2, 6, 6), -3.25)
    np.testing.assert_array_equal(O.maxpool(c, (3, 3), (1, 1), (1, 1)), c)   # padding is -inf, not 0
    a = O.avgpool(np.ones((1, 5, 5)), (3, 3), (1, 1), (1, 1))
    assert a[0, 0, 0] == pytest.approx(4 / 9) and a[0, 2, 2] == pytest.approx(1.0)
    g = O.gavgpool(np.arange(8.0).reshape(2, 2, 2))
    np.testing.assert_allclose(g.reshape(-1), [1.5, 5.5])
    # output sizes used by the CNN configs (floor mode)
    assert O.maxpool(np.zeros((1, 112, 112)), (3, 3), (2, 2), (1, 1)).shape == (1, 56, 56)
    assert O.maxpool(np.zeros((1, 147, 147)), (3, 3), (2, 2), (0, 0)).shape == (1, 73, 73)


def test_concat_bit_identical():
    xs = [RNG.standard_normal((c, 3, 3)) for c in (2, 5, 1)]
    y = O.concat(xs, 0)
    o = 0
    for x in xs:
        assert y[o:o + x.shape[0]].tobytes() == x.tobytes()
        o += x.shape[0]
    ys = O.concat([x.reshape(x.shape[0], 9).T for x in xs], 1)
    assert ys.shape == (9, 8) and ys[:, 2:7].tobytes() == np.ascontiguousarray(xs[1].reshape(5, 9).T).tobytes()


def test_softmax_pins():
    x = RNG.standard_normal((6, 33)) * 5
    y = O.softmax([x])
    np.testing.assert_allclose(y.sum(-1), 1.0, rtol=0, atol=1e-12)
    assert (y >= 0).all() and (y <= 1).all()
    np.testing.assert_allclose(O.softmax([x + 1000.0]), y, rtol=1e-9, atol=1e-15)  # shift invariance, no overflow
    np.testing.assert_allclose(O.softmax([np.array([[0.0, math.log(2.0)]])]), [[1 / 3, 2 / 3]], rtol=1e-15)
    np.testing.assert_allclose(O.softmax([x[:, :5], 2 * x[:, :5]]), O.softmax([3 * x[:, :5]]), rtol=1e-12)


def test_layernorm_pins():
    x = RNG.standard_normal((5, 64)) * 3 + 7
    y = O.layernorm([x], 1e-5)
    np.testing.assert_allclose(y.mean(-1), 0.0, atol=1e-12)
    var = x.var(-1)
    np.testing.assert_allclose(y.var(-1), var / (var + 1e-5), rtol=1e-12)
    np.testing.assert_allclose(O.layernorm([np.array([[1.0, 2.0, 3.0, 4.0]])], 0.0),
                               [[-1.5 / math.sqrt(1.25), -0.5 / math.sqrt(1.25), 0.5 / math.sqrt(1.25), 1.5 / math.sqrt(1.25)]], rtol=1e-15)
    # eps enters under the root, added to the variance
    np.testing.assert_allclose(O.layernorm([np.array([[0.0, 2.0]])], 3.0), [[-0.5, 0.5]], rtol=1e-15)


def test_gelu_pins():
    x = np.linspace(-6, 6, 101)
    np.testing.assert_allclose(O.gelu([x]) - O.gelu([-x]), x, atol=1e-14)
    assert O.gelu([np.zeros(1)])[0] == 0.0
    # x * Phi(x) with the standard normal CDF: Phi(1) = 0.8413447460685429...
    assert O.gelu([np.ones(1)])[0] == pytest.approx(0.8413447460685429, abs=1e-15)
    assert O.gelu([np.array([2.0])])[0] == pytest.approx(2 * 0.9772498680518208, abs=1e-15)
    # the tanh approximation differs from the exact form by > 5e-5 at x = 2
    tanh_form = 0.5 * 2 * (1 + math.tanh(math.sqrt(2 / math.pi) * (2 + 0.044715 * 8)))
    assert abs(O.gelu([np.array([2.0])])[0] - tanh_form) > 5e-5


def test_relu_add():
    a, b = RNG.standard_normal((3, 4)), RNG.standard_normal((3, 4))
    np.testing.assert_array_equal(O.add([a, b]), a + b)
    np.testing.assert_array_equal(O.relu([a]), np.where(a > 0, a, 0))


def test_executor_rounds_between_ops_and_is_order_independent():
    wl = inception_block(random_bias=True)
    out = executor.run_dag(wl)
    assert all(v.dtype == np.float32 for v in out.values())
    # concat preserves the branch outputs bit for bit
    cat = out[7]
    assert cat.shape == (80, 28, 28)
    o = 0
    for u in wl.ops[7].inputs:
        c = out[u].shape[0]
        assert cat[o:o + c].tobytes() == out[u].tobytes()
        o += c
    # another valid topological order (largest id first) gives the same bits
    other = executor.kahn_order(len(wl.ops), wl.edges(), key=lambda v: -v)
    assert other != executor.kahn_order(len(wl.ops), wl.edges())
    out2 = executor.run_dag(wl, order=other)
    for v in out:
        assert out[v].tobytes() == out2[v].tobytes()


def test_executor_fp16_storage_and_prefix_views():
    wl = random_small_dag(5, dtype="f16", n_ops=30)
    out = executor.run_dag(wl)
    assert all(v.dtype == np.float16 for v in out.values())
    for op in wl.ops:
        assert out[op.id].shape == tuple(op.out_shape)
        assert np.isfinite(out[op.id].astype(np.float64)).all()
        if op.type == "softmax":
            s = out[op.id].astype(np.float64).sum(-1)
            assert np.abs(s - 1).max() <= op.out_shape[1] * 2.0 ** -11
    with pytest.raises(ValueError):
        executor.kahn_order(2, [(0, 1), (1, 0)])


def test_executor_batch_is_per_image():
    """With a batch, image operators act on every image alone and the FC sees one row per image."""
    from workloads import googlenet_like
    from workloads.dag import Workload
    wl = inception_block(batch=3, random_bias=True)
    out = executor.run_dag(wl)
    for b in range(3):
        one = Workload(wl.name, wl.dtype, wl.ops, [wl.ext_inputs[0][b]], wl.weights, wl.seed, 1)
        ref = executor.run_dag(one)
        assert all(out[v][b].tobytes() == ref[v].tobytes() for v in ref)
    g = googlenet_like(batch=2, he_init=True)
    og = executor.run_dag(g, keep=g.sinks())
    assert og[80].shape == (2, 1000) and not np.array_equal(og[80][0], og[80][1])


def test_elementwise_on_images_and_nasnet_like_wiring():
    """Element-wise operators stated on [C, H, W] shapes act per image; the NASNet-cell-like
    DAG feeds every cell from the two cells before it (skip connections across cells)."""
    from workloads import nasnet_like, Builder
    b = Builder("img_add", "f32", batch=2)
    x, y = b.ext((3, 4, 5)), b.ext((3, 4, 5))
    b.add_images([x, y])
    wl = b.build(9)
    out = executor.run_dag(wl)[0]
    assert out.shape == (2, 3, 4, 5)
    assert np.array_equal(out, (wl.ext_inputs[0].astype(np.float64) + wl.ext_inputs[1].astype(np.float64)).astype(np.float32))
    wl = nasnet_like(cells=3, width=8, hw=9, dtype="f32", he_init=True)
    cats = [op for op in wl.ops if op.type == "concat"]
    assert len(cats) == 3 and all(len(c.inputs) == 5 and c.out_shape == (40, 9, 9) for c in cats)
    # cell 2 reads cell 0's and cell 1's outputs
    readers_of = lambda v: [op.name for op in wl.ops if v in op.inputs]
    assert any(n.startswith("c2.sq_prev") for n in readers_of(cats[0].id))
    assert any(n.startswith("c2.sq_cur") for n in readers_of(cats[1].id))
    o1 = executor.run_dag(wl)
    o2 = executor.run_dag(nasnet_like(cells=3, width=8, hw=9, dtype="f32", he_init=True, batch=2))
    sink = wl.sinks()[0]
    assert o2[sink].shape == (2, 100) and np.isfinite(o2[sink]).all() and np.abs(o1[sink]).max() > 1e-3


def test_prefix_view_rule_on_a_hand_computed_dag():
    """An operator reads the leading prefix of its producer's flat row-major buffer in its
    own input shape.  Producer [2, 6] = relu of the external tensor, consumer views [3, 3]:
    elements 0..8 of the row-major buffer, i.e. the whole first row and half of the second."""
    from workloads.dag import Op, Workload
    x = np.array([[1, -2, 3, -4, 5, -6], [7, -8, 9, -10, 11, -12]], dtype=np.float32)
    ones = np.ones((3, 3), dtype=np.float32)
    ops = [Op(0, "relu", [-1], [(2, 6)], (2, 6), {}, "producer"),
           Op(1, "add", [0, -2], [(3, 3), (3, 3)], (3, 3), {}, "consumer")]
    out = executor.run_dag(Workload("prefix", "f32", ops, [x, ones], {}))
    assert np.array_equal(out[0], [[1, 0, 3, 0, 5, 0], [7, 0, 9, 0, 11, 0]])
    assert np.array_equal(out[1], [[2, 1, 4], [1, 6, 1], [8, 1, 10]])
    with pytest.raises(AssertionError):          # a consumer may not view more than the producer holds
        bad = [ops[0], Op(1, "relu", [0], [(13,)], (13,), {}, "too_long")]
        executor.run_dag(Workload("prefix", "f32", bad, [x], {}))
