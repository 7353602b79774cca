"""Builders for the five seeded synthetic DAGs plus small random DAGs for tests.

Operators are emitted in trace order (branch by branch inside a block), which is a
topological order.  Tensors come from numpy Generator(PCG64(seed)); draw order is
external inputs first (slot order), then per operator in id order: weight (bias is
all zeros unless `random_bias`).  Values are drawn in fp32 and rounded once to the
workload dtype.  `he_init` replaces the fixed weight deviation by sqrt(2/fan_in), which
keeps activations of the deep CNNs at order one (a test aid: with the configs' fixed
deviation of 0.02 the deep fp16 networks decay into the subnormal range).
"""
import numpy as np
from .dag import Op, Workload

BASE_SEED = 231210351
CONFIG_NAMES = ("inception_block", "googlenet_like", "inception_v3_like",
                "bert_base_like", "random_wide_dag", "nasnet_like")


class Builder:
    """Tiny DAG builder: appends operators, tracks output shapes."""

    def __init__(self, name, dtype, batch=1):
        self.name, self.dtype, self.batch = name, dtype, batch
        self.ops = []
        self.ext_shapes = []

    def ext(self, shape):
        self.ext_shapes.append(tuple(shape))
        return -len(self.ext_shapes)

    def shape(self, t):
        return self.ext_shapes[-t - 1] if t < 0 else self.ops[t].out_shape

    def add(self, type_, inputs, in_shapes, out_shape, params=None, name=""):
        op = Op(len(self.ops), type_, list(inputs), [tuple(s) for s in in_shapes],
                tuple(out_shape), dict(params or {}), name or f"{type_}{len(self.ops)}")
        self.ops.append(op)
        return op.id

    # ---- CNN operators, logical [C,H,W] ----
    def conv(self, x, cout, k, stride=1, pad=0, relu=True, name=""):
        cin, h, w = self.shape(x)
        kh, kw = (k, k) if isinstance(k, int) else k
        sh, sw = (stride, stride) if isinstance(stride, int) else stride
        ph, pw = (pad, pad) if isinstance(pad, int) else pad
        ho = (h + 2 * ph - kh) // sh + 1
        wo = (w + 2 * pw - kw) // sw + 1
        p = dict(cin=cin, cout=cout, kh=kh, kw=kw, sh=sh, sw=sw, ph=ph, pw=pw, relu=bool(relu))
        return self.add("conv2d", [x], [(cin, h, w)], (cout, ho, wo), p, name)

    def pool(self, kind, x, k, stride, pad, name=""):
        c, h, w = self.shape(x)
        ho = (h + 2 * pad - k) // stride + 1
        wo = (w + 2 * pad - k) // stride + 1
        p = dict(kh=k, kw=k, sh=stride, sw=stride, ph=pad, pw=pad)
        return self.add(kind, [x], [(c, h, w)], (c, ho, wo), p, name)

    def gavgpool(self, x, name=""):
        c, h, w = self.shape(x)
        return self.add("gavgpool", [x], [(c, h, w)], (c, 1, 1), {}, name)

    def concat_c(self, xs, name=""):
        shapes = [self.shape(x) for x in xs]
        h, w = shapes[0][1:]
        assert all(s[1:] == (h, w) for s in shapes)
        return self.add("concat", xs, shapes, (sum(s[0] for s in shapes), h, w), {"axis": 0}, name)

    # ---- matrix operators, logical [R,C] ----
    def gemm(self, x, m, k, n, extras=(), relu=False, name=""):
        p = dict(m=m, k=k, n=n, relu=bool(relu))
        return self.add("gemm", [x] + list(extras), [(m, k)] + [(m, n)] * len(extras), (m, n), p, name)

    def add_images(self, xs, name=""):
        """Element-wise sum of image tensors of one shape ([C, H, W] each)."""
        shp = self.shape(xs[0])
        assert len(shp) == 3 and all(self.shape(x) == shp for x in xs)
        return self.add("add", list(xs), [shp] * len(xs), shp, {}, name)

    def rowwise(self, kind, xs, r, c, params=None, name=""):
        return self.add(kind, xs, [(r, c)] * len(xs), (r, c), params or {}, name)

    def build(self, seed, random_bias=False, w_std=0.02, he_init=False):
        rng = np.random.Generator(np.random.PCG64(seed))
        npdt = np.float32 if self.dtype == "f32" else np.float16
        lead = lambda s: ((self.batch,) + s) if (self.batch > 1 and len(s) == 3) else s
        ext = [rng.standard_normal(lead(s), dtype=np.float32).astype(npdt) for s in self.ext_shapes]
        weights = {}
        for op in self.ops:
            p = op.params
            if op.type == "conv2d":
                wshape, nb = (p["cout"], p["cin"], p["kh"], p["kw"]), p["cout"]
            elif op.type == "gemm":
                wshape, nb = (p["k"], p["n"]), p["n"]
            else:
                continue
            w = rng.standard_normal(wshape, dtype=np.float32)
            fan_in = int(np.prod(wshape[1:])) if op.type == "conv2d" else wshape[0]
            w *= np.float32(np.sqrt(2.0 / fan_in) if he_init else w_std)
            if random_bias:
                b = rng.standard_normal(nb, dtype=np.float32) * np.float32(0.1)
            else:
                b = np.zeros(nb, dtype=np.float32)
            weights[op.id] = {"w": w.astype(npdt), "b": b.astype(npdt)}
        return Workload(self.name, self.dtype, self.ops, ext, weights, seed, self.batch)


def _inception(b, x, c1, c3r, c3, c5r, c5, pp, tag):
    """Four-branch block: 1x1 | 1x1,3x3 | 1x1,5x5 | maxpool,1x1 -> channel concat."""
    b1 = b.conv(x, c1, 1, name=f"{tag}.b1.1x1")
    b2 = b.conv(x, c3r, 1, name=f"{tag}.b2.1x1")
    b2 = b.conv(b2, c3, 3, pad=1, name=f"{tag}.b2.3x3")
    b3 = b.conv(x, c5r, 1, name=f"{tag}.b3.1x1")
    b3 = b.conv(b3, c5, 5, pad=2, name=f"{tag}.b3.5x5")
    b4 = b.pool("maxpool", x, 3, 1, 1, name=f"{tag}.b4.pool")
    b4 = b.conv(b4, pp, 1, name=f"{tag}.b4.1x1")
    return b.concat_c([b1, b2, b3, b4], name=f"{tag}.cat")


def inception_block(seed=BASE_SEED + 0, dtype="f32", random_bias=False, batch=1):
    b = Builder("inception_block", dtype, batch)
    x = b.ext((64, 28, 28))
    _inception(b, x, 16, 24, 32, 8, 16, 16, "blk")
    return b.build(seed, random_bias)


GOOGLENET_WIDTHS = {  # (1x1, 3x3-reduce, 3x3, 5x5-reduce, 5x5, pool-proj)
    "3a": (64, 96, 128, 16, 32, 32), "3b": (128, 128, 192, 32, 96, 64),
    "4a": (192, 96, 208, 16, 48, 64), "4b": (160, 112, 224, 24, 64, 64),
    "4c": (128, 128, 256, 24, 64, 64), "4d": (112, 144, 288, 32, 64, 64),
    "4e": (256, 160, 320, 32, 128, 128), "5a": (256, 160, 320, 32, 128, 128),
    "5b": (384, 192, 384, 48, 128, 128),
}


def googlenet_like(seed=BASE_SEED + 1, dtype="f16", he_init=False, batch=1):
    b = Builder("googlenet_like", dtype, batch)
    x = b.ext((3, 224, 224))
    x = b.conv(x, 64, 7, stride=2, pad=3, name="stem.conv7x7")
    x = b.pool("maxpool", x, 3, 2, 1, name="stem.pool1")
    x = b.conv(x, 64, 1, name="stem.conv1x1")
    x = b.conv(x, 192, 3, pad=1, name="stem.conv3x3")
    x = b.pool("maxpool", x, 3, 2, 1, name="stem.pool2")
    for tag in ("3a", "3b"):
        x = _inception(b, x, *GOOGLENET_WIDTHS[tag], tag)
    x = b.pool("maxpool", x, 3, 2, 1, name="pool3")
    for tag in ("4a", "4b", "4c", "4d", "4e"):
        x = _inception(b, x, *GOOGLENET_WIDTHS[tag], tag)
    x = b.pool("maxpool", x, 3, 2, 1, name="pool4")
    for tag in ("5a", "5b"):
        x = _inception(b, x, *GOOGLENET_WIDTHS[tag], tag)
    x = b.gavgpool(x, name="gap")
    b.gemm(x, batch, 1024, 1000, name="fc")
    return b.build(seed, he_init=he_init)


def inception_v3_like(seed=BASE_SEED + 2, dtype="f16", he_init=False, batch=1):
    b = Builder("inception_v3_like", dtype, batch)
    x = b.ext((3, 299, 299))
    x = b.conv(x, 32, 3, stride=2, name="stem.1")
    x = b.conv(x, 32, 3, name="stem.2")
    x = b.conv(x, 64, 3, pad=1, name="stem.3")
    x = b.pool("maxpool", x, 3, 2, 0, name="stem.pool1")
    x = b.conv(x, 80, 1, name="stem.4")
    x = b.conv(x, 192, 3, name="stem.5")
    x = b.pool("maxpool", x, 3, 2, 0, name="stem.pool2")
    for i, pf in enumerate((32, 64, 64)):          # block A x3 at 35x35
        t = f"A{i}"
        b1 = b.conv(x, 64, 1, name=f"{t}.b1")
        b2 = b.conv(x, 48, 1, name=f"{t}.b2.1x1")
        b2 = b.conv(b2, 64, 5, pad=2, name=f"{t}.b2.5x5")
        b3 = b.conv(x, 64, 1, name=f"{t}.b3.1x1")
        b3 = b.conv(b3, 96, 3, pad=1, name=f"{t}.b3.3x3a")
        b3 = b.conv(b3, 96, 3, pad=1, name=f"{t}.b3.3x3b")
        b4 = b.pool("avgpool", x, 3, 1, 1, name=f"{t}.b4.pool")
        b4 = b.conv(b4, pf, 1, name=f"{t}.b4.1x1")
        x = b.concat_c([b1, b2, b3, b4], name=f"{t}.cat")
    # reduction B: 35 -> 17
    b1 = b.conv(x, 384, 3, stride=2, name="B.b1")
    b2 = b.conv(x, 64, 1, name="B.b2.1x1")
    b2 = b.conv(b2, 96, 3, pad=1, name="B.b2.3x3a")
    b2 = b.conv(b2, 96, 3, stride=2, name="B.b2.3x3b")
    b3 = b.pool("maxpool", x, 3, 2, 0, name="B.b3.pool")
    x = b.concat_c([b1, b2, b3], name="B.cat")
    for i, c in enumerate((128, 160, 160, 192)):   # block C x4 at 17x17
        t = f"C{i}"
        b1 = b.conv(x, 192, 1, name=f"{t}.b1")
        b2 = b.conv(x, c, 1, name=f"{t}.b2.1x1")
        b2 = b.conv(b2, c, (1, 7), pad=(0, 3), name=f"{t}.b2.1x7")
        b2 = b.conv(b2, 192, (7, 1), pad=(3, 0), name=f"{t}.b2.7x1")
        b3 = b.conv(x, c, 1, name=f"{t}.b3.1x1")
        b3 = b.conv(b3, c, (7, 1), pad=(3, 0), name=f"{t}.b3.7x1a")
        b3 = b.conv(b3, c, (1, 7), pad=(0, 3), name=f"{t}.b3.1x7a")
        b3 = b.conv(b3, c, (7, 1), pad=(3, 0), name=f"{t}.b3.7x1b")
        b3 = b.conv(b3, 192, (1, 7), pad=(0, 3), name=f"{t}.b3.1x7b")
        b4 = b.pool("avgpool", x, 3, 1, 1, name=f"{t}.b4.pool")
        b4 = b.conv(b4, 192, 1, name=f"{t}.b4.1x1")
        x = b.concat_c([b1, b2, b3, b4], name=f"{t}.cat")
    # reduction D: 17 -> 8
    b1 = b.conv(x, 192, 1, name="D.b1.1x1")
    b1 = b.conv(b1, 320, 3, stride=2, name="D.b1.3x3")
    b2 = b.conv(x, 192, 1, name="D.b2.1x1")
    b2 = b.conv(b2, 192, (1, 7), pad=(0, 3), name="D.b2.1x7")
    b2 = b.conv(b2, 192, (7, 1), pad=(3, 0), name="D.b2.7x1")
    b2 = b.conv(b2, 192, 3, stride=2, name="D.b2.3x3")
    b3 = b.pool("maxpool", x, 3, 2, 0, name="D.b3.pool")
    x = b.concat_c([b1, b2, b3], name="D.cat")
    for i in range(2):                              # block E x2 at 8x8
        t = f"E{i}"
        b1 = b.conv(x, 320, 1, name=f"{t}.b1")
        b2 = b.conv(x, 384, 1, name=f"{t}.b2.1x1")
        b2a = b.conv(b2, 384, (1, 3), pad=(0, 1), name=f"{t}.b2.1x3")
        b2b = b.conv(b2, 384, (3, 1), pad=(1, 0), name=f"{t}.b2.3x1")
        b3 = b.conv(x, 448, 1, name=f"{t}.b3.1x1")
        b3 = b.conv(b3, 384, 3, pad=1, name=f"{t}.b3.3x3")
        b3a = b.conv(b3, 384, (1, 3), pad=(0, 1), name=f"{t}.b3.1x3")
        b3b = b.conv(b3, 384, (3, 1), pad=(1, 0), name=f"{t}.b3.3x1")
        b4 = b.pool("avgpool", x, 3, 1, 1, name=f"{t}.b4.pool")
        b4 = b.conv(b4, 192, 1, name=f"{t}.b4.1x1")
        x = b.concat_c([b1, b2a, b2b, b3a, b3b, b4], name=f"{t}.cat")
    x = b.gavgpool(x, name="gap")
    b.gemm(x, batch, 2048, 1000, name="fc")
    return b.build(seed, he_init=he_init)


def bert_base_like(seed=BASE_SEED + 3, dtype="f16", layers=12, seq=128, hidden=768,
                   heads=12, ffn=3072):
    b = Builder("bert_base_like", dtype)
    d = hidden // heads
    x = b.ext((seq, hidden))
    for l in range(layers):
        t = f"L{l}"
        q = b.gemm(x, seq, hidden, hidden, name=f"{t}.q")
        k = b.gemm(x, seq, hidden, hidden, name=f"{t}.k")
        v = b.gemm(x, seq, hidden, hidden, name=f"{t}.v")
        att = dict(heads=heads, seq=seq, dhead=d)
        s = b.add("bgemm", [q, k], [(seq, hidden)] * 2, (heads, seq, seq),
                  dict(mode="qk", alpha=1.0 / float(np.sqrt(d)), **att), f"{t}.scores")
        p = b.rowwise("softmax", [s], heads * seq, seq, name=f"{t}.softmax")
        c = b.add("bgemm", [p, v], [(heads, seq, seq), (seq, hidden)], (seq, hidden),
                  dict(mode="pv", alpha=1.0, **att), f"{t}.context")
        o = b.gemm(c, seq, hidden, hidden, name=f"{t}.out")
        a1 = b.rowwise("add", [o, x], seq, hidden, name=f"{t}.add1")
        n1 = b.rowwise("layernorm", [a1], seq, hidden, {"eps": 1e-5}, f"{t}.ln1")
        f1 = b.gemm(n1, seq, hidden, ffn, name=f"{t}.ffn1")
        g = b.rowwise("gelu", [f1], seq, ffn, name=f"{t}.gelu")
        f2 = b.gemm(g, seq, ffn, hidden, name=f"{t}.ffn2")
        a2 = b.rowwise("add", [f2, n1], seq, hidden, name=f"{t}.add2")
        x = b.rowwise("layernorm", [a2], seq, hidden, {"eps": 1e-5}, f"{t}.ln2")
    return b.build(seed)


_MEM_KINDS = ("add", "gelu", "layernorm", "softmax", "concat")


def nasnet_like(seed=BASE_SEED + 5, dtype="f16", cells=6, width=32, hw=28, he_init=False, batch=1):
    """An irregular cell-structured CNN in the manner of NASNet-A's normal cell (the paper
    evaluates NASNet, Sec. 5.1): every cell takes the outputs of the two previous cells,
    squeezes each with a 1x1 convolution, forms five blocks add(op(a), op(b)) with operators
    drawn from {3x3 conv, 5x5 conv, 3x3 average pool, 3x3 max pool, identity}, and
    concatenates the five sums.  Ordinary convolutions stand in for NASNet's separable ones
    (this operator set has no depthwise convolution); the wiring is what matters here."""
    b = Builder("nasnet_like", dtype, batch)
    x = b.ext((3, hw, hw))
    stem = b.conv(x, 5 * width, 3, pad=1, name="stem")
    prev, cur = stem, stem
    for c in range(cells):
        t = f"c{c}"
        hp = b.conv(prev, width, 1, name=t + ".sq_prev")
        hc = b.conv(cur, width, 1, name=t + ".sq_cur")
        conv3 = lambda v, n: b.conv(v, width, 3, pad=1, relu=False, name=n)
        conv5 = lambda v, n: b.conv(v, width, 5, pad=2, relu=False, name=n)
        avg = lambda v, n: b.pool("avgpool", v, 3, 1, 1, name=n)
        mx = lambda v, n: b.pool("maxpool", v, 3, 1, 1, name=n)
        blocks = [
            b.add_images([conv3(hc, t + ".b0.c3"), hc], name=t + ".b0"),
            b.add_images([conv3(hp, t + ".b1.c3"), conv5(hc, t + ".b1.c5")], name=t + ".b1"),
            b.add_images([avg(hc, t + ".b2.avg"), hp], name=t + ".b2"),
            b.add_images([avg(hp, t + ".b3.avg"), mx(hp, t + ".b3.max")], name=t + ".b3"),
            b.add_images([conv5(hp, t + ".b4.c5"), conv3(hp, t + ".b4.c3")], name=t + ".b4"),
        ]
        out = b.concat_c(blocks, name=t + ".cat")
        prev, cur = cur, out
    g = b.gavgpool(cur, name="gap")
    b.gemm(g, batch, 5 * width, 100, name="fc")
    return b.build(seed, he_init=he_init)


def _numel(shape):
    n = 1
    for s in shape:
        n *= s
    return n


def _random_dag(name, seed, dtype, n_ops, max_width, gemm_units, mem_elems, col_units,
                max_m_units=8, unit=64, w_std=0.02):
    """Level-structured random DAG.  gemm_units=(lo,hi): N,K = unit*U{lo..hi};
    mem_elems=(lo,hi): element count range of memory-bound tensors; col_units: their
    column count = unit*U{lo..hi}."""
    rs = np.random.Generator(np.random.PCG64([seed, 7]))   # structure stream
    b = Builder(name, dtype)
    levels = []
    while len(b.ops) < n_ops:
        width = min(int(rs.integers(1, max_width + 1)), n_ops - len(b.ops))
        this_level = []
        for _ in range(width):
            is_gemm = rs.random() < 0.45
            kind = "gemm" if is_gemm else _MEM_KINDS[int(rs.integers(0, len(_MEM_KINDS)))]
            fan_in = int(rs.integers(1, 4))
            if kind == "add":
                fan_in = max(fan_in, 2)
            if is_gemm:
                m = unit * int(rs.integers(1, max_m_units + 1))
                n = unit * int(rs.integers(gemm_units[0], gemm_units[1] + 1))
                k = unit * int(rs.integers(gemm_units[0], gemm_units[1] + 1))
                out_shape = (m, n)
                in_shapes = [(m, k)] + [(m, n)] * (fan_in - 1)
            else:
                c = unit * int(rs.integers(col_units[0], col_units[1] + 1))
                r_lo = max(1, -(-mem_elems[0] // c))
                r_hi = max(r_lo, mem_elems[1] // c)
                r = int(rs.integers(r_lo, r_hi + 1))
                out_shape = (r, c)
                if kind == "concat":
                    cu = c // unit
                    fan_in = min(fan_in, cu)
                    parts = [cu // fan_in + (1 if i < cu % fan_in else 0) for i in range(fan_in)]
                    in_shapes = [(r, unit * pu) for pu in parts]
                else:
                    in_shapes = [(r, c)] * fan_in
            prev = levels[-1] if levels else []
            earlier = [i for lv in levels for i in lv]
            inputs, shapes = [], []
            for j, shp in enumerate(in_shapes):
                need = _numel(shp)
                pool = prev if j == 0 else earlier
                cand = [i for i in pool if i not in inputs and _numel(b.ops[i].out_shape) >= need]
                if not cand and j == 0:
                    cand = [i for i in earlier if _numel(b.ops[i].out_shape) >= need]
                if cand:
                    inputs.append(cand[int(rs.integers(0, len(cand)))])
                    shapes.append(shp)
                elif j == 0 or kind == "concat":
                    inputs.append(b.ext(shp))
                    shapes.append(shp)
                # else: drop this optional extra input
            params = {}
            if is_gemm:
                params = dict(m=m, k=k, n=n, relu=False)
            elif kind == "layernorm":
                params = {"eps": 1e-5}
            elif kind == "concat":
                params = {"axis": 1}
            this_level.append(b.add(kind, inputs, shapes, out_shape, params))
        levels.append(this_level)
    wl = b.build(seed, w_std=w_std)
    wl.levels = levels
    return wl


def random_wide_dag(seed=BASE_SEED + 4, dtype="f16", n_ops=400):
    return _random_dag("random_wide_dag", seed, dtype, n_ops, 12, gemm_units=(4, 64),
                       mem_elems=(1 << 19, 1 << 22), col_units=(4, 64))


def random_small_dag(seed, dtype="f16", n_ops=40, max_width=6):
    """Same generator at toy sizes (tensors of a few KB) for fast parity tests."""
    return _random_dag("random_small_dag", seed, dtype, n_ops, max_width, gemm_units=(1, 5),
                       mem_elems=(1 << 10, 1 << 13), col_units=(1, 5), max_m_units=3, unit=16,
                       w_std=0.1)


def appendix_example_edges():
    """A 13-operator DAG consistent with the four placement rules of the paper's
    appendix example (the figure itself is not available; this edge set is a
    reconstruction).  Operators are numbered 1..13 as in the text."""
    return [(1, 2), (1, 3), (1, 4), (2, 5), (3, 6), (4, 7), (5, 8), (6, 8), (7, 8),
            (8, 9), (8, 10), (9, 11), (9, 12), (10, 13), (11, 13), (12, 13)]


def build_config(index):
    return (inception_block, googlenet_like, inception_v3_like, bert_base_like,
            random_wide_dag, nasnet_like)[index]()
