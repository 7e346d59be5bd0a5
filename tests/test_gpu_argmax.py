"""GPU parity for Argmax (Algorithm 6) and MaxPool (Algorithm 7): the same protocol flow
(tests/argmax_flow.py) driven once over the oracle and once over the HIP library through its
C ABI; every intermediate of both parties must match bit for bit."""
import numpy as np
import pytest

import argmax_flow as F
import paper_2006_04593_amd as fss
from paper_2006_04593_amd import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

DEV = "cuda:0"


def to_dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).to(DEV)


def new(count):
    return torch.full((int(count),), -1, dtype=torch.int32, device=DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy().view(np.uint32)


class GpuBackend:
    """Same interface as argmax_flow.OracleBackend; numpy in, numpy out; keys stay on the device."""

    def gen(self, kind, n, g):
        nbytes = (fss.cmp_key_bytes if kind == "cmp" else fss.eq_key_bytes)(n, g.batch)
        k = [torch.zeros(nbytes, dtype=torch.uint8, device=DEV) for _ in range(2)]
        (fss.cmp_gen if kind == "cmp" else fss.eq_gen)(n, g.batch, to_dev(g.alpha), to_dev(g.r), to_dev(g.seed0), to_dev(g.seed1), k[0], k[1])
        return k

    def argmax_diff_mask(self, n, rows, m, key, x):
        out = new(rows * m * (m - 1))
        fss.argmax_diff_mask(n, rows, m, key, to_dev(x), out)
        return host(out)

    def sign_eval(self, j, n, key, m0, m1):
        out = new(len(m0))
        fss.sign_eval(j, n, len(m0), key, to_dev(m0), to_dev(m1), out)
        return host(out)

    def argmax_count_mask(self, j, n, rows, m, w, key):
        out = new(rows * m)
        fss.argmax_count_mask(j, n, rows, m, to_dev(w), key, out)
        return host(out)

    def eq_masked_eval(self, j, n, key, m0, m1):
        out = new(len(m0))
        fss.eq_masked_eval(j, n, len(m0), key, to_dev(m0), to_dev(m1), out)
        return host(out)

    def maxpool_unroll(self, c, h, w, k, s, x):
        oh, ow = (h - k) // s + 1, (w - k) // s + 1
        out = new(c * oh * ow * k * k)
        fss.maxpool_unroll(c, h, w, k, s, to_dev(x), out)
        return host(out).reshape(c * oh * ow, k * k)

    def mul_open(self, n, u, v, a, b):
        cnt = int(np.asarray(u).size)
        d, e = new(cnt), new(cnt)
        fss.mul_open(n, cnt, to_dev(np.asarray(u).reshape(-1)), to_dev(np.asarray(v).reshape(-1)), to_dev(a), to_dev(b), d, e)
        return host(d), host(e)

    def dot_finish(self, j, n, rows, m, d0, d1, e0, e1, a, b, c):
        out = new(rows)
        fss.dot_finish(j, n, rows, m, *[to_dev(np.asarray(t).reshape(-1)) for t in (d0, d1, e0, e1, a, b, c)], out)
        return host(out)


def shares_of(rng, n, values):
    s0, s1 = W.additive_shares(rng, n, values.reshape(-1).astype(np.int64).astype(np.uint64))
    return s0.reshape(values.shape), s1.reshape(values.shape)


def same(a, b, names):
    for name in names:
        for j in (0, 1):
            assert np.array_equal(np.asarray(a[name][j]).reshape(-1), np.asarray(b[name][j]).reshape(-1)), (name, j)


# rows = None: sized from the library's switch of register layouts so that BOTH evaluations of the
# flow -- the m(m-1) comparisons per row and the m equalities per row -- run one lane per element;
# (32, 12800, 9) has 921,600 comparisons in that layout and 115,200 equalities four lanes per element
@pytest.mark.parametrize("n,rows,m", [(32, 1, 2), (32, 100, 10), (16, 257, 4), (32, 64, 9), (12, 31, 3), (32, 12800, 9), (32, None, 4)])
def test_argmax_matches_oracle(n, rows, m):
    if rows is None:
        switch = fss.quad_layout_below()
        rows = switch // m + 64
        assert rows * m >= switch and rows * m * (m - 1) >= switch
    print(f"case argmax n={n} rows={rows} m={m}", flush=True)
    rng = np.random.default_rng(n * 100 + rows + m)
    x = W.fixed_point_normal(rng, (rows, m), frac_bits=max(1, min(10, n - 14)))
    if rows > 1:
        x[0] = x[0, 0]
    xs = shares_of(rng, n, x)
    mat = F.material(rng, n, rows, m)
    got = F.argmax(GpuBackend(), mat, xs)
    want = F.argmax(F.OracleBackend(), mat, xs)
    same(got, want, ("masked_cmp", "w", "masked_eq", "onehot"))
    onehot = (got["onehot"][0] + got["onehot"][1]) & np.uint32(W.ring_mask(n))
    w = ((got["w"][0] + got["w"][1]) & np.uint32(W.ring_mask(n))).reshape(rows, m, m - 1)
    assert np.array_equal(onehot.reshape(rows, m), (w.sum(axis=2) == m - 1).astype(np.uint32))


@pytest.mark.parametrize("k,channels,h,w", [(2, 3, 8, 10), (3, 2, 9, 11), (2, 1, 2, 2)])
def test_maxpool_matches_oracle(k, channels, h, w):
    print(f"case maxpool k={k} c={channels} h={h} w={w}", flush=True)
    n = 32
    rng = np.random.default_rng(k * 1000 + h)
    x = W.fixed_point_normal(rng, (channels, h, w))
    xs = shares_of(rng, n, x)
    oh, ow = (h - k) // 2 + 1, (w - k) // 2 + 1
    rows, m = channels * oh * ow, k * k
    mat = F.material(rng, n, rows, m)
    got = F.maxpool(GpuBackend(), mat, channels, h, w, k, xs)
    want = F.maxpool(F.OracleBackend(), mat, channels, h, w, k, xs)
    same(got, want, ("rows", "masked_cmp", "w", "masked_eq", "onehot", "delta", "eps", "out"))
    win = np.stack([x[c, 2 * i:2 * i + k, 2 * j:2 * j + k].reshape(-1) for c in range(channels) for i in range(oh) for j in range(ow)])
    out = got["out"][0] + got["out"][1]
    ok = ((got["onehot"][0] + got["onehot"][1]).reshape(rows, m).sum(axis=1) == 1) & ((win == win.max(axis=1, keepdims=True)).sum(axis=1) == 1)
    assert np.array_equal(out[ok], (win.max(axis=1)[ok] & 0xFFFFFFFF).astype(np.uint32))


def test_maxpool_2x2_layer_shape():
    """A VGG-style 2x2/2 max-pool of 64 x 32 x 32 activations: 16,384 windows, 196,608 comparisons
    and 65,536 equalities on the GPU; the oracle replays a sample of windows through the same flow."""
    n, k, channels, h, w = 32, 2, 64, 32, 32
    rng = np.random.default_rng(2232)
    x = W.fixed_point_normal(rng, (channels, h, w))
    xs = shares_of(rng, n, x)
    rows, m = channels * 16 * 16, 4
    mat = F.material(rng, n, rows, m)
    got = F.maxpool(GpuBackend(), mat, channels, h, w, k, xs)
    win = x.reshape(channels, 16, 2, 16, 2).transpose(0, 1, 3, 2, 4).reshape(rows, 4)
    out = got["out"][0] + got["out"][1]
    onehot = (got["onehot"][0] + got["onehot"][1]).reshape(rows, m)
    assert np.array_equal(out, ((win * onehot.astype(np.int64)).sum(axis=1) & 0xFFFFFFFF).astype(np.uint32))
    good = (onehot.sum(axis=1) == 1) & ((win == win.max(axis=1, keepdims=True)).sum(axis=1) == 1)
    assert good.mean() > 0.95
    assert np.array_equal(out[good], (win.max(axis=1)[good] & 0xFFFFFFFF).astype(np.uint32))
    # oracle on a sample of windows, with the material of exactly those windows
    idx = np.sort(np.random.default_rng(5).choice(rows, size=512, replace=False))
    e_cmp = (idx[:, None] * (m * (m - 1)) + np.arange(m * (m - 1))[None, :]).reshape(-1)
    e_eq = (idx[:, None] * m + np.arange(m)[None, :]).reshape(-1)
    pick = lambda g, e: W.GenInputs(n=n, alpha=g.alpha[e], r=g.r[e], seed0=g.seed0[e], seed1=g.seed1[e])
    tr = mat.triples
    sub = F.ArgmaxMaterial(n=n, rows=len(idx), m=m, cmp_gen=pick(mat.cmp_gen, e_cmp), eq_gen=pick(mat.eq_gen, e_eq),
                           triples=W.TripleShares(a=tuple(t[e_eq] for t in tr.a), b=tuple(t[e_eq] for t in tr.b), c=tuple(t[e_eq] for t in tr.c)))
    ob = F.OracleBackend()
    ref = F.argmax(ob, sub, [got["rows"][j][idx] for j in (0, 1)])
    assert np.array_equal(ref["onehot"][0], got["onehot"][0].reshape(rows, m)[idx].reshape(-1))
    assert np.array_equal(ref["onehot"][1], got["onehot"][1].reshape(rows, m)[idx].reshape(-1))
    assert np.array_equal(ref["w"][0], got["w"][0].reshape(rows, m * (m - 1))[idx].reshape(-1))


def test_maxpool_2x2_binary_tree_variant():
    """The paper's k = 2 optimisation (appendix C.3): max of columns 0,1 and 2,3, then the max of
    the two, 4 rounds and k^2 - 1 = 3 comparisons per window.  max(a, b) = b + ReLU(a - b), so each
    level is one ReLU layer of this library (fss_sign_mask / fss_relu_open / fss_relu_finish); the
    additions between levels are local share arithmetic done here by the test."""
    import oracle
    n, channels, h, w = 32, 8, 16, 16
    rng = np.random.default_rng(404)
    x = W.fixed_point_normal(rng, (channels, h, w))
    rows = channels * 8 * 8
    win = x.reshape(channels, 8, 2, 8, 2).transpose(0, 1, 3, 2, 4).reshape(rows, 4)
    ws = [s.reshape(rows, 4) for s in W.additive_shares(rng, n, win.reshape(-1).astype(np.uint64))]

    def relu_layer(d_shares, seed):
        """ReLU of shared values on the GPU, checked against the oracle; returns both parties' shares."""
        batch = d_shares[0].shape[0]
        r2 = np.random.default_rng(seed)
        g = W.gen_inputs(r2, n, batch)
        tr = W.triple_shares(r2, n, batch)
        key = GpuBackend().gen("cmp", n, g)
        ys = [to_dev(d) for d in d_shares]
        masked, delta, eps, z = [new(batch) for _ in range(2)], [new(batch) for _ in range(2)], [new(batch) for _ in range(2)], [new(batch) for _ in range(2)]
        for j in (0, 1):
            fss.sign_mask(n, batch, key[j], ys[j], masked[j])
        for j in (0, 1):
            fss.relu_open(j, n, batch, key[j], masked[0], masked[1], ys[j], to_dev(tr.a[j]), to_dev(tr.b[j]), delta[j], eps[j])
        for j in (0, 1):
            fss.relu_finish(j, n, batch, delta[0], delta[1], eps[0], eps[1], to_dev(tr.a[j]), to_dev(tr.b[j]), to_dev(tr.c[j]), z[j])
        got = [host(v) for v in z]
        ok = oracle.gen("cmp", n, g.alpha, g.r, g.seed0, g.seed1)
        om = [oracle.sign_mask(n, ok[j], d_shares[j]) for j in (0, 1)]
        oo = [oracle.relu_open(j, n, ok[j], om[0], om[1], d_shares[j], tr.a[j], tr.b[j]) for j in (0, 1)]
        for j in (0, 1):
            want = oracle.relu_finish(j, n, oo[0][0], oo[1][0], oo[0][1], oo[1][1], tr.a[j], tr.b[j], tr.c[j])
            assert np.array_equal(got[j], want)
        return got

    # level 1: max(x0, x1) and max(x2, x3) in one batch of 2 * rows comparisons
    a = [np.concatenate([s[:, 0], s[:, 2]]) for s in ws]
    b = [np.concatenate([s[:, 1], s[:, 3]]) for s in ws]
    r1 = relu_layer([a[j] - b[j] for j in (0, 1)], seed=1)
    m1 = [b[j] + r1[j] for j in (0, 1)]
    # level 2: max of the two partial maxima
    r2 = relu_layer([m1[j][:rows] - m1[j][rows:] for j in (0, 1)], seed=2)
    out = (m1[0][rows:] + r2[0]) + (m1[1][rows:] + r2[1])
    assert np.array_equal(out, (win.max(axis=1) & 0xFFFFFFFF).astype(np.uint32))
