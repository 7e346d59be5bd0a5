"""Pins for the oracle's Argmax (Algorithm 6) and MaxPool (Algorithm 7): reconstructed values
against plain definitions (numpy), including ties and every pair of a small ring."""
import numpy as np
import pytest

import argmax_flow as F
from paper_2006_04593_amd import workloads as W


def shares_of(rng, n, values):
    flat = values.reshape(-1)
    s0, s1 = W.additive_shares(rng, n, flat.astype(np.int64).astype(np.uint64))
    return s0.reshape(values.shape), s1.reshape(values.shape)


def rec(pair, n):
    return (pair[0] + pair[1]) & np.uint32(W.ring_mask(n))


@pytest.mark.parametrize("n,m", [(16, 2), (16, 4), (32, 9), (32, 10)])
def test_argmax_is_one_hot_of_the_maximum(n, m):
    rng = np.random.default_rng(600 + m)
    rows = 50
    x = W.fixed_point_normal(rng, (rows, m), frac_bits=min(10, n - 14))      # |differences| << 2^n
    x[0] = x[0, 0]                       # a row of all-equal values: every position is an argmax
    x[1, 1] = x[1, 0] = x[1].max() + 1   # a two-way tie at the top
    mat = F.material(rng, n, rows, m)
    t = F.argmax(F.OracleBackend(), mat, shares_of(rng, n, x))
    onehot = rec(t["onehot"], n).reshape(rows, m)
    # counts reconstruct to the number of elements not above x_j
    w = rec(t["w"], n).reshape(rows, m, m - 1)
    assert set(np.unique(w)) <= {0, 1}
    want_w = np.stack([[np.delete(x[r], j) <= x[r, j] for j in range(m)] for r in range(rows)])
    assert (w != want_w).sum() <= 1                              # Sign wrap-around: |d| / 2^n each
    assert np.array_equal(onehot, (w.sum(axis=2) == m - 1).astype(np.uint32))
    agree = (w == want_w).all(axis=(1, 2))
    assert np.array_equal(onehot[agree], (x == x.max(axis=1, keepdims=True)).astype(np.uint32)[agree])
    assert onehot[0].sum() == m and onehot[1].sum() == 2


def test_argmax_every_pair_of_a_small_ring():
    """m = 2 over Z_{2^6}: all 4096 (x_0, x_1) pairs; the identity in terms of the revealed
    comparisons holds for every pair, including those whose difference wraps."""
    n, m = 6, 2
    size = 1 << n
    a, b = np.meshgrid(np.arange(size), np.arange(size), indexing="ij")
    x = np.stack([a.reshape(-1), b.reshape(-1)], axis=1).astype(np.int64)
    rows = x.shape[0]
    rng = np.random.default_rng(66)
    mat = F.material(rng, n, rows, m)
    t = F.argmax(F.OracleBackend(), mat, shares_of(rng, n, x))
    mask = W.ring_mask(n)
    xm = rec(t["masked_cmp"], n).reshape(rows, m, m - 1)[:, :, 0]
    alpha = mat.cmp_gen.alpha.reshape(rows, m)
    d = np.stack([x[:, 1] - x[:, 0], x[:, 0] - x[:, 1]], axis=1)           # pair (j, i): x_i - x_j
    assert np.array_equal(xm, ((d + alpha.astype(np.int64)) & mask).astype(np.uint32))
    le = (xm <= alpha).astype(np.uint32)
    assert np.array_equal(rec(t["w"], n).reshape(rows, m), le)
    assert np.array_equal(rec(t["onehot"], n).reshape(rows, m), (le == 1).astype(np.uint32))


@pytest.mark.parametrize("k,h", [(2, 8), (3, 9)])
def test_maxpool_equals_plain_maxpool(k, h):
    n, channels, w = 32, 3, h + 2
    rng = np.random.default_rng(700 + k)
    x = W.fixed_point_normal(rng, (channels, h, w))
    oh, ow = (h - k) // 2 + 1, (w - k) // 2 + 1
    rows, m = channels * oh * ow, k * k
    mat = F.material(rng, n, rows, m)
    t = F.maxpool(F.OracleBackend(), mat, channels, h, w, k, shares_of(rng, n, x))
    # the unrolled rows reconstruct to the windows
    win = np.stack([x[c, 2 * i:2 * i + k, 2 * j:2 * j + k].reshape(-1) for c in range(channels) for i in range(oh) for j in range(ow)])
    assert np.array_equal(rec(t["rows"], n).reshape(rows, m), (win & 0xFFFFFFFF).astype(np.uint32))
    onehot = rec(t["onehot"], n).reshape(rows, m)
    out = rec(t["out"], n)
    # the inner product identity, whatever the one-hot vector is
    assert np.array_equal(out, ((win * onehot.astype(np.int64)).sum(axis=1) & 0xFFFFFFFF).astype(np.uint32))
    # and with a unique maximum per window that is the plain max-pool
    unique = (win == win.max(axis=1, keepdims=True)).sum(axis=1) == 1
    good = unique & (onehot.sum(axis=1) == 1)
    assert good.mean() > 0.9
    assert np.array_equal(out[good], (win.max(axis=1)[good] & 0xFFFFFFFF).astype(np.uint32))


@pytest.mark.parametrize("n", [5, 8, 32])
def test_equality_on_shared_inputs(n):
    """The wrapper lines of Algorithm 2: publish [[alpha]] + [[y]], reveal, evaluate -> 1{y = 0}."""
    import oracle
    rng = np.random.default_rng(40 + n)
    size = 1 << min(n, 10)
    y = np.arange(size, dtype=np.uint64) if n <= 10 else np.where(rng.random(size) < 0.3, 0, W.uniform_ring(rng, n, size)).astype(np.uint64)
    g = W.gen_inputs(rng, n, size)
    ys = W.additive_shares(rng, n, y)
    k = oracle.gen("eq", n, g.alpha, g.r, g.seed0, g.seed1)
    m = [oracle.eq_mask(n, k[j], ys[j]) for j in (0, 1)]
    assert np.array_equal(rec(m, n), ((y + g.alpha) & W.ring_mask(n)).astype(np.uint32))
    o = [oracle.eq_masked_eval(j, n, k[j], m[0], m[1]) for j in (0, 1)]
    assert np.array_equal(rec(o, n), (y == 0).astype(np.uint32))
