"""Pins for the oracle's Sign protocol (Algorithm 5) and ReLU (section 4.2): plain
definitions on reconstructed values, for every input of a small ring and for the
fixed-point activations of the benchmark shape."""
import numpy as np
import pytest

import oracle
from paper_2006_04593_amd import workloads as W


def run_relu(n, y, seed):
    """Both parties through mask -> open -> finish; returns the reconstructed output and x, alpha."""
    rng = np.random.default_rng(seed)
    batch = y.shape[0]
    g = W.gen_inputs(rng, n, batch)
    ri = W.relu_inputs(rng, n, y)
    k = oracle.gen("cmp", n, g.alpha, g.r, g.seed0, g.seed1)
    masked = [oracle.sign_mask(n, k[j], ri.y_share[j]) for j in (0, 1)]
    opened = [oracle.relu_open(j, n, k[j], masked[0], masked[1], ri.y_share[j], ri.tri_a[j], ri.tri_b[j]) for j in (0, 1)]
    z = [oracle.relu_finish(j, n, opened[0][0], opened[1][0], opened[0][1], opened[1][1], ri.tri_a[j], ri.tri_b[j], ri.tri_c[j])
         for j in (0, 1)]
    mask = np.uint32(W.ring_mask(n))
    x = (masked[0] + masked[1]) & mask
    sign = [oracle.sign_eval(j, n, k[j], masked[0], masked[1]) for j in (0, 1)]
    return (z[0] + z[1]) & mask, x, g.alpha, (sign[0] + sign[1]) & mask, masked, opened, ri


@pytest.mark.parametrize("n", [4, 8, 12])
def test_every_activation_value_of_a_small_ring(n):
    """z_0 + z_1 = y * (1 - 1{x <= alpha}) with x = y + alpha mod 2^n -- an identity in Z_{2^n}
    that holds for every y, including the wrap-around cases where Sign differs from 1{y <= 0}."""
    size = 1 << n
    y = np.arange(size, dtype=np.int64)                     # every ring element, read as two's complement
    rec, x, alpha, sign, masked, opened, ri = run_relu(n, y, seed=50 + n)
    mask = W.ring_mask(n)
    assert np.array_equal(x, ((y + alpha.astype(np.int64)) & mask).astype(np.uint32))          # the reveal
    le = (x <= alpha).astype(np.uint32)
    assert np.array_equal(sign, le)                                                             # Algorithm 5
    assert np.array_equal(rec, ((y.astype(np.uint64) * (1 - le)) & mask).astype(np.uint32))     # the product
    # where the sum did not wrap, that is ReLU of the signed value
    signed = np.where(y >= size // 2, y - size, y)
    ok = le == (signed <= 0)
    assert ok.mean() > 0.4
    assert np.array_equal(rec[ok], (np.maximum(signed, 0)[ok] & mask).astype(np.uint32))


def test_relu_on_fixed_point_activations_n32():
    rng = np.random.default_rng(77)
    y = W.fixed_point_normal(rng, 4096)
    rec, x, alpha, sign, masked, opened, ri = run_relu(32, y, seed=78)
    fail = sign != (y <= 0)
    assert fail.sum() <= 1                                   # |y| / 2^32 per element
    want = (np.maximum(y, 0) & 0xFFFFFFFF).astype(np.uint32)
    assert np.array_equal(rec[~fail], want[~fail])


def test_messages_are_what_the_protocol_says():
    """delta and eps reconstruct to y - a and 1{y > 0} - b; the masked shares to y + alpha."""
    n = 16
    rng = np.random.default_rng(5)
    y = W.fixed_point_normal(rng, 512, frac_bits=6)
    rec, x, alpha, sign, masked, opened, ri = run_relu(n, y, seed=6)
    mask = np.uint32(W.ring_mask(n))
    a = (ri.tri_a[0] + ri.tri_a[1]) & mask
    b = (ri.tri_b[0] + ri.tri_b[1]) & mask
    c = (ri.tri_c[0] + ri.tri_c[1]) & mask
    assert np.array_equal(c, (a.astype(np.uint64) * b.astype(np.uint64)).astype(np.uint32) & mask)
    delta = (opened[0][0] + opened[1][0]) & mask
    eps = (opened[0][1] + opened[1][1]) & mask
    yy = (y & int(mask)).astype(np.uint32)
    assert np.array_equal(delta, (yy - a) & mask)
    assert np.array_equal(eps, ((1 - sign) - b) & mask)


def test_sign_mask_uses_the_keys_alpha_share():
    n, batch = 32, 100
    rng = np.random.default_rng(9)
    g = W.gen_inputs(rng, n, batch)
    k0, k1 = oracle.gen("cmp", n, g.alpha, g.r, g.seed0, g.seed1)
    ys = W.uniform_ring(rng, n, batch)
    assert np.array_equal(oracle.sign_mask(n, k0, ys), ys + g.r)
    assert np.array_equal(oracle.sign_mask(n, k1, ys), ys + (g.alpha - g.r))
