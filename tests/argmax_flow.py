"""The Argmax / MaxPool protocol flow of the paper (Algorithms 6 and 7) written once over an
abstract backend, so that the oracle tests and the GPU parity tests drive exactly the same
sequence of steps.  A backend provides the per-party primitives; this module only moves
arrays between the two parties (the 'network')."""
from dataclasses import dataclass

import numpy as np

from paper_2006_04593_amd import workloads as W


@dataclass
class ArgmaxMaterial:
    """Dealer material for `rows` vectors of length m."""
    n: int
    rows: int
    m: int
    cmp_gen: W.GenInputs        # rows * m * (m-1) comparison keys
    eq_gen: W.GenInputs         # rows * m equality keys
    triples: W.TripleShares     # rows * m multiplication triples (MaxPool only)


def material(rng, n, rows, m):
    return ArgmaxMaterial(n=n, rows=rows, m=m, cmp_gen=W.gen_inputs(rng, n, rows * m * (m - 1)),
                          eq_gen=W.gen_inputs(rng, n, rows * m), triples=W.triple_shares(rng, n, rows * m))


def argmax(backend, mat, x_shares, keys=None):
    """x_shares: ([rows, m], [rows, m]).  Returns every intermediate of both parties."""
    n, rows, m = mat.n, mat.rows, mat.m
    if keys is None:
        keys = dict(cmp=backend.gen("cmp", n, mat.cmp_gen), eq=backend.gen("eq", n, mat.eq_gen))
    t = {"keys": keys}
    # round 1: masked differences, reveal, comparison shares
    t["masked_cmp"] = [backend.argmax_diff_mask(n, rows, m, keys["cmp"][j], x_shares[j]) for j in (0, 1)]
    t["w"] = [backend.sign_eval(j, n, keys["cmp"][j], t["masked_cmp"][0], t["masked_cmp"][1]) for j in (0, 1)]
    # round 2: counts, masked, reveal, equality shares = one-hot argmax
    t["masked_eq"] = [backend.argmax_count_mask(j, n, rows, m, t["w"][j], keys["eq"][j]) for j in (0, 1)]
    t["onehot"] = [backend.eq_masked_eval(j, n, keys["eq"][j], t["masked_eq"][0], t["masked_eq"][1]) for j in (0, 1)]
    return t


def maxpool(backend, mat, channels, h, w, k, x_shares):
    """x_shares: ([channels, h, w], [channels, h, w]); stride 2, no padding (Algorithm 7)."""
    n, rows, m = mat.n, mat.rows, mat.m
    unrolled = [backend.maxpool_unroll(channels, h, w, k, 2, x_shares[j]) for j in (0, 1)]
    t = argmax(backend, mat, unrolled)
    t["rows"] = unrolled
    tr = mat.triples
    # round 3: inner product of each row with its one-hot argmax
    op = [backend.mul_open(n, unrolled[j], t["onehot"][j], tr.a[j], tr.b[j]) for j in (0, 1)]
    t["delta"] = [op[0][0], op[1][0]]
    t["eps"] = [op[0][1], op[1][1]]
    t["out"] = [backend.dot_finish(j, n, rows, m, t["delta"][0], t["delta"][1], t["eps"][0], t["eps"][1],
                                   tr.a[j], tr.b[j], tr.c[j]) for j in (0, 1)]
    return t


class OracleBackend:
    def __init__(self):
        import oracle
        self.o = oracle

    def gen(self, kind, n, g):
        return self.o.gen(kind, n, g.alpha, g.r, g.seed0, g.seed1)

    def argmax_diff_mask(self, n, rows, m, key, x):
        return self.o.argmax_diff_mask(n, rows, m, key, x)

    def sign_eval(self, j, n, key, m0, m1):
        return self.o.sign_eval(j, n, key, m0, m1)

    def argmax_count_mask(self, j, n, rows, m, w, key):
        return self.o.argmax_count_mask(j, n, rows, m, w, key)

    def eq_masked_eval(self, j, n, key, m0, m1):
        return self.o.eq_masked_eval(j, n, key, m0, m1)

    def maxpool_unroll(self, c, h, w, k, s, x):
        return self.o.maxpool_unroll(c, h, w, k, s, x)

    def mul_open(self, n, u, v, a, b):
        return self.o.mul_open(n, u, v, a, b)

    def dot_finish(self, j, n, rows, m, d0, d1, e0, e1, a, b, c):
        return self.o.dot_finish(j, n, rows, m, d0, d1, e0, e1, a, b, c)
