#!/usr/bin/env python3
"""Generator of the Boolean circuit for the AES S-box used by the bit-plane AES engine.

Writes `aes_sbox_circuit.inc` (beside this file): a straight-line sequence of two- and
three-input bitwise operations that maps the eight bit planes of a byte to the eight bit
planes of S(byte).  Run it again after changing anything here; the result is checked
exhaustively (all 256 byte values) before it is written.

Construction (from the definition of the S-box in FIPS-197, section 5.1.1: multiplicative
inverse in GF(2^8) followed by an affine map), using the standard composite-field method:

  GF(2^8) (AES polynomial x^8+x^4+x^3+x+1)  ~  GF(2^4)[y] / (y^2 + y + lam),
  GF(2^4) = GF(2)[z] / (z^4 + z + 1).

  An element a*y + b has inverse (a*y + (a + b)) * d^-1 with d = a^2*lam + a*b + b^2 in GF(2^4),
  so one byte inversion costs three GF(2^4) multiplications, one GF(2^4) inversion and a few
  linear maps.  The change of basis into the composite field and back (with the affine map
  folded in) are 8x8 bit matrices.

All choices that do not change the function (lam, which root of the AES polynomial defines
the isomorphism) are searched for the smallest operation count.  Linear parts are shrunk with
a greedy shared-subexpression pass; single-use intermediate results are then fused into
three-input operations (gfx950 has v_bitop3_b32, any 3-input bitwise function in one
instruction).
"""
import itertools
import os
import sys

# ----------------------------------------------------------------------------- fields

def gf256_mul(a, b):
    p = 0
    for _ in range(8):
        if b & 1:
            p ^= a
        hi = a & 0x80
        a = (a << 1) & 0xFF
        if hi:
            a ^= 0x1B
        b >>= 1
    return p


def gf256_inv(a):
    if a == 0:
        return 0
    r = 1
    for _ in range(254):
        r = gf256_mul(r, a)
    return r


def aes_sbox(v):
    x = gf256_inv(v)
    out = 0
    for i in range(8):
        bit = ((x >> i) ^ (x >> ((i + 4) % 8)) ^ (x >> ((i + 5) % 8)) ^ (x >> ((i + 6) % 8)) ^ (x >> ((i + 7) % 8)) ^ (0x63 >> i)) & 1
        out |= bit << i
    return out


def gf16_mul(a, b):      # z^4 = z + 1
    p = 0
    for i in range(4):
        if (b >> i) & 1:
            p ^= a << i
    for k in (6, 5, 4):
        if (p >> k) & 1:
            p ^= (1 << k) | (0b0011 << (k - 4))
    return p & 0xF


def gf16_inv(a):
    if a == 0:
        return 0
    for b in range(1, 16):
        if gf16_mul(a, b) == 1:
            return b


class Tower:
    """GF(16)[y]/(y^2+y+lam); element = (hi << 4) | lo meaning hi*y + lo."""

    def __init__(self, lam):
        self.lam = lam

    def mul(self, u, v):
        a, b = u >> 4, u & 15
        c, d = v >> 4, v & 15
        ac = gf16_mul(a, c)
        hi = gf16_mul(a, d) ^ gf16_mul(b, c) ^ ac           # y^2 = y + lam
        lo = gf16_mul(b, d) ^ gf16_mul(ac, self.lam)
        return (hi << 4) | lo


def irreducible_lams():
    out = []
    for lam in range(1, 16):
        if all(gf16_mul(t, t) ^ t ^ lam for t in range(16)):   # y^2+y+lam has no root in GF(16)
            out.append(lam)
    return out


def isomorphisms(lam):
    """All 8x8 bit matrices M (as 8 column images) mapping the AES basis to the tower field."""
    T = Tower(lam)
    res = []
    for g in range(2, 256):
        # is g a root of x^8 + x^4 + x^3 + x + 1 in the tower field?
        pw = [1]
        for _ in range(8):
            pw.append(T.mul(pw[-1], g))
        if pw[8] ^ pw[4] ^ pw[3] ^ pw[1] ^ pw[0] == 0:
            res.append(pw[:8])          # image of x^k is g^k
    return res


def apply_cols(cols, v):
    r = 0
    for k in range(8):
        if (v >> k) & 1:
            r ^= cols[k]
    return r


def invert_cols(cols):
    table = {apply_cols(cols, v): v for v in range(256)}
    assert len(table) == 256
    return [table[1 << k] for k in range(8)]


# ----------------------------------------------------------------------------- circuits

class Circuit:
    """Straight-line program over GF(2).  Nodes: ('in', k) | ('xor', a, b) | ('and', a, b) |
    ('not', a) | ('lut3', tt, a, b, c).  Values are simulated on all 256 inputs at once."""

    def __init__(self):
        self.nodes = []
        self.cache = {}
        self.inputs = [self._add(('in', k)) for k in range(8)]

    def _add(self, node):
        if node in self.cache:
            return self.cache[node]
        self.nodes.append(node)
        self.cache[node] = len(self.nodes) - 1
        return len(self.nodes) - 1

    def xor(self, a, b):
        if a == b:
            raise ValueError("xor of a node with itself")
        if a > b:
            a, b = b, a
        return self._add(('xor', a, b))

    def and_(self, a, b):
        if a > b:
            a, b = b, a
        return self._add(('and', a, b))

    def not_(self, a):
        return self._add(('not', a))

    def xor_many(self, xs):
        xs = list(xs)
        assert xs
        acc = xs[0]
        for x in xs[1:]:
            acc = self.xor(acc, x)
        return acc


ALL = (1 << 256) - 1
IN_MASKS = [sum(1 << v for v in range(256) if (v >> k) & 1) for k in range(8)]


def simulate(nodes):
    val = []
    for nd in nodes:
        if nd[0] == 'in':
            val.append(IN_MASKS[nd[1]])
        elif nd[0] == 'xor':
            val.append(val[nd[1]] ^ val[nd[2]])
        elif nd[0] == 'and':
            val.append(val[nd[1]] & val[nd[2]])
        elif nd[0] == 'not':
            val.append(val[nd[1]] ^ ALL)
        elif nd[0] == 'lut3':
            tt, a, b, c = nd[1:]
            va, vb, vc = val[a], val[b], val[c]
            r = 0
            for idx in range(8):
                if (tt >> idx) & 1:
                    ta = va if idx & 4 else va ^ ALL
                    tb = vb if idx & 2 else vb ^ ALL
                    tc = vc if idx & 1 else vc ^ ALL
                    r |= ta & tb & tc
            val.append(r)
        else:
            raise ValueError(nd)
    return val


def linear_layer(circ, in_nodes, rows):
    """rows[i] = bit mask over in_nodes; returns output nodes.  Greedy pair sharing (Paar)."""
    n = len(in_nodes)
    nodes = list(in_nodes)
    rows = [r for r in rows]
    while True:
        best, best_pair = 1, None
        for i, j in itertools.combinations(range(len(nodes)), 2):
            m = (1 << i) | (1 << j)
            cnt = sum(1 for r in rows if r & m == m)
            if cnt > best:
                best, best_pair = cnt, (i, j)
        if best_pair is None:
            break
        i, j = best_pair
        new = circ.xor(nodes[i], nodes[j])
        nodes.append(new)
        k = len(nodes) - 1
        m = (1 << i) | (1 << j)
        rows = [(r & ~m) | (1 << k) if r & m == m else r for r in rows]
    outs = []
    for r in rows:
        terms = [nodes[k] for k in range(len(nodes)) if (r >> k) & 1]
        outs.append(circ.xor_many(terms) if terms else None)
    return outs


def gf16_mul_circuit(c, p, q):
    """p, q: lists of 4 nodes (bit 0 first).  Schoolbook product, z^4 = z + 1."""
    prod = {}
    for i in range(4):
        for j in range(4):
            prod[(i, j)] = c.and_(p[i], q[j])
    h4 = c.xor_many([prod[(1, 3)], prod[(2, 2)], prod[(3, 1)]])
    h5 = c.xor(prod[(2, 3)], prod[(3, 2)])
    h6 = prod[(3, 3)]
    c0 = c.xor(prod[(0, 0)], h4)
    c1 = c.xor_many([prod[(0, 1)], prod[(1, 0)], h4, h5])
    c2 = c.xor_many([prod[(0, 2)], prod[(1, 1)], prod[(2, 0)], h5, h6])
    c3 = c.xor_many([prod[(0, 3)], prod[(1, 2)], prod[(2, 1)], prod[(3, 0)], h6])
    return [c0, c1, c2, c3]


def gf16_linear(c, p, fn):
    """Apply a GF(2)-linear map fn on GF(16) to the 4 nodes p."""
    cols = [fn(1 << k) for k in range(4)]
    rows = [sum(((cols[k] >> i) & 1) << k for k in range(4)) for i in range(4)]
    return linear_layer(c, p, rows)


def gf16_inv_circuit(c, d):
    """d^-1 = d^14 = d^2 * d^4 * d^8 would cost two multiplications; instead synthesise the
    4-bit function from its algebraic normal form with shared monomials."""
    # ANF of each output bit
    anf = []
    for ob in range(4):
        coeffs = {}
        tt = [(gf16_inv(v) >> ob) & 1 for v in range(16)]
        # Moebius transform
        a = tt[:]
        for i in range(4):
            for v in range(16):
                if v & (1 << i):
                    a[v] ^= a[v ^ (1 << i)]
        anf.append([m for m in range(16) if a[m]])
    mono = {}

    def monomial(m):
        if m in mono:
            return mono[m]
        bits = [k for k in range(4) if (m >> k) & 1]
        if len(bits) == 1:
            node = d[bits[0]]
        else:
            # split off the highest variable; reuse smaller monomials
            node = c.and_(monomial(m & ~(1 << bits[-1])), d[bits[-1]])
        mono[m] = node
        return node

    outs = []
    for ob in range(4):
        assert 0 not in anf[ob]
        outs.append(c.xor_many([monomial(m) for m in anf[ob]]))
    return outs


def build(lam, iso_cols):
    """S-box circuit for one (lam, isomorphism) choice."""
    c = Circuit()
    # AES basis -> tower basis
    rows_in = [sum(((iso_cols[k] >> i) & 1) << k for k in range(8)) for i in range(8)]
    t = linear_layer(c, c.inputs, rows_in)
    b, a = t[0:4], t[4:8]                  # value = a*y + b
    ab = gf16_mul_circuit(c, a, b)
    a2l = gf16_linear(c, a, lambda v: gf16_mul(gf16_mul(v, v), lam))
    b2 = gf16_linear(c, b, lambda v: gf16_mul(v, v))
    d = [c.xor_many([x for x in (a2l[i], ab[i], b2[i]) if x is not None]) for i in range(4)]
    dinv = gf16_inv_circuit(c, d)
    apb = [c.xor(a[i], b[i]) for i in range(4)]
    hi = gf16_mul_circuit(c, a, dinv)
    lo = gf16_mul_circuit(c, apb, dinv)
    inv_nodes = lo + hi
    # tower basis -> AES basis, then the affine map's linear part; constant 0x63 = output inversions
    back = invert_cols(iso_cols)

    def affine_lin(v):
        r = 0
        for i in range(8):
            bit = ((v >> i) ^ (v >> ((i + 4) % 8)) ^ (v >> ((i + 5) % 8)) ^ (v >> ((i + 6) % 8)) ^ (v >> ((i + 7) % 8))) & 1
            r |= bit << i
        return r

    cols_out = [affine_lin(back[k]) for k in range(8)]
    rows_out = [sum(((cols_out[k] >> i) & 1) << k for k in range(8)) for i in range(8)]
    lin = linear_layer(c, inv_nodes, rows_out)
    outs = []
    for i in range(8):
        outs.append(c.not_(lin[i]) if (0x63 >> i) & 1 else lin[i])
    return c, outs


# ----------------------------------------------------------------------------- fusion into 3-input ops

def prune(nodes, outs):
    """Drop dead nodes, renumber."""
    live = set()
    stack = list(outs)
    while stack:
        k = stack.pop()
        if k in live:
            continue
        live.add(k)
        nd = nodes[k]
        if nd[0] in ('xor', 'and'):
            stack += [nd[1], nd[2]]
        elif nd[0] == 'not':
            stack.append(nd[1])
        elif nd[0] == 'lut3':
            stack += list(nd[2:])
    order = sorted(live)
    remap = {k: i for i, k in enumerate(order)}
    new = []
    for k in order:
        nd = nodes[k]
        if nd[0] == 'in':
            new.append(nd)
        elif nd[0] in ('xor', 'and'):
            new.append((nd[0], remap[nd[1]], remap[nd[2]]))
        elif nd[0] == 'not':
            new.append(('not', remap[nd[1]]))
        else:
            new.append(('lut3', nd[1]) + tuple(remap[x] for x in nd[2:]))
    return new, [remap[o] for o in outs]


def truth3(fn):
    """8-bit truth table with a = 0xF0, b = 0xCC, c = 0xAA."""
    tt = 0
    for idx in range(8):
        a, b, c = (idx >> 2) & 1, (idx >> 1) & 1, idx & 1
        if fn(a, b, c):
            tt |= 1 << idx
    return tt


def fuse(nodes, outs):
    """Absorb single-use producers into their consumer while the consumer stays a function of
    at most three distinct nodes; such a consumer becomes one three-input operation."""
    changed = True
    while changed:
        changed = False
        uses = [0] * len(nodes)
        for nd in nodes:
            if nd[0] in ('xor', 'and'):
                uses[nd[1]] += 1
                uses[nd[2]] += 1
            elif nd[0] == 'not':
                uses[nd[1]] += 1
            elif nd[0] == 'lut3':
                for x in set(nd[2:]):
                    uses[x] += 1
        for o in outs:
            uses[o] += 1

        def node_fn(k):
            """(operand list, function of an env {node: bit}) for node k itself."""
            nd = nodes[k]
            if nd[0] == 'xor':
                return [nd[1], nd[2]], (lambda env, a=nd[1], b=nd[2]: env[a] ^ env[b])
            if nd[0] == 'and':
                return [nd[1], nd[2]], (lambda env, a=nd[1], b=nd[2]: env[a] & env[b])
            if nd[0] == 'not':
                return [nd[1]], (lambda env, a=nd[1]: 1 - env[a])
            if nd[0] == 'lut3':
                tt, a, b, c = nd[1:]
                return [a, b, c], (lambda env, tt=tt, a=a, b=b, c=c: (tt >> ((env[a] << 2) | (env[b] << 1) | env[c])) & 1)
            return None

        for k in range(len(nodes)):
            if nodes[k][0] == 'in':
                continue
            ops, fn = node_fn(k)
            leaves = list(dict.fromkeys(ops))
            absorbed = False
            progress = True
            while progress:
                progress = False
                for x in list(leaves):
                    if nodes[x][0] == 'in' or uses[x] != 1:
                        continue
                    xops, xfn = node_fn(x)
                    cand = [l for l in leaves if l != x]
                    for o in xops:
                        if o not in cand:
                            cand.append(o)
                    if len(cand) > 3:
                        continue
                    # substitute x
                    fn = (lambda env, fn=fn, xfn=xfn, x=x: fn({**env, x: xfn(env)}))
                    leaves = cand
                    absorbed = True
                    progress = True
                    break
            if not absorbed:
                continue
            L = leaves + [leaves[0]] * (3 - len(leaves))
            tt = 0
            for idx in range(8):
                vals = ((idx >> 2) & 1, (idx >> 1) & 1, idx & 1)
                env = {}
                for node, v in zip(L, vals):
                    env.setdefault(node, v)
                if fn(env):
                    tt |= 1 << idx
            nodes[k] = ('lut3', tt, L[0], L[1], L[2])
            changed = True
            nodes, outs = prune(nodes, outs)
            break
    return nodes, outs


def count_ops(nodes):
    return sum(1 for nd in nodes if nd[0] != 'in')


def verify(nodes, outs):
    val = simulate(nodes)
    for v in range(256):
        got = sum(((val[outs[i]] >> v) & 1) << i for i in range(8))
        if got != aes_sbox(v):
            return False
    return True


def emit(nodes, outs, path, note):
    lines = []
    lines.append("// GENERATED by gen_sbox_circuit.py -- do not edit.  " + note)
    lines.append("// AES S-box on bit planes: x0..x7 are the planes of bit 0..7 of the input bytes,")
    lines.append("// y0..y7 the planes of S(input).  FSS_B3(tt, a, b, c) is a three-input bitwise")
    lines.append("// function with truth table tt (a = 0xF0, b = 0xCC, c = 0xAA).")
    name = {}
    tmp = 0
    body = []
    for k, nd in enumerate(nodes):
        if nd[0] == 'in':
            name[k] = f"x{nd[1]}"
            continue
        nm = f"t{tmp}"
        tmp += 1
        name[k] = nm
        if nd[0] == 'xor':
            body.append(f"const W {nm} = {name[nd[1]]} ^ {name[nd[2]]};")
        elif nd[0] == 'and':
            body.append(f"const W {nm} = {name[nd[1]]} & {name[nd[2]]};")
        elif nd[0] == 'not':
            body.append(f"const W {nm} = ~{name[nd[1]]};")
        else:
            tt, a, b, c = nd[1:]
            body.append(f"const W {nm} = FSS_B3(0x{tt:02x}, {name[a]}, {name[b]}, {name[c]});")
    lines += body
    for i in range(8):
        lines.append(f"y{i} = {name[outs[i]]};")
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")


def main():
    best = None
    for lam in irreducible_lams():
        for iso in isomorphisms(lam):
            c, outs = build(lam, iso)
            nodes, outs2 = prune(c.nodes, outs)
            assert verify(nodes, outs2), "construction is wrong"
            plain = count_ops(nodes)
            fnodes, fouts = fuse(list(nodes), list(outs2))
            assert verify(fnodes, fouts), "fusion broke the circuit"
            ops = count_ops(fnodes)
            if best is None or ops < best[0]:
                best = (ops, plain, lam, iso, fnodes, fouts)
    ops, plain, lam, iso, nodes, outs = best
    note = f"{ops} operations ({plain} two-input gates before fusion); lam = {lam}, root = 0x{iso[1]:02x}."
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "aes_sbox_circuit.inc")
    emit(nodes, outs, out, note)
    print(note, "->", out)


if __name__ == "__main__":
    main()
