"""Do the pins bite?  Each case plants ONE plausible mistake (a dropped term, a wrong sign
or index, swapped operands) in a temporary copy of the oracle's C source, builds it on the
CPU, and checks that the pins of test_oracle_aes / test_oracle_fss reject it.  The mistakes
live only in the temporary copy; nothing here touches the GPU."""
import os
import subprocess

import numpy as np
import pytest

import oracle
from paper_2006_04593_amd import workloads as W

SRC = os.path.join(os.path.dirname(oracle.__file__), "fss_oracle.c")

# (name, text in the oracle, replacement, which pin must fail)
MUTANTS = [
    ("leaf_sign_dropped", "if (tau_next[1]) cw_leaf = (0u - cw_leaf) & mask;", "", "cmp"),
    ("leaf_operands_swapped", "cw_leaf = ((uint32_t)a - sigma_next[0] + sigma_next[1]) & mask;",
     "cw_leaf = ((uint32_t)a + sigma_next[0] - sigma_next[1]) & mask;", "cmp"),
    ("leaf_alpha_bit_dropped", "cw_leaf = ((uint32_t)a - sigma_next[0] + sigma_next[1]) & mask;",
     "cw_leaf = (0u - sigma_next[0] + sigma_next[1]) & mask;", "cmp"),
    ("t_cw_sides_swapped", "t_cw[L] = g[0].t[L] ^ g[1].t[L] ^ a ^ 1;", "t_cw[L] = g[0].t[L] ^ g[1].t[L] ^ a;", "both"),
    ("tau_cw_sides_swapped", "tau_cw[L] = g[0].tau[L] ^ g[1].tau[L] ^ a;", "tau_cw[L] = g[0].tau[L] ^ g[1].tau[L] ^ a ^ 1;", "cmp"),
    ("sigma_cw_from_lose_side", "sigma_cw = g[0].sigma[keep] ^ g[1].sigma[keep];", "sigma_cw = g[0].sigma[lose] ^ g[1].sigma[lose];", "cmp"),
    ("s_cw_from_keep_side", "s_cw[k] = g[0].s[lose][k] ^ g[1].s[lose][k];", "s_cw[k] = g[0].s[keep][k] ^ g[1].s[keep][k];", "both"),
    ("gen_walks_lose_branch", "memcpy(next, g[j].s[keep], 16);", "memcpy(next, g[j].s[lose], 16);", "both"),
    ("bits_lsb_first", "return (int)((x >> (n - i)) & 1u);", "return (int)((x >> (i - 1)) & 1u);", "cmp"),
    ("final_term_dropped", "acc = (acc + out_last) & mask;", "", "both"),
    ("final_cw_sign_dropped", "if (t[1]) last = (0u - last) & mask;", "", "both"),
    ("final_cw_constant_dropped", "uint32_t last = (1u - conv(s[0], n) + conv(s[1], n)) & mask;",
     "uint32_t last = (0u - conv(s[0], n) + conv(s[1], n)) & mask;", "both"),
    ("party_sign_dropped", "if (party == 1) acc = (0u - acc) & mask;", "", "both"),
    ("eval_starts_with_t_zero", "int t = party;                                   /* t^(1) = j */", "int t = 0;", "both"),
    ("eval_tau_uses_other_side", "int tau = g.tau[b] ^ (t & ctrl_bit(k, e, 2 + b, i));", "int tau = g.tau[b] ^ (t & ctrl_bit(k, e, 3 - b, i));", "cmp"),
    ("eval_t_uses_other_side", "int t_next = g.t[b] ^ (t & ctrl_bit(k, e, b, i));", "int t_next = g.t[b] ^ (t & ctrl_bit(k, e, 1 - b, i));", "both"),
    ("leaf_added_without_tau_gate", "uint32_t out_i = ((tau ? le32(leaf_at(k, i, e)) : 0u) + sigma) & mask;",
     "uint32_t out_i = (le32(leaf_at(k, i, e)) + sigma) & mask;", "cmp"),
    ("shiftrows_wrong_direction", "tmp[4 * c + r] = st[4 * ((c + r) % 4) + r];", "tmp[4 * c + r] = st[4 * ((c + 4 - r) % 4) + r];", "aes"),
    ("mixcolumns_coefficients_swapped", "st[4 * c + 0] = g_mul2[a[0]] ^ g_mul3[a[1]] ^ a[2] ^ a[3];",
     "st[4 * c + 0] = g_mul3[a[0]] ^ g_mul2[a[1]] ^ a[2] ^ a[3];", "aes"),
    ("affine_constant_wrong", "(0x63 >> i)) & 1;", "(0x36 >> i)) & 1;", "aes"),
    ("mmo_feedforward_dropped", "out[i] = enc[i] ^ seed[i];", "out[i] = enc[i];", "prg"),
    ("relu_public_product_dropped", "if (party == 0) z += delta * eps;", "", "relu"),
    ("relu_constant_one_dropped", "uint32_t v = ((party == 0 ? 1u : 0u) - w) & mask;", "uint32_t v = (0u - w) & mask;", "relu"),
    ("relu_eps_sign", "eps[e] = (v - tri_b[e]) & mask;", "eps[e] = (v + tri_b[e]) & mask;", "relu"),
    ("relu_triple_operands_swapped", "uint32_t z = delta * tri_b[e] + eps * tri_a[e] + tri_c[e];",
     "uint32_t z = delta * tri_a[e] + eps * tri_b[e] + tri_c[e];", "relu"),
    ("argmax_pair_index_off", "const int i = t < j ? t : t + 1;", "const int i = t;", "argmax"),
    ("argmax_difference_reversed", "const uint32_t y = x_share[r * (size_t)m + (size_t)i] - x_share[r * (size_t)m + (size_t)j];",
     "const uint32_t y = x_share[r * (size_t)m + (size_t)j] - x_share[r * (size_t)m + (size_t)i];", "argmax"),
    ("argmax_count_constant", "if (party == 0) sum -= (uint32_t)(m - 1);", "if (party == 0) sum -= (uint32_t)m;", "argmax"),
    ("dot_public_product_dropped", "if (party == 0) acc += delta * eps;", "", "argmax"),
    ("unroll_stride_ignored", "rows[out++] = x_share[(c * (size_t)h + (size_t)(oy * s + dy)) * (size_t)w + (size_t)(ox * s + dx)];",
     "rows[out++] = x_share[(c * (size_t)h + (size_t)(oy + dy)) * (size_t)w + (size_t)(ox + dx)];", "argmax"),
    ("eq_mask_drops_alpha", "masked[e] = (le32(k.alpha_share + 4 * e) + y_share[e]) & mask;",
     "masked[e] = y_share[e] & mask;", "eqshared"),
    ("sigma_tau_block_under_key_1", "oracle_prg(3, seed, w);", "oracle_prg(1, seed, w);", "layout"),
    ("sigma_words_swapped", "e->sigma[L] = le32(w + 0) & ring_mask(n);\n        e->sigma[R] = le32(w + 4) & ring_mask(n);",
     "e->sigma[L] = le32(w + 4) & ring_mask(n);\n        e->sigma[R] = le32(w + 0) & ring_mask(n);", "layout"),
    ("children_under_swapped_keys", "oracle_prg(1 + b, seed, blk);", "oracle_prg(2 - b, seed, blk);", "layout"),
    ("conv_reads_another_word", "return le32(s + 12) & ring_mask(n); }", "return le32(s + 8) & ring_mask(n); }", "layout"),
    ("final_cw_from_other_party_bit", "if (t[1]) last = (0u - last) & mask;", "if (t[0]) last = (0u - last) & mask;", "both"),
    ("final_term_reads_another_plane", "uint32_t out_last = ((t ? le32(k->last + 4 * e) : 0u) + conv(s, n)) & mask;",
     "uint32_t out_last = ((t ? le32(k->last + 4 * e) : 0u) + (le32(s + 4) & mask)) & mask;", "both"),
    ("sign_mask_subtracts", "masked[e] = (y_share[e] + le32(k.alpha_share + 4 * e)) & mask;",
     "masked[e] = (y_share[e] - le32(k.alpha_share + 4 * e)) & mask;", "relu"),
]


def build_mutant(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"{name}: pattern must occur exactly once in the oracle source"
    src = tmp_path / f"{name}.c"
    so = tmp_path / f"lib{name}.so"
    src.write_text(text.replace(old, new))
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", str(src), "-o", str(so)], check=True)
    return oracle.load(str(so))


def reconstruction_holds(kind, n=8):
    rng = np.random.default_rng(31337)
    alphas = np.concatenate([W.edge_inputs(n), W.uniform_ring(rng, n, 10)])
    g = W.gen_inputs(rng, n, len(alphas), alpha=alphas)
    k0, k1 = oracle.gen(kind, n, g.alpha, g.r, g.seed0, g.seed1)
    xs = np.arange(1 << n, dtype=np.uint32)
    for e, a in enumerate(g.alpha):
        rec = (oracle.eval_all_x(kind, 0, n, g.batch, k0, e) + oracle.eval_all_x(kind, 1, n, g.batch, k1, e)) & np.uint32(W.ring_mask(n))
        want = ((xs <= a) if kind == "cmp" else (xs == a)).astype(np.uint32)
        if not np.array_equal(rec, want):
            return False
    return True


def aes_known_answer_holds():
    return oracle.aes128_encrypt(bytes(range(16)), bytes.fromhex("00112233445566778899aabbccddeeff")).hex() == \
        "69c4e0d86a7b0430d8cdb78070b4c55a"


def prg_definition_holds():
    s = bytes(range(2, 34, 2))
    enc = oracle.aes128_encrypt(oracle.prg_key(2), s)
    return oracle.prg(2, s) == bytes(a ^ b for a, b in zip(enc, s))


def relu_identity_holds(n=8):
    """z_0 + z_1 = y (1 - 1{y + alpha <= alpha}) for every y, and the reveal is y + alpha."""
    size = 1 << n
    y = np.arange(size, dtype=np.int64)
    rng = np.random.default_rng(4242)
    g = W.gen_inputs(rng, n, size)
    ri = W.relu_inputs(rng, n, y)
    k = oracle.gen("cmp", n, g.alpha, g.r, g.seed0, g.seed1)
    masked = [oracle.sign_mask(n, k[j], ri.y_share[j]) for j in (0, 1)]
    op = [oracle.relu_open(j, n, k[j], masked[0], masked[1], ri.y_share[j], ri.tri_a[j], ri.tri_b[j]) for j in (0, 1)]
    z = [oracle.relu_finish(j, n, op[0][0], op[1][0], op[0][1], op[1][1], ri.tri_a[j], ri.tri_b[j], ri.tri_c[j]) for j in (0, 1)]
    mask = W.ring_mask(n)
    x = (masked[0] + masked[1]) & np.uint32(mask)
    if not np.array_equal(x, ((y + g.alpha.astype(np.int64)) & mask).astype(np.uint32)):
        return False
    le = (x <= g.alpha).astype(np.uint64)
    return np.array_equal((z[0] + z[1]) & np.uint32(mask), ((y.astype(np.uint64) * (1 - le)) & mask).astype(np.uint32))


def maxpool_holds():
    import argmax_flow as F
    n, channels, h, w, k = 32, 2, 6, 8, 2
    rng = np.random.default_rng(99)
    x = W.fixed_point_normal(rng, (channels, h, w))
    x[0, 0, 0] = x[0, 0, 1] = x[0, :2, :2].max() + 5          # a tie inside the first window
    oh, ow = (h - k) // 2 + 1, (w - k) // 2 + 1
    rows, m = channels * oh * ow, k * k
    mat = F.material(rng, n, rows, m)
    s0, s1 = W.additive_shares(rng, n, x.reshape(-1).astype(np.int64).astype(np.uint64))
    t = F.maxpool(F.OracleBackend(), mat, channels, h, w, k, (s0.reshape(x.shape), s1.reshape(x.shape)))
    win = np.stack([x[c, 2 * i:2 * i + k, 2 * j:2 * j + k].reshape(-1) for c in range(channels) for i in range(oh) for j in range(ow)])
    onehot = (t["onehot"][0] + t["onehot"][1]).reshape(rows, m)
    out = t["out"][0] + t["out"][1]
    want_hot = (win == win.max(axis=1, keepdims=True)).astype(np.uint32)
    want = ((win * want_hot).sum(axis=1) & 0xFFFFFFFF).astype(np.uint32)
    return np.array_equal(onehot, want_hot) and np.array_equal(out, want)


def shared_equality_holds(n=8):
    """Algorithm 2 with its wrapper lines: shares of y in, shares of 1{y = 0} out, for every y."""
    size = 1 << n
    y = np.arange(size, dtype=np.uint64)
    rng = np.random.default_rng(808)
    g = W.gen_inputs(rng, n, size)
    ys = W.additive_shares(rng, n, y)
    k = oracle.gen("eq", n, g.alpha, g.r, g.seed0, g.seed1)
    m = [oracle.eq_mask(n, k[j], ys[j]) for j in (0, 1)]
    o = [oracle.eq_masked_eval(j, n, k[j], m[0], m[1]) for j in (0, 1)]
    return np.array_equal((o[0] + o[1]) & np.uint32(W.ring_mask(n)), (y == 0).astype(np.uint32))


def test_unmodified_oracle_passes_the_compact_pins():
    assert maxpool_holds() and shared_equality_holds()
    assert reconstruction_holds("cmp") and reconstruction_holds("eq")
    assert aes_known_answer_holds() and prg_definition_holds()
    assert relu_identity_holds()
    from test_oracle_fss import walk_uses_the_documented_blocks
    assert walk_uses_the_documented_blocks()


@pytest.mark.parametrize("name,old,new,pin", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, monkeypatch, name, old, new, pin):
    monkeypatch.setattr(oracle, "_lib", build_mutant(tmp_path, name, old, new))
    if pin == "aes":
        assert not aes_known_answer_holds()
    elif pin == "prg":
        assert aes_known_answer_holds() and not prg_definition_holds()
    elif pin == "layout":
        # mistakes that still reconstruct (any PRG layout does) but leave the documented one
        from test_oracle_fss import walk_uses_the_documented_blocks
        assert reconstruction_holds("cmp") and not walk_uses_the_documented_blocks()
    elif pin == "eqshared":
        assert reconstruction_holds("eq") and not shared_equality_holds()
    elif pin == "argmax":
        assert reconstruction_holds("cmp") and not maxpool_holds()
    elif pin == "relu":
        assert reconstruction_holds("cmp") and not relu_identity_holds()
    elif pin == "cmp":
        assert not reconstruction_holds("cmp")
    else:
        assert not reconstruction_holds("cmp") and not reconstruction_holds("eq")
