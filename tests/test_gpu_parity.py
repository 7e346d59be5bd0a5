"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle --
bit-exact keys (KeyGen) and shares (Eval) on the same seeded inputs, plus cross-pairing
(oracle keys -> GPU Eval, GPU keys -> oracle Eval)."""
import numpy as np
import pytest

import oracle
import paper_2006_04593_amd as fss
from paper_2006_04593_amd import workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def dev():
    return torch.device("cuda:0")


def to_dev(a: np.ndarray):
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev())


def u32(t) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def key_bytes(kind, n, batch):
    return (fss.cmp_key_bytes if kind == "cmp" else fss.eq_key_bytes)(n, batch)


def gpu_gen(kind, n, g: W.GenInputs):
    nbytes = key_bytes(kind, n, g.batch)
    k0 = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device=dev())   # poison: Gen must write every byte
    k1 = torch.full((nbytes,), 0x5A, dtype=torch.uint8, device=dev())
    f = fss.cmp_gen if kind == "cmp" else fss.eq_gen
    f(n, g.batch, to_dev(g.alpha), to_dev(g.r), to_dev(g.seed0), to_dev(g.seed1), k0, k1)
    torch.cuda.synchronize()
    return k0, k1


def gpu_eval(kind, party, n, key, x: np.ndarray):
    batch = x.shape[0]
    out = torch.full((batch,), -1, dtype=torch.int32, device=dev())
    f = fss.cmp_eval if kind == "cmp" else fss.eq_eval
    f(party, n, batch, key, to_dev(x), out)
    torch.cuda.synchronize()
    return u32(out)


def truth(kind, x, alpha):
    x = x.astype(np.uint64); alpha = alpha.astype(np.uint64)
    return ((x <= alpha) if kind == "cmp" else (x == alpha)).astype(np.uint32)


def check_full(kind, n, g: W.GenInputs, x: np.ndarray):
    print(f"case kind={kind} n={n} batch={g.batch}", flush=True)
    k0, k1 = gpu_gen(kind, n, g)
    r0, r1 = oracle.gen(kind, n, g.alpha, g.r, g.seed0, g.seed1)
    assert np.array_equal(k0.cpu().numpy(), r0), "party-0 key differs from the oracle's"
    assert np.array_equal(k1.cpu().numpy(), r1), "party-1 key differs from the oracle's"
    o0, o1 = gpu_eval(kind, 0, n, k0, x), gpu_eval(kind, 1, n, k1, x)
    assert np.array_equal(o0, oracle.eval_(kind, 0, n, r0, x))
    assert np.array_equal(o1, oracle.eval_(kind, 1, n, r1, x))
    assert np.array_equal((o0 + o1) & np.uint32(W.ring_mask(n)), truth(kind, x & np.uint32(W.ring_mask(n)), g.alpha & np.uint32(W.ring_mask(n))))


# sizes: below one wavefront, ragged tails, several 1024-element workgroup tiles
@pytest.mark.parametrize("kind", ["cmp", "eq"])
@pytest.mark.parametrize("n,batch", [(32, 1), (32, 63), (32, 64), (32, 65), (32, 1000), (32, 1024), (32, 5000),
                                     (32, 16384), (1, 100), (2, 129), (8, 300), (12, 2049), (16, 4097), (31, 777),
                                     (24, 5000), (28, 4097)])
def test_gen_and_eval_match_oracle(kind, n, batch):
    w = W.uniform_workload(kind, n, batch, seed=1000 * n + batch)
    x = w.x.copy()
    x[::3] = w.gen.alpha[::3]                      # equality hits / the x = alpha boundary
    x[1::7] = w.gen.alpha[1::7] + np.uint32(1)
    x &= np.uint32(W.ring_mask(n))
    check_full(kind, n, w.gen, x)


# The kernels exist in two register layouts (four lanes per element below
# fss.quad_layout_below() elements, one lane per element from there on).  The sizes above all
# fall into the first; these straddle the switch, with ragged tails on both sides.
@pytest.mark.parametrize("kind", ["cmp", "eq"])
@pytest.mark.parametrize("n,offset", [(32, -17), (32, -1), (32, 0), (32, 1), (32, 63), (32, 65), (12, 1000), (8, 129), (1, 3),
                                      (24, -3), (24, 71), (28, -64), (28, 200), (16, 1)])
def test_both_layouts_around_the_switch(kind, n, offset):
    switch = fss.quad_layout_below()
    assert switch > 0 and switch % 64 == 0
    batch = switch + offset
    w = W.uniform_workload(kind, n, batch, seed=7000 + 10 * n + offset)
    x = w.x.copy()
    x[::5] = w.gen.alpha[::5]
    x &= np.uint32(W.ring_mask(n))
    check_full(kind, n, w.gen, x)


# Up to fss.quad_layout_below() / 4 elements, KeyGen (comparison and equality) and the comparison Eval
# run eight lanes per element (the equality Eval four); both sides of that switch, ragged.
@pytest.mark.parametrize("kind", ["cmp", "eq"])
@pytest.mark.parametrize("n,offset", [(32, -9), (32, -1), (32, 0), (32, 1), (32, 17), (12, -3), (16, 5)])
def test_around_the_eight_lane_switch(kind, n, offset):
    batch = fss.quad_layout_below() // 4 + offset
    w = W.uniform_workload(kind, n, batch, seed=6000 + 10 * n + offset)
    x = w.x.copy()
    x[::5] = w.gen.alpha[::5]
    x &= np.uint32(W.ring_mask(n))
    check_full(kind, n, w.gen, x)


# From the switch on, full passes (one 64-element tile for every wavefront of the grid: twice
# fss.quad_layout_below() elements) run one lane per element, and what is left after the last full
# pass runs four lanes per element INSIDE THE SAME LAUNCH when it is shorter than the switch, one lane
# per element otherwise.  Remainders of every kind, on both sides of that second switch.
@pytest.mark.parametrize("kind", ["cmp", "eq"])
@pytest.mark.parametrize("n,passes,rest", [(32, 1, 1), (32, 1, 15), (32, 1, 16), (32, 1, 17), (32, 1, 1000), (32, 1, 64 * 256),
                                           (32, 1, -1), (32, 1, 0), (32, 1, 63), (12, 2, 777), (16, 1, 4097), (32, 3, 16384)])
def test_remainder_after_full_passes(kind, n, passes, rest):
    switch = fss.quad_layout_below()
    full = 2 * switch                                   # elements of one full pass
    batch = passes * full + (rest if rest > 0 else switch + rest)      # rest <= 0: around the second switch
    w = W.uniform_workload(kind, n, batch, seed=9000 + 10 * n + passes + rest)
    x = w.x.copy()
    x[::5] = w.gen.alpha[::5]
    x &= np.uint32(W.ring_mask(n))
    check_full(kind, n, w.gen, x)


def test_seeded_sweep_of_sizes_nobody_picked():
    """Twenty (kind, n, batch) triples drawn from a fixed seed, batches log-uniform between 1 and
    four times the lane/quad switch: whatever split into passes, rows, rest tiles and layouts the
    host computes for them, every key byte and share equals the oracle's."""
    rng = np.random.default_rng(20060459)
    top = np.log2(4 * fss.quad_layout_below())
    for case in range(20):
        kind = ("cmp", "eq")[int(rng.integers(2))]
        n = int(rng.choice([1, 5, 8, 12, 16, 17, 24, 28, 31, 32, 32, 32]))
        batch = int(2 ** rng.uniform(0, top))
        w = W.uniform_workload(kind, n, batch, seed=9000 + case)
        check_full(kind, n, w.gen, w.x)


def test_the_two_layouts_produce_the_same_bytes():
    """One set of per-element arguments placed in a batch below the switch and, repeated, in a batch
    above it: keys and shares of an element depend on that element's arguments only."""
    n, small = 32, 1000
    big = fss.quad_layout_below() + 64
    w = W.uniform_workload("cmp", n, small, seed=4242)
    rep = -(-big // small)
    tile = lambda a: np.ascontiguousarray(np.concatenate([a] * rep)[:big])
    gb = W.GenInputs(n=n, alpha=tile(w.gen.alpha), r=tile(w.gen.r), seed0=tile(w.gen.seed0), seed1=tile(w.gen.seed1))
    xb = tile(w.x)
    for kind in ("cmp", "eq"):
        ks, kb = gpu_gen(kind, n, w.gen), gpu_gen(kind, n, gb)
        for j in (0, 1):
            ps = oracle.split_key(kind, n, small, ks[j].cpu().numpy())
            pb = oracle.split_key(kind, n, big, kb[j].cpu().numpy())
            for plane in ps:
                if plane == "bp":
                    continue
                a, b = ps[plane], pb[plane]
                if plane in ("s_cw", "sigma_cw", "leaf"):
                    assert np.array_equal(a[:, :small], b[:, :small]), (kind, plane)
                else:
                    assert np.array_equal(a[:small], b[:small]), (kind, plane)
            assert np.array_equal(gpu_eval(kind, j, n, ks[j], w.x), gpu_eval(kind, j, n, kb[j], xb)[:small])


@pytest.mark.parametrize("kind", ["cmp", "eq"])
@pytest.mark.parametrize("n,batch", [(32, 1), (32, 65), (12, 1000), (32, None)])
def test_nothing_is_written_outside_the_buffers(kind, n, batch):
    """Key and output buffers sit between guard regions inside larger allocations; Gen and Eval must
    leave the guards alone (batch None = just above the switch of register layouts, ragged)."""
    if batch is None:
        batch = fss.quad_layout_below() + 77
    print(f"case guards kind={kind} n={n} batch={batch}", flush=True)
    guard = 4096
    w = W.uniform_workload(kind, n, batch, seed=31 * n + batch)
    g = w.gen
    nbytes = key_bytes(kind, n, batch)
    arena = torch.full((2 * nbytes + 3 * guard,), 0xC3, dtype=torch.uint8, device=dev())
    k0 = arena[guard:guard + nbytes]
    k1 = arena[2 * guard + nbytes:2 * guard + 2 * nbytes]
    assert k0.data_ptr() % 256 == 0 and k1.data_ptr() % 256 == 0
    gen = fss.cmp_gen if kind == "cmp" else fss.eq_gen
    gen(n, batch, to_dev(g.alpha), to_dev(g.r), to_dev(g.seed0), to_dev(g.seed1), k0, k1)
    outs = torch.full((2 * batch + 3 * 1024,), 0x3C3C3C3C, dtype=torch.int32, device=dev())
    o0, o1 = outs[1024:1024 + batch], outs[2048 + batch:2048 + 2 * batch]
    ev = fss.cmp_eval if kind == "cmp" else fss.eq_eval
    xd = to_dev(w.x)
    ev(0, n, batch, k0, xd, o0)
    ev(1, n, batch, k1, xd, o1)
    torch.cuda.synchronize()
    a = arena.cpu().numpy()
    for lo, hi in ((0, guard), (guard + nbytes, 2 * guard + nbytes), (2 * guard + 2 * nbytes, 3 * guard + 2 * nbytes)):
        assert (a[lo:hi] == 0xC3).all(), f"key guard [{lo},{hi}) was written"
    o = outs.cpu().numpy()
    for lo, hi in ((0, 1024), (1024 + batch, 2048 + batch), (2048 + 2 * batch, 3072 + 2 * batch)):
        assert (o[lo:hi] == 0x3C3C3C3C).all(), f"output guard [{lo},{hi}) was written"
    r0, r1 = oracle.gen(kind, n, g.alpha, g.r, g.seed0, g.seed1)
    assert np.array_equal(a[guard:guard + nbytes], r0) and np.array_equal(a[2 * guard + nbytes:2 * guard + 2 * nbytes], r1)
    assert np.array_equal(u32(o0), oracle.eval_(kind, 0, n, r0, w.x)) and np.array_equal(u32(o1), oracle.eval_(kind, 1, n, r1, w.x))


@pytest.mark.parametrize("kind", ["cmp", "eq"])
def test_edge_offsets_and_inputs(kind):
    n = 32
    edges = W.edge_inputs(n)
    alpha = np.repeat(edges, len(edges))
    x = np.tile(edges, len(edges))
    g = W.gen_inputs(np.random.default_rng(12), n, len(alpha), alpha=alpha)
    check_full(kind, n, g, x)


@pytest.mark.parametrize("kind", ["cmp", "eq"])
@pytest.mark.parametrize("n", [8, 12])
def test_every_input_of_a_small_ring(kind, n):
    """All 2^n inputs against each of a few keys: the batch holds one key repeated 2^n times."""
    rng = np.random.default_rng(800 + n)
    for a in [0, W.ring_mask(n), int(rng.integers(0, 1 << n))]:
        size = 1 << n
        one = W.gen_inputs(rng, n, 1, alpha=np.array([a], dtype=np.uint32))
        g = W.GenInputs(n=n, alpha=np.repeat(one.alpha, size), r=np.repeat(one.r, size),
                        seed0=np.repeat(one.seed0, size, axis=0), seed1=np.repeat(one.seed1, size, axis=0))
        x = np.arange(size, dtype=np.uint32)
        k0, k1 = gpu_gen(kind, n, g)
        o0, o1 = gpu_eval(kind, 0, n, k0, x), gpu_eval(kind, 1, n, k1, x)
        r0, r1 = oracle.gen(kind, n, one.alpha, one.r, one.seed0, one.seed1)
        assert np.array_equal(o0, oracle.eval_all_x(kind, 0, n, 1, r0, 0))
        assert np.array_equal(o1, oracle.eval_all_x(kind, 1, n, 1, r1, 0))
        assert np.array_equal((o0 + o1) & np.uint32(W.ring_mask(n)), truth(kind, x, g.alpha))


@pytest.mark.parametrize("kind", ["cmp", "eq"])
def test_cross_pairing(kind):
    """Keys made by one side evaluate identically on the other."""
    n, batch = 32, 3333
    w = W.uniform_workload(kind, n, batch, seed=99)
    g, x = w.gen, w.x
    r0, r1 = oracle.gen(kind, n, g.alpha, g.r, g.seed0, g.seed1)
    # oracle keys -> GPU Eval
    o0 = gpu_eval(kind, 0, n, torch.from_numpy(r0).to(dev()), x)
    o1 = gpu_eval(kind, 1, n, torch.from_numpy(r1).to(dev()), x)
    assert np.array_equal(o0, oracle.eval_(kind, 0, n, r0, x)) and np.array_equal(o1, oracle.eval_(kind, 1, n, r1, x))
    # GPU keys -> oracle Eval
    k0, k1 = gpu_gen(kind, n, g)
    c0 = oracle.eval_(kind, 0, n, k0.cpu().numpy(), x)
    c1 = oracle.eval_(kind, 1, n, k1.cpu().numpy(), x)
    assert np.array_equal(c0 + c1, truth(kind, x, g.alpha))


def test_values_above_the_ring_are_reduced():
    n, batch = 12, 500
    w = W.uniform_workload("cmp", n, batch, seed=5)
    g = w.gen
    flip = np.zeros_like(g.seed0)
    flip[:, 0] = 1                                  # the control-bit position of a seed block is ignored
    hi = W.GenInputs(n=n, alpha=g.alpha | np.uint32(0xABC000), r=g.r | np.uint32(0x1000), seed0=g.seed0 ^ flip, seed1=g.seed1)
    k0, k1 = gpu_gen("cmp", n, hi)
    r0, r1 = oracle.gen("cmp", n, g.alpha, g.r, g.seed0, g.seed1)
    assert np.array_equal(k0.cpu().numpy(), r0) and np.array_equal(k1.cpu().numpy(), r1)
    assert np.array_equal(gpu_eval("cmp", 0, n, k0, w.x | np.uint32(0xFFFFF000)), oracle.eval_("cmp", 0, n, r0, w.x))


def test_empty_batch_is_a_noop_and_errors_raise():
    fss.prepare()                                   # idempotent per-device set-up
    fss.prepare()
    fss.cmp_eval(0, 32, 0, None, None, None)
    fss.eq_gen(32, 0, None, None, None, None, None, None)
    with pytest.raises(fss.FssError):
        fss.cmp_eval(3, 32, 0, None, None, None)
    torch.cuda.synchronize()


def test_clock_probe_reads_a_plausible_clock():
    ticks = torch.zeros(2, dtype=torch.int64, device=dev())
    fss.clock_probe(ticks, 100)
    torch.cuda.synchronize()
    shader, wall = (int(v) for v in ticks.cpu())
    khz = fss.wall_clock_khz()
    assert khz > 0 and wall > 0 and shader >= 100 * 64 * 127
    assert 500 < shader / wall * khz / 1e3 < 3500          # MHz


def test_binding_rejects_buffers_that_are_too_short_or_not_on_the_gpu():
    n, batch = 32, 1000
    i32 = lambda count: torch.zeros(count, dtype=torch.int32, device=dev())
    key = torch.zeros(fss.cmp_key_bytes(n, batch), dtype=torch.uint8, device=dev())
    with pytest.raises(ValueError, match="out"):
        fss.cmp_eval(0, n, batch, key, i32(batch), i32(batch - 1))
    with pytest.raises(ValueError, match="key"):
        fss.cmp_eval(0, n, batch, key[:-64], i32(batch), i32(batch))
    with pytest.raises(ValueError, match="GPU tensor"):
        fss.cmp_eval(0, n, batch, key, torch.zeros(batch, dtype=torch.int32), i32(batch))
    with pytest.raises(ValueError, match="contiguous"):
        fss.cmp_eval(0, n, batch, key, i32(2 * batch)[::2], i32(batch))
    with pytest.raises(ValueError, match="seed1"):
        fss.cmp_gen(n, batch, i32(batch), i32(batch), torch.zeros((batch, 16), dtype=torch.uint8, device=dev()),
                    torch.zeros((batch, 8), dtype=torch.uint8, device=dev()), key, torch.zeros_like(key))
    with pytest.raises(ValueError, match="masked"):
        fss.argmax_diff_mask(n, 10, 3, torch.zeros(fss.cmp_key_bytes(n, 60), dtype=torch.uint8, device=dev()), i32(30), i32(59))


def test_launches_on_two_streams_at_once():
    """KeyGen on one stream and the two parties' Evals of another batch on a second one, all in flight
    together (the kernels change their own wavefront priorities while they run): same bytes as one
    after the other."""
    n = 32
    a = W.uniform_workload("cmp", n, fss.quad_layout_below() + 4097, seed=71)
    b = W.uniform_workload("cmp", n, 50_000, seed=72)
    ka = gpu_gen("cmp", n, a.gen)
    want = [gpu_eval("cmp", j, n, ka[j], a.x) for j in (0, 1)]
    kb_ref = gpu_gen("cmp", n, b.gen)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    xa = to_dev(a.x)
    outs = [torch.full((a.gen.batch,), -1, dtype=torch.int32, device=dev()) for _ in range(2)]
    nbytes = fss.cmp_key_bytes(n, b.gen.batch)
    kb = [torch.zeros(nbytes, dtype=torch.uint8, device=dev()) for _ in range(2)]
    gargs = [to_dev(v) for v in (b.gen.alpha, b.gen.r, b.gen.seed0, b.gen.seed1)]
    torch.cuda.synchronize()
    for rep in range(3):
        fss.cmp_eval(0, n, a.gen.batch, ka[0], xa, outs[0], stream=s1)
        fss.cmp_gen(n, b.gen.batch, *gargs, kb[0], kb[1], stream=s2)
        fss.cmp_eval(1, n, a.gen.batch, ka[1], xa, outs[1], stream=s1)
    torch.cuda.synchronize()
    for j in (0, 1):
        assert np.array_equal(u32(outs[j]), want[j])
        assert torch.equal(kb[j], kb_ref[j])


def test_non_default_stream():
    n, batch = 32, 2048
    w = W.uniform_workload("eq", n, batch, seed=31)
    g = w.gen
    st = torch.cuda.Stream()
    nbytes = fss.eq_key_bytes(n, batch)
    k0 = torch.zeros(nbytes, dtype=torch.uint8, device=dev())
    k1 = torch.zeros(nbytes, dtype=torch.uint8, device=dev())
    out = torch.zeros(batch, dtype=torch.int32, device=dev())
    args = [to_dev(a) for a in (g.alpha, g.r, g.seed0, g.seed1)]
    xd = to_dev(w.x)
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        fss.eq_gen(n, batch, *args, k0, k1, stream=st)
        fss.eq_eval(1, n, batch, k1, xd, out, stream=st)
    st.synchronize()
    r0, r1 = oracle.gen("eq", n, g.alpha, g.r, g.seed0, g.seed1)
    assert np.array_equal(u32(out), oracle.eval_("eq", 1, n, r1, w.x))


# ---------------------------------------------------------------- benchmark configurations

def check_sampled(kind, n, g: W.GenInputs, x: np.ndarray, samples: int, seed: int):
    """Full-size run on the GPU; the oracle recomputes a seeded sample of elements (keys of
    an element depend on that element's arguments only) and the reconstruction identity is
    checked on every element.  Only for batches the oracle cannot walk in a test's time."""
    print(f"case kind={kind} n={n} batch={g.batch} sampled={samples}", flush=True)
    k0, k1 = gpu_gen(kind, n, g)
    o0, o1 = gpu_eval(kind, 0, n, k0, x), gpu_eval(kind, 1, n, k1, x)
    assert np.array_equal(o0 + o1, truth(kind, x, g.alpha))
    idx = np.sort(np.random.default_rng(seed).choice(g.batch, size=samples, replace=False))
    idx[0], idx[-1] = 0, g.batch - 1
    sub = W.GenInputs(n=n, alpha=g.alpha[idx], r=g.r[idx], seed0=g.seed0[idx], seed1=g.seed1[idx])
    r0, r1 = oracle.gen(kind, n, sub.alpha, sub.r, sub.seed0, sub.seed1)
    assert np.array_equal(o0[idx], oracle.eval_(kind, 0, n, r0, x[idx]))
    assert np.array_equal(o1[idx], oracle.eval_(kind, 1, n, r1, x[idx]))
    # key planes of the sampled elements, byte for byte
    for kd, rk in ((k0, r0), (k1, r1)):
        full = oracle.split_key(kind, n, g.batch, kd.cpu().numpy())
        part = oracle.split_key(kind, n, samples, rk)
        for plane in ("alpha_share", "seed", "ctrl", "last"):
            assert np.array_equal(full[plane][idx], part[plane][:samples]), plane
        planes = ("s_cw", "sigma_cw", "leaf") if kind == "cmp" else ("s_cw",)
        for plane in planes:
            assert np.array_equal(full[plane][:, idx], part[plane][:, :samples]), plane
        del full
    return o0, o1


ELEMENT_PLANES = ("alpha_share", "seed", "ctrl", "last")          # [Bp, ...]
LEVEL_PLANES = {"cmp": ("s_cw", "sigma_cw", "leaf"), "eq": ("s_cw",)}   # [n, Bp, ...]


def compare_with_oracle_in_chunks(kind, n, g: W.GenInputs, x, keys, shares, chunk=1 << 20):
    """EVERY element of a full-size GPU run against the oracle: all planes of both key buffers byte
    for byte and both parties' shares.  An element's key depends on that element's arguments only,
    so the oracle walks the batch in chunks of `chunk` elements (bounded host memory) and each
    chunk's planes are compared with the matching slice of the GPU's planes; padding elements of
    the GPU buffers must be zero."""
    batch = g.batch
    host = [oracle.split_key(kind, n, batch, k.cpu().numpy()) for k in keys]
    for c0 in range(0, batch, chunk):
        c1 = min(c0 + chunk, batch)
        r = oracle.gen(kind, n, g.alpha[c0:c1], g.r[c0:c1], g.seed0[c0:c1], g.seed1[c0:c1])
        for j in (0, 1):
            part = oracle.split_key(kind, n, c1 - c0, r[j])
            for plane in ELEMENT_PLANES:
                assert np.array_equal(host[j][plane][c0:c1], part[plane][:c1 - c0]), (plane, j, c0)
            for plane in LEVEL_PLANES[kind]:
                assert np.array_equal(host[j][plane][:, c0:c1], part[plane][:, :c1 - c0]), (plane, j, c0)
            assert np.array_equal(shares[j][c0:c1], oracle.eval_(kind, j, n, r[j], x[c0:c1])), ("share", j, c0)
        print(f"  elements [{c0}, {c1}) match the oracle", flush=True)
    for j in (0, 1):
        for plane in ELEMENT_PLANES:
            assert not host[j][plane][batch:].any(), (plane, "padding")
        for plane in LEVEL_PLANES[kind]:
            assert not host[j][plane][:, batch:].any(), (plane, "padding")


def check_every_element(kind, n, g: W.GenInputs, x: np.ndarray):
    print(f"case kind={kind} n={n} batch={g.batch} every element", flush=True)
    k0, k1 = gpu_gen(kind, n, g)
    o0, o1 = gpu_eval(kind, 0, n, k0, x), gpu_eval(kind, 1, n, k1, x)
    assert np.array_equal((o0 + o1) & np.uint32(W.ring_mask(n)), truth(kind, x, g.alpha))
    compare_with_oracle_in_chunks(kind, n, g, x, (k0, k1), (o0, o1))
    return o0, o1


def test_config1_comparison_16k():
    w = W.config_workload(1)
    check_full("cmp", 32, w.gen, w.x)


def test_config2_equality_1m():
    w = W.config_workload(2)
    o0, o1 = check_every_element("eq", 32, w.gen, w.x)
    assert np.array_equal((o0 + o1).astype(bool), w.extra["hit"] | (w.x == w.gen.alpha))


def test_config3_relu_layer():
    w = W.config_workload(3)
    o0, o1 = check_every_element("cmp", 32, w.gen, w.x)
    # Sign protocol: disagrees with 1{y <= 0} only on the rare wrap-around (|y| / 2^32 each)
    assert ((o0 + o1) != (w.extra["y"] <= 0)).sum() <= 8


def test_config4_maxpool_dependent_rounds():
    """8 dependent comparison rounds of 200,704 elements: running maximum over the nine
    taps of each 3x3 window; the reveal between rounds is done in the clear by the test.
    Every key byte and every share of every round is compared with the oracle."""
    n = 32
    taps = W.maxpool_taps(W.BASE_SEED + 4)
    batch = taps.shape[1]
    assert batch == 64 * 56 * 56
    m = taps[0].copy()
    for rnd in range(1, W.MAXPOOL_ROUNDS + 1):
        g = W.maxpool_round_keys(W.BASE_SEED + 4, rnd, batch)
        d = m - taps[rnd]                                   # m <= w  <=>  d <= 0
        x = ((d + g.alpha.astype(np.int64)) & 0xFFFFFFFF).astype(np.uint32)
        print(f"round {rnd}", flush=True)
        o0, o1 = check_every_element("cmp", n, g, x)
        m = np.where((o0 + o1) == 1, taps[rnd], m)
    # wrap-around failures are ~|d|/2^32 per comparison: allow a handful of windows to differ
    assert (m != taps.max(axis=0)).sum() <= 8


def test_config5_large_batch():
    """2^22 elements, the benchmark's launch (16 passes of the one-lane-per-element kernels):
    every key byte and share against the oracle."""
    w = W.config_workload(5)
    check_every_element("cmp", 32, w.gen, w.x)


def test_small_ring_large_batch_every_element():
    """n = 16 at 2^20 elements: the multi-pass loop of the one-lane-per-element kernels on a short ring."""
    w = W.uniform_workload("cmp", 16, 1 << 20, seed=1620)
    check_every_element("cmp", 16, w.gen, w.x)


def test_key_buffer_beyond_4_gib():
    """B = 2^23 + 1000: one party's key is 6.8 GB, so every plane offset past the first few
    needs 64-bit arithmetic; sampled elements (including the first and the last) against the oracle."""
    n, batch = 32, (1 << 23) + 1000
    w = W.uniform_workload("cmp", n, batch, seed=823)
    assert fss.cmp_key_bytes(n, batch) > (1 << 32)
    check_sampled("cmp", n, w.gen, w.x, samples=2048, seed=23)


def test_calls_can_be_captured_in_a_hip_graph_and_replayed():
    """Gen + both Evals recorded once into a graph (the library only enqueues kernels on the
    caller's stream), then replayed on fresh inputs written into the same buffers; every replay
    is checked against the eager result and the oracle."""
    n, batch = 32, 5000
    nbytes = fss.cmp_key_bytes(n, batch)
    bufs = dict(alpha=torch.zeros(batch, dtype=torch.int32, device=dev()), r=torch.zeros(batch, dtype=torch.int32, device=dev()),
                s0=torch.zeros((batch, 16), dtype=torch.uint8, device=dev()), s1=torch.zeros((batch, 16), dtype=torch.uint8, device=dev()),
                x=torch.zeros(batch, dtype=torch.int32, device=dev()))
    k0 = torch.zeros(nbytes, dtype=torch.uint8, device=dev())
    k1 = torch.zeros(nbytes, dtype=torch.uint8, device=dev())
    o0 = torch.zeros(batch, dtype=torch.int32, device=dev())
    o1 = torch.zeros(batch, dtype=torch.int32, device=dev())

    def enqueue():
        fss.cmp_gen(n, batch, bufs["alpha"], bufs["r"], bufs["s0"], bufs["s1"], k0, k1)
        fss.cmp_eval(0, n, batch, k0, bufs["x"], o0)
        fss.cmp_eval(1, n, batch, k1, bufs["x"], o1)

    def load(seed):
        w = W.uniform_workload("cmp", n, batch, seed=seed)
        for name, arr in (("alpha", w.gen.alpha), ("r", w.gen.r), ("s0", w.gen.seed0), ("s1", w.gen.seed1), ("x", w.x)):
            bufs[name].copy_(to_dev(arr))
        torch.cuda.synchronize()
        return w

    load(1)
    enqueue()                                   # eager once: also configures the kernels outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue()
    for seed in (2, 3, 4):
        w = load(seed)
        o0.fill_(-1); o1.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        g0, g1 = u32(o0).copy(), u32(o1).copy()
        r0, r1 = oracle.gen("cmp", n, w.gen.alpha, w.gen.r, w.gen.seed0, w.gen.seed1)
        assert np.array_equal(k0.cpu().numpy(), r0) and np.array_equal(k1.cpu().numpy(), r1)
        assert np.array_equal(g0, oracle.eval_("cmp", 0, n, r0, w.x)) and np.array_equal(g1, oracle.eval_("cmp", 1, n, r1, w.x))
        o0.fill_(-1); o1.fill_(-1)
        enqueue()                               # eager work between replays
        torch.cuda.synchronize()
        assert np.array_equal(u32(o0), g0) and np.array_equal(u32(o1), g1)
