#!/usr/bin/env python3
"""Benchmark of the FSS hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: comparison KeyGen for B
elements, then both parties' Eval.  The headline workload is the large-batch configuration
(B = 2^22, n = 32, uniform alpha and x), with every input and both key buffers resident in
HBM before the timed region.  Prints ONE JSON line.

  value        comparison evaluations per second per party = B / mean duration of one Eval launch
  roofline     the dominant kernel (comparison Eval) against the LDS lookup rate that binds it
               (algorithmic and issued lookups), with the vector-ALU and HBM fractions beside it;
               roofline.gen: the same for the KeyGen kernel
  configs      after the timed steps: each of the five benchmark configurations (and n = 16)
               measured the same way -- Eval and KeyGen times (median, min), rates, fractions
  sustained_clock_mhz   shader clock measured by a probe wavefront beside the Eval kernel
  cpu_baseline the plain-C oracle timed on this host's cores on the first elements of the SAME
               arrays the GPU step used, after the GPU's keys and shares for those elements have
               been compared with the oracle's byte for byte

Other lines on request: --batch N, --workload eq / relu / maxpool / rounds / config (one
configuration alone, the form the profiles under profiles/ are taken from).
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# ---- work model -----------------------------------------------------------------------------
# The AES of this path is table-driven out of LDS: 16 four-byte lookups per round and block, and
# the LDS serves at most 32 such lookups per clock and CU (ds_read_b32; wider reads move more bytes
# but fewer lookups, see the micro-benchmark).  That rate, as bytes, is the peak the kernels are
# priced against; the vector ALU and HBM are reported beside it.
N_BITS = 32
LOOKUPS_PER_BLOCK = 160                     # 16 table lookups x 10 rounds, 4 bytes each
PEAK_LDS_GBS = 256 * 128 * 2.4              # 256 CUs x 32 lookups x 4 B per clock x 2.4 GHz = 78,643 GB/s
PEAK_LANE_TOPS = 256 * 64 * 2.4e9 / 1e12    # 256 CUs x 64 lanes x 2.4 GHz = 39.3 T 32-bit lane-ops/s
PEAK_HBM_GBS = 8000.0


def aes_blocks(kind: str, op: str, n: int) -> int:
    """AES blocks per element (Eval, per party) or per key pair (KeyGen), as the algorithms state them."""
    return {("cmp", "eval"): 2 * n, ("eq", "eval"): n, ("cmp", "gen"): 6 * n, ("eq", "gen"): 4 * n}[(kind, op)]


def hbm_bytes(kind: str, op: str, n: int) -> int:
    """HBM bytes per element: Eval reads its key planes (all but the alpha share) and x, writes the
    share; KeyGen reads alpha, r and two seeds and writes both keys."""
    key = (40 + 24 * n) if kind == "cmp" else (32 + 16 * n)
    return key - 4 + 4 + 4 if op == "eval" else 40 + 2 * key


# Instructions the kernels actually issue, per launch, from rocprofv3 --pmc runs of
# `bench.py --workload config --config <name>` (SQ_INSTS_LDS, SQ_INSTS_VALU: wavefront instructions,
# 64 lanes each) and HBM traffic per launch (FETCH_SIZE + WRITE_SIZE scaled by a plain copy).
# tests/test_profiles_match_bench.py checks every figure against the summaries under profiles/.
ISSUED = {          # profiles/configs_sq_counters.txt
    "config1": {"eval": {"lds": 2654208, "valu": 9156600}, "gen": {"lds": 7503872, "valu": 21788672}},
    "config2": {"eval": {"lds": 83918848, "valu": 163463168}, "gen": {"lds": 311459840, "valu": 527695872}},
    "config3": {"eval": {"lds": 116588544, "valu": 218301440}, "gen": {"lds": 343310336, "valu": 593693696}},
    "config4": {"eval": {"lds": 29171712, "valu": 55027968}, "gen": {"lds": 85852160, "valu": 149083904}},
    "config5": {"eval": {"lds": 608206848, "valu": 1124593664}, "gen": {"lds": 1791000576, "valu": 3062915072}},
    "n16": {"eval": {"lds": 304119808, "valu": 563605504}, "gen": {"lds": 895516672, "valu": 1536188416}},
}
MEASURED_HBM_BYTES = {   # profiles/hbm_counters.txt
    "config2": {"eval": 574728806, "gen": 1183088332},
    "config3": {"eval": 656437140, "gen": 1330162535},
    "config5": {"eval": 3405830699, "gen": 6946240421},
}

CONFIG_NAMES = ("config1", "config2", "config3", "config4", "config5", "n16")     # the `configs` block of the default run
RING_NAMES = ("n8", "n16", "n24", "n28")                                            # smaller rings, each measurable alone


def median(v):
    return statistics.median(v)


WARM_MS = 40.0


def warm_up(step, at_least, min_ms=WARM_MS):
    """Untimed repetitions of `step` before a measurement: at least `at_least`, and at least `min_ms` of
    them.  After an idle stretch the chip's power management needs about 30 ms of load to settle:
    launch times first rise by a fifth and then fall to their steady value (see the per-dispatch
    traces behind profiles/), so a few short repetitions alone would time that transient."""
    import torch
    torch.cuda.synchronize()
    t0, done = time.perf_counter(), 0
    while done < at_least or (time.perf_counter() - t0) * 1e3 < min_ms:
        step()
        torch.cuda.synchronize()
        done += 1
    return done


def lds_gbs(kind, op, n, batch, ms):
    return batch * aes_blocks(kind, op, n) * LOOKUPS_PER_BLOCK * 4 / (ms * 1e-3) / 1e9


def fractions(name, kind, op, n, batch, ms):
    """Roofline fractions of one launch of `ms` milliseconds."""
    algo = lds_gbs(kind, op, n, batch, ms)
    out = {"lds_algorithmic_gbs": algo, "lds_frac_algorithmic": algo / PEAK_LDS_GBS,
           "hbm_gbs": batch * hbm_bytes(kind, op, n) / (ms * 1e-3) / 1e9}
    out["hbm_frac"] = out["hbm_gbs"] / PEAK_HBM_GBS
    issued = ISSUED.get(name, {}).get(op)
    if issued:
        out["lds_frac_issued"] = issued["lds"] * 64 * 4 / (ms * 1e-3) / 1e9 / PEAK_LDS_GBS
        out["alu_frac"] = issued["valu"] * 64 / (ms * 1e-3) / 1e12 / PEAK_LANE_TOPS
    return out


class Device:
    """Device buffers of one workload (inputs, both key buffers, both outputs)."""

    def __init__(self, kind, n, w, dev):
        import numpy as np
        import torch
        import paper_2006_04593_amd as fss
        g = w.gen
        self.kind, self.n, self.batch, self.w = kind, n, g.batch, w
        self.alpha, self.r, self.x = (torch.from_numpy(a.view(np.int32)).to(dev) for a in (g.alpha, g.r, w.x))
        self.s0, self.s1 = torch.from_numpy(g.seed0).to(dev), torch.from_numpy(g.seed1).to(dev)
        nbytes = (fss.cmp_key_bytes if kind == "cmp" else fss.eq_key_bytes)(n, self.batch)
        self.k = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(2)]
        self.o = [torch.empty(self.batch, dtype=torch.int32, device=dev) for _ in range(2)]
        self.gen_fn = fss.cmp_gen if kind == "cmp" else fss.eq_gen
        self.eval_fn = fss.cmp_eval if kind == "cmp" else fss.eq_eval

    def gen(self, stream):
        self.gen_fn(self.n, self.batch, self.alpha, self.r, self.s0, self.s1, self.k[0], self.k[1], stream=stream)

    def eval(self, party, stream, x=None):
        self.eval_fn(party, self.n, self.batch, self.k[party], self.x if x is None else x, self.o[party], stream=stream)

    def step(self, stream, marks=None):
        """KeyGen, Eval of party 0, Eval of party 1; with `marks`, HIP events around each call."""
        import torch
        if marks is None:
            self.gen(stream); self.eval(0, stream); self.eval(1, stream)
            return
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        e[0].record(stream); self.gen(stream)
        e[1].record(stream); self.eval(0, stream)
        e[2].record(stream); self.eval(1, stream)
        e[3].record(stream)
        marks.append(e)

    def check_reconstruction(self):
        import numpy as np
        rec = (self.o[0] + self.o[1]).cpu().numpy().view(np.uint32)
        g, x = self.w.gen, self.w.x
        truth = (x <= g.alpha) if self.kind == "cmp" else (x == g.alpha)
        mask = np.uint32(0xFFFFFFFF if self.n == 32 else (1 << self.n) - 1)
        assert np.array_equal(rec & mask, truth.astype(np.uint32)), "reconstruction failed"


def kernel_names(kind, batch):
    import paper_2006_04593_amd as fss
    switch = fss.quad_layout_below()
    quad = batch < switch
    octo = kind == "cmp" and batch <= switch // 4          # the equality Eval keeps four lanes
    gen_octo = batch <= switch // 4
    return (f"{'eval_octo_kernel' if octo else 'eval_quad_kernel' if quad else 'eval_kernel'}<{kind}>",
            f"{'gen_octo_kernel' if gen_octo else 'gen_quad_kernel' if quad else 'gen_kernel'}<{kind}>",
            "eight lanes per element" if octo else "four lanes per element" if quad
            else "one lane per element (a short rest four lanes per element)")


def split_marks(marks):
    gen_ms = [e[0].elapsed_time(e[1]) for e in marks]
    ev_ms = [e[1].elapsed_time(e[2]) for e in marks] + [e[2].elapsed_time(e[3]) for e in marks]
    return gen_ms, ev_ms


def sig(v, digits=5):
    """Floats of the JSON line to `digits` significant figures (the line stays short enough to be read from a log tail)."""
    if isinstance(v, float):
        return float(f"{v:.{digits}g}")
    if isinstance(v, dict):
        return {k: sig(x, digits) for k, x in v.items()}
    if isinstance(v, (list, tuple)):
        return [sig(x, digits) for x in v]
    return v


def entry(name, kind, n, batch, gen_ms, ev_ms, what):
    """One configuration's figures in the short form CONFIGS_LEGEND describes."""
    ek, gk, layout = kernel_names(kind, batch)
    em, gm = median(ev_ms), median(gen_ms)
    fe, fg = fractions(name, kind, "eval", n, batch, em), fractions(name, kind, "gen", n, batch, gm)
    short = lambda f: [f["lds_frac_algorithmic"], f.get("lds_frac_issued"), f.get("alu_frac"), f["hbm_frac"]]
    return {"name": name, "kind": kind, "n": n, "batch": batch, "kernel": ek,
            "eval_ms": [em, min(ev_ms)], "gen_ms": [gm, min(gen_ms)],
            "evals_per_s": batch / (em * 1e-3), "pairs_per_s": batch / (gm * 1e-3),
            "eval_frac": short(fe), "gen_frac": short(fg)}


CONFIGS_LEGEND = ("kernel: the Eval kernel that ran; *_ms: [median, min] over the timed launches; evals_per_s: per party; pairs_per_s: KeyGen; "
                  "*_frac: [LDS lookups the algorithm states, LDS lookups issued, vector ALU, HBM] as fractions of the nominal peaks")


def config_workload(name):
    """(kind, n, workload, description) of a named configuration; config4 is handled by bench_rounds."""
    from paper_2006_04593_amd import workloads as W
    if name == "config1":
        return "cmp", 32, W.config_workload(1), "cmp Gen + both Evals, 16,384 elements, uniform alpha and x"
    if name == "config2":
        return "eq", 32, W.config_workload(2), "eq Gen + both Evals, 2^20 elements, x = alpha on a seeded tenth"
    if name == "config3":
        return "cmp", 32, W.config_workload(3), "ReLU-layer comparison batch, 64x112x112 = 802,816 masked fixed-point activations"
    if name == "config5":
        return "cmp", 32, W.config_workload(5), "cmp Gen + both Evals, 2^22 elements, uniform alpha and x"
    if name in RING_NAMES:
        n = int(name[1:])
        return "cmp", n, W.uniform_workload("cmp", n, 1 << 22, seed=W.BASE_SEED + n), f"cmp Gen + both Evals on the ring Z_2^{n}, 2^22 elements"
    raise ValueError(name)


def bench_pair(name, dev, reps, warm):
    """One configuration of the form KeyGen + both parties' Eval."""
    import torch
    kind, n, w, what = config_workload(name)
    d = Device(kind, n, w, dev)
    stream = torch.cuda.current_stream()
    warmed = warm_up(lambda: d.step(stream), warm)
    marks = []
    for _ in range(reps):
        d.step(stream, marks)
    torch.cuda.synchronize()
    d.check_reconstruction()
    gen_ms, ev_ms = split_marks(marks)
    out = entry(name, kind, n, d.batch, gen_ms, ev_ms, what)
    out["warmup_steps"] = warmed
    return out


def bench_rounds(dev, reps, warm):
    """Configuration 4: a 3x3 stride-2 pad-1 max-pool of 64 x 112 x 112 activations as a running
    maximum, eight DEPENDENT comparison rounds of 200,704 elements (round k compares the running
    maximum with tap k under fresh keys).  The reveal and the update between rounds are done in the
    clear by a few torch ops: they stand in for the protocol's messages and are not part of the method."""
    import numpy as np
    import torch
    import paper_2006_04593_amd as fss
    from paper_2006_04593_amd import workloads as W

    n = N_BITS
    taps = W.maxpool_taps(W.BASE_SEED + 4)                       # [9, B] int64
    B = taps.shape[1]
    T = lambda a: torch.from_numpy(a.view(np.int32) if a.dtype == np.uint32 else a).to(dev)
    d_taps = [T((taps[k] & 0xFFFFFFFF).astype(np.uint32)) for k in range(9)]
    stream = torch.cuda.current_stream()
    keys, d_alpha, gen_ms = [], [], []
    for rnd in range(1, W.MAXPOOL_ROUNDS + 1):
        g = W.maxpool_round_keys(W.BASE_SEED + 4, rnd, B)
        kk = [torch.empty(fss.cmp_key_bytes(n, B), dtype=torch.uint8, device=dev) for _ in range(2)]
        args = [T(v) for v in (g.alpha, g.r, g.seed0, g.seed1)]
        if rnd == 1:
            warm_up(lambda: fss.cmp_gen(n, B, *args, kk[0], kk[1], stream=stream), warm)
        for rep in range(max(reps // 4, 2)):                          # KeyGen of the round's 200,704 key pairs
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fss.cmp_gen(n, B, *args, kk[0], kk[1], stream=stream)
            e1.record(stream)
            gen_ms.append((e0, e1))
        keys.append(kk)
        d_alpha.append(args[0])
    torch.cuda.synchronize()
    gen_ms = [a.elapsed_time(b) for a, b in gen_ms]
    o = [torch.empty(B, dtype=torch.int32, device=dev) for _ in range(2)]
    marks = []

    def step(timed):
        m = d_taps[0].clone()
        for k in range(1, 9):
            x = m - d_taps[k] + d_alpha[k - 1]                  # the value both parties would reveal: (m - w_k) + alpha_k
            for j in (0, 1):
                if timed:
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                fss.cmp_eval(j, n, B, keys[k - 1][j], x, o[j], stream=stream)
                if timed:
                    e1.record(stream)
                    marks.append((e0, e1))
            m = torch.where((o[0] + o[1]) == 1, d_taps[k], m)   # 1{m - w_k <= 0}: the tap is at least the running maximum
        return m

    warmed = warm_up(lambda: step(False), warm)
    t0 = time.perf_counter()
    for _ in range(reps):
        m = step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    agree = (m.cpu().numpy().astype(np.int64) == taps.max(axis=0)).mean()
    assert agree > 0.9999, f"running maximum agrees with the plain max-pool on {agree} of the outputs"
    ev_ms = [a.elapsed_time(b) for a, b in marks]
    out = entry("config4", "cmp", n, B, gen_ms, ev_ms,
                "running-maximum max-pool 3x3/2 of 64x112x112: 8 dependent rounds x both parties' Eval of 200,704 elements, fresh keys per round")
    out.update({"warmup_steps": warmed, "rounds": 8, "step_ms_with_glue": wall * 1e3 / reps, "agrees_with_maxpool": agree})
    return out


def bench_named(name, dev, reps, warm):
    return bench_rounds(dev, reps, warm) if name == "config4" else bench_pair(name, dev, reps, warm)


def sustained_clock_mhz(d, dev):
    """Shader clock while the comparison Eval kernel runs: a one-wavefront probe on a second stream
    (it sleeps, so it takes nothing from the kernel) spans a few Eval launches."""
    import torch
    import paper_2006_04593_amd as fss
    khz = fss.wall_clock_khz()
    if khz <= 0:
        return None
    ticks = torch.zeros(2, dtype=torch.int64, device=dev)
    side = torch.cuda.Stream()
    stream = torch.cuda.current_stream()
    torch.cuda.synchronize()
    d.eval(0, stream)                                            # the chip is under load when the probe starts
    fss.clock_probe(ticks, 1200, stream=side)                    # about 4 ms
    for _ in range(3):
        d.eval(0, stream); d.eval(1, stream)
    torch.cuda.synchronize()
    c, wticks = (int(v) for v in ticks.cpu())
    return c / wticks * khz / 1e3 if wticks > 0 else None


def cpu_baseline(d, sample):
    """The oracle as it stands, on the host cores, on the first `sample` elements of the very arrays
    the GPU step used -- after the GPU's key planes and both parties' shares for those elements have
    been compared with the oracle's."""
    import numpy as np
    import oracle
    threads = oracle.set_threads(0)
    g, x, n, kind = d.w.gen, d.w.x, d.n, d.kind
    sample = min(sample, d.batch)
    a, r, s0, s1, xs = g.alpha[:sample], g.r[:sample], g.seed0[:sample], g.seed1[:sample], x[:sample]
    t0 = time.perf_counter()
    ok = oracle.gen(kind, n, a, r, s0, s1)
    t1 = time.perf_counter()
    oo = [None, None]
    oo[0] = oracle.eval_(kind, 0, n, ok[0], xs)
    t2 = time.perf_counter()
    oo[1] = oracle.eval_(kind, 1, n, ok[1], xs)
    t3 = time.perf_counter()
    # parity of the GPU step with the oracle on those elements: every plane of both keys, both shares
    for j in (0, 1):
        mine = oracle.split_key(kind, n, d.batch, d.k[j].cpu().numpy())
        ref = oracle.split_key(kind, n, sample, ok[j])
        for plane, v in ref.items():
            if plane == "bp":
                continue
            got = mine[plane][:, :sample] if plane in ("s_cw", "sigma_cw", "leaf") else mine[plane][:sample]
            want = v[:, :sample] if plane in ("s_cw", "sigma_cw", "leaf") else v[:sample]
            assert np.array_equal(got, want), f"GPU key {j} differs from the oracle's in plane {plane}"
        assert np.array_equal(d.o[j].cpu().numpy().view(np.uint32)[:sample], oo[j]), f"GPU share {j} differs from the oracle's"
        del mine
    per_party = ((t2 - t1) + (t3 - t2)) / 2
    small = max(sample // 16, 1)                                 # the same code on one thread, on a sixteenth of the sample
    oracle.set_threads(1)
    t4 = time.perf_counter()
    ks, _ = oracle.gen(kind, n, a[:small], r[:small], s0[:small], s1[:small])
    t5 = time.perf_counter()
    oracle.eval_(kind, 0, n, ks, xs[:small])
    t6 = time.perf_counter()
    oracle.set_threads(0)
    return {
        "value": sample / per_party, "unit": "evals/s/party", "cores": threads, "kind": "oracle",
        "sample": f"first {sample} of the {d.batch} elements the GPU step ran on (same alpha, r, seeds, x): Gen {t1 - t0:.2f} s, "
                  f"Eval {t2 - t1:.2f} + {t3 - t2:.2f} s",
        "parity": "GPU keys (every plane, both parties) and both shares equal the oracle's on those elements",
        "gen_pairs_per_s": sample / (t1 - t0),
        "one_thread_evals_per_s": small / (t6 - t5), "one_thread_gen_pairs_per_s": small / (t5 - t4),
    }


def relu_layer_bench(args, dev):
    """One shared ReLU layer (paper section 4.2) of 64 x 112 x 112 fixed-point activations, both
    parties on the one GPU: a step = each party's Sign mask, fused comparison + open round, finish.
    Keys and multiplication triples are dealer material, generated before the timed region."""
    import numpy as np
    import torch

    import paper_2006_04593_amd as fss
    from paper_2006_04593_amd import workloads as W

    n, B = N_BITS, 64 * 112 * 112
    rng = np.random.default_rng(W.BASE_SEED + 3)
    y = W.fixed_point_normal(rng, B)
    g = W.gen_inputs(rng, n, B)
    ri = W.relu_inputs(rng, n, y)

    def T(a):
        return torch.from_numpy(a.view(np.int32) if a.dtype == np.uint32 else a).to(dev)

    keys = [torch.empty(fss.cmp_key_bytes(n, B), dtype=torch.uint8, device=dev) for _ in range(2)]
    fss.cmp_gen(n, B, T(g.alpha), T(g.r), T(g.seed0), T(g.seed1), keys[0], keys[1])
    ys, ta, tb, tc = ([T(p[j]) for j in (0, 1)] for p in (ri.y_share, ri.tri_a, ri.tri_b, ri.tri_c))
    buf = lambda: [torch.empty(B, dtype=torch.int32, device=dev) for _ in range(2)]
    masked, delta, eps, z = buf(), buf(), buf(), buf()
    stream = torch.cuda.current_stream()
    open_ms = []

    def step(timed):
        for j in (0, 1):
            fss.sign_mask(n, B, keys[j], ys[j], masked[j], stream=stream)
        for j in (0, 1):
            if timed:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
            fss.relu_open(j, n, B, keys[j], masked[0], masked[1], ys[j], ta[j], tb[j], delta[j], eps[j], stream=stream)
            if timed:
                e1.record(stream)
                open_ms.append((e0, e1))
        for j in (0, 1):
            fss.relu_finish(j, n, B, delta[0], delta[1], eps[0], eps[1], ta[j], tb[j], tc[j], z[j], stream=stream)

    warm_up(lambda: step(False), args.warmup)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    rec = (z[0] + z[1]).cpu().numpy().view(np.uint32)
    x = (masked[0] + masked[1]).cpu().numpy().view(np.uint32)
    le = (x <= g.alpha)
    assert np.array_equal(rec, np.where(le, 0, y & 0xFFFFFFFF).astype(np.uint32)), "ReLU reconstruction failed"
    ms = median([a.elapsed_time(b) for a, b in open_ms])
    gbs = lds_gbs("cmp", "eval", n, B, ms)
    return {
        "metric": "shared ReLU elements/sec per party (n=32, lambda=128)",
        "value": B / (ms * 1e-3), "unit": "elements/s/party", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": "ReLU layer 64x112x112 = 802816 fixed-point activations: Sign mask + fused comparison/open "
                               "round + finish, both parties", "batch": B, "n": n, "lambda": 128},
        "relu_open_ms": ms,
        "roofline": {"bound": "lds", "kernel": "eval_kernel<cmp, relu-open>", "achieved": gbs, "peak": PEAK_LDS_GBS,
                     "unit": "GB/s", "frac": gbs / PEAK_LDS_GBS, "traffic": None},
    }


def maxpool_layer_bench(args, dev):
    """The paper's MaxPool (Algorithm 7: unroll, Argmax per window with k^2(k^2-1) comparisons and
    k^2 equalities, inner product), 3x3 windows, stride 2, no padding, over 64 x 112 x 112 shared
    activations: 193,600 windows, 13.9 M comparisons and 1.7 M equalities per party.  A step is
    every online kernel of BOTH parties; keys and triples are dealer material made beforehand."""
    import numpy as np
    import torch

    import paper_2006_04593_amd as fss
    from paper_2006_04593_amd import workloads as W

    n, C, H, Wd, k = N_BITS, 64, 112, 112, 3
    oh, ow = (H - k) // 2 + 1, (Wd - k) // 2 + 1
    rows, m = C * oh * ow, k * k
    ncmp, neq = rows * m * (m - 1), rows * m
    rng = np.random.default_rng(W.BASE_SEED + 4)
    x = W.fixed_point_normal(rng, (C, H, Wd))
    xs = W.additive_shares(rng, n, x.reshape(-1).astype(np.int64).astype(np.uint64))
    tr = W.triple_shares(rng, n, neq)

    def T(a):
        return torch.from_numpy(a.view(np.int32) if a.dtype == np.uint32 else a).to(dev)

    def keys(kind, count):
        g = W.gen_inputs(rng, n, count)
        nb = (fss.cmp_key_bytes if kind == "cmp" else fss.eq_key_bytes)(n, count)
        kk = [torch.empty(nb, dtype=torch.uint8, device=dev) for _ in range(2)]
        (fss.cmp_gen if kind == "cmp" else fss.eq_gen)(n, count, T(g.alpha), T(g.r), T(g.seed0), T(g.seed1), kk[0], kk[1])
        torch.cuda.synchronize()
        return kk

    kc, ke = keys("cmp", ncmp), keys("eq", neq)
    xd = [T(v) for v in xs]
    ta, tb, tc = ([T(p[j]) for j in (0, 1)] for p in (tr.a, tr.b, tr.c))
    buf = lambda cnt: [torch.empty(cnt, dtype=torch.int32, device=dev) for _ in range(2)]
    unrolled, mc, w, me, hot, dl, ep, out = buf(neq), buf(ncmp), buf(ncmp), buf(neq), buf(neq), buf(neq), buf(neq), buf(rows)
    stream = torch.cuda.current_stream()
    marks = []

    def step(timed):
        ev = lambda: torch.cuda.Event(enable_timing=True)
        for j in (0, 1):
            fss.maxpool_unroll(C, H, Wd, k, 2, xd[j], unrolled[j], stream=stream)
            fss.argmax_diff_mask(n, rows, m, kc[j], unrolled[j], mc[j], stream=stream)
        for j in (0, 1):
            e = [ev(), ev(), ev(), ev()] if timed else None
            if timed:
                e[0].record(stream)
            fss.sign_eval(j, n, ncmp, kc[j], mc[0], mc[1], w[j], stream=stream)
            if timed:
                e[1].record(stream)
            fss.argmax_count_mask(j, n, rows, m, w[j], ke[j], me[j], stream=stream)
            if timed:
                marks.append(e)
        for j in (0, 1):
            if timed:
                marks[-2 + j][2].record(stream)
            fss.eq_masked_eval(j, n, neq, ke[j], me[0], me[1], hot[j], stream=stream)
            if timed:
                marks[-2 + j][3].record(stream)
            fss.mul_open(n, neq, unrolled[j], hot[j], ta[j], tb[j], dl[j], ep[j], stream=stream)
        for j in (0, 1):
            fss.dot_finish(j, n, rows, m, dl[0], dl[1], ep[0], ep[1], ta[j], tb[j], tc[j], out[j], stream=stream)

    warm_up(lambda: step(False), args.warmup)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    y = (out[0] + out[1]).cpu().numpy().view(np.uint32)
    win = np.lib.stride_tricks.sliding_window_view(x, (k, k), axis=(1, 2))[:, ::2, ::2].reshape(rows, m)
    agree = (y == (win.max(axis=1) & 0xFFFFFFFF).astype(np.uint32)).mean()
    assert agree > 0.99, f"max-pool agreement {agree}"       # ties and Sign wrap-arounds aside
    cmp_ms = median([e[0].elapsed_time(e[1]) for e in marks])
    eq_ms = median([e[2].elapsed_time(e[3]) for e in marks])
    gbs = lds_gbs("cmp", "eval", n, ncmp, cmp_ms)
    return {
        "metric": "shared MaxPool windows/sec per party (3x3 stride 2, n=32, lambda=128)",
        "value": rows / ((wall / args.steps) / 2), "unit": "windows/s/party", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u32", "data": "synthetic",
        "config": {"workload": "MaxPool 3x3 stride 2 (no padding) over 64x112x112 shared activations, Algorithm 7: "
                               f"{rows} windows, {ncmp} comparisons + {neq} equalities + {neq} products per party",
                   "n": n, "lambda": 128},
        "cmp_eval_ms": cmp_ms, "cmp_evals_per_s": ncmp / (cmp_ms * 1e-3), "eq_eval_ms": eq_ms,
        "eq_evals_per_s": neq / (eq_ms * 1e-3), "eq_lds_frac_algorithmic": lds_gbs("eq", "eval", n, neq, eq_ms) / PEAK_LDS_GBS,
        "agreement_with_plain_maxpool": agree,
        "roofline": {"bound": "lds", "kernel": "eval_kernel<cmp, sign>", "achieved": gbs, "peak": PEAK_LDS_GBS,
                     "unit": "GB/s", "frac": gbs / PEAK_LDS_GBS, "traffic": None},
    }


def streamed_bench(args, dev):
    """Keys in pinned host memory, imported chunk by chunk during evaluation (fss_cmp_eval_streamed)."""
    import numpy as np
    import torch
    import paper_2006_04593_amd as fss
    from paper_2006_04593_amd import workloads as W

    n, B, chunk = N_BITS, args.batch, 1 << 18
    w = W.uniform_workload("cmp", n, B, seed=W.BASE_SEED + 5)
    d = Device("cmp", n, w, dev)
    stream = torch.cuda.current_stream()
    total = fss.cmp_chunked_key_bytes(n, B, chunk)
    host = torch.empty(total, dtype=torch.uint8, pin_memory=True)
    off = 0
    T = lambda a: torch.from_numpy(a.view(np.int32) if a.dtype == np.uint32 else a).to(dev)
    for first in range(0, B, chunk):
        sl = slice(first, min(first + chunk, B))
        ln = sl.stop - sl.start
        nb = fss.cmp_key_bytes(n, ln)
        kk = [torch.empty(nb, dtype=torch.uint8, device=dev) for _ in range(2)]
        fss.cmp_gen(n, ln, T(w.gen.alpha[sl]), T(w.gen.r[sl]), T(w.gen.seed0[sl]), T(w.gen.seed1[sl]), kk[0], kk[1])
        torch.cuda.synchronize()
        host[off:off + nb].copy_(kk[0])
        off += nb
    staging = torch.empty(2 * fss.cmp_key_bytes(n, chunk), dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream()
    ms = []
    for rep in range(args.warmup + args.steps):
        t0 = time.perf_counter()
        fss.cmp_eval_streamed(0, n, B, chunk, host, d.x, d.o[0], staging, side, stream=stream)      # blocks until done
        if rep >= args.warmup:
            ms.append((time.perf_counter() - t0) * 1e3)
    d.gen(stream); d.eval(0, stream)
    ref = d.o[0].clone()
    fss.cmp_eval_streamed(0, n, B, chunk, host, d.x, d.o[0], staging, side, stream=stream)
    assert torch.equal(ref, d.o[0]), "streamed evaluation differs from the resident one"
    t = median(ms)
    dst = torch.empty(total, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    dst.copy_(host, non_blocking=True)
    torch.cuda.synchronize()
    copy_ms = (time.perf_counter() - t0) * 1e3
    return {"metric": "FSS comparison evals/sec per party with keys streamed from host memory (n=32, lambda=128)",
            "value": B / (t * 1e-3), "unit": "evals/s/party", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": t, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32", "data": "synthetic",
            "config": {"workload": f"cmp Eval of {B} elements, keys in pinned host memory in chunks of {chunk}", "batch": B, "n": n},
            "host_link_gbs": total / (t * 1e-3) / 1e9, "bare_copy_of_the_same_bytes_ms": copy_ms,
            "bare_copy_gbs": total / (copy_ms * 1e-3) / 1e9,
            "roofline": {"bound": "host link", "achieved": total / (t * 1e-3) / 1e9, "peak": total / (copy_ms * 1e-3) / 1e9,
                         "unit": "GB/s", "frac": copy_ms / t, "traffic": None}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=1 << 22, help="elements per step (default: the 2^22 configuration)")
    ap.add_argument("--cpu-sample", type=int, default=1 << 18, help="elements for the oracle timing; 0 skips it")
    ap.add_argument("--workload", choices=["large", "eq", "relu", "maxpool", "rounds", "streamed", "config"], default="large",
                    help="large: the headline 2^22 comparison Gen+Eval step, then every benchmark configuration; eq: the same step "
                         "with the equality keys; relu: one shared ReLU layer of 64x112x112 activations; maxpool: the paper's "
                         "MaxPool (Algorithm 7), 3x3 stride 2 over 64x112x112; rounds: configuration 4 alone; streamed: keys "
                         "imported from pinned host memory; config: ONE configuration (--config) measured alone")
    ap.add_argument("--config", choices=sorted(set(CONFIG_NAMES + RING_NAMES)), default="config5", help="with --workload config")
    ap.add_argument("--configs", default="all", help="with --workload large: 'all', 'none' or a comma list of configurations "
                                                     "to measure after the timed steps")
    ap.add_argument("--config-reps", type=int, default=10, help="timed repetitions of each configuration in the configs block")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also launch one plain elementwise copy over 1 GiB, so that a rocprofv3 --pmc run of this "
                         "command holds the counter's reading for a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on ONE GPU (elements are independent; more GPUs would only shard the "
              "batch with no exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2006_04593_amd as fss
    from paper_2006_04593_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    fss.prepare()
    if args.pmc_calibration:
        src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst
    if args.workload == "relu":
        print(json.dumps(relu_layer_bench(args, dev)))
        return
    if args.workload == "maxpool":
        print(json.dumps(maxpool_layer_bench(args, dev)))
        return
    if args.workload == "streamed":
        print(json.dumps(streamed_bench(args, dev)))
        return
    if args.workload == "rounds":
        print(json.dumps(sig(bench_rounds(dev, args.steps, args.warmup))))
        return
    if args.workload == "config":
        print(json.dumps(sig(bench_named(args.config, dev, args.steps, args.warmup))))
        return

    B, n = args.batch, N_BITS
    cmp = args.workload != "eq"
    kind = "cmp" if cmp else "eq"
    name = "config5" if (cmp and B == 1 << 22) else ("config2" if (not cmp and B == 1 << 20) else f"{kind}-{B}")
    if cmp:
        w = W.uniform_workload("cmp", n, B, seed=W.BASE_SEED + 5, name="config5")
    else:
        w = W.equality_workload(n, B, seed=W.BASE_SEED + 2)           # x = alpha on a seeded tenth of the elements
    d = Device(kind, n, w, dev)
    stream = torch.cuda.current_stream()

    for _ in range(args.warmup):
        d.step(stream)
    torch.cuda.synchronize()
    marks = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        d.step(stream, marks)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    d.check_reconstruction()                       # correctness of what was just timed, on every element

    gen_ms, ev_ms = split_marks(marks)
    eval_ms = sum(ev_ms) / len(ev_ms)              # mean over the timed region: what `value` is quoted on
    gen_mean = sum(gen_ms) / len(gen_ms)
    ek, gk, layout = kernel_names(kind, B)
    fe, fg = fractions(name, kind, "eval", n, B, eval_ms), fractions(name, kind, "gen", n, B, gen_mean)

    def roofline(kernel, f, op):
        # achieved: the algorithm's lookups (AES blocks x 160 x 4 B per element) over the mean launch duration of the
        # timed steps (HIP events on the launch stream); peak: 32 lookups x 4 B per clock and CU at 2.4 GHz
        return {
            "bound": "lds", "kernel": kernel, "achieved": f["lds_algorithmic_gbs"], "peak": PEAK_LDS_GBS, "unit": "GB/s",
            "frac": f["lds_frac_algorithmic"], "frac_issued": f.get("lds_frac_issued"),
            "traffic": MEASURED_HBM_BYTES.get(name, {}).get(op), "traffic_algorithmic": B * hbm_bytes(kind, op, n),     # HBM bytes per launch
            "alu_frac": f.get("alu_frac"), "hbm_frac": f["hbm_frac"], "hbm_gbs": f["hbm_gbs"],
        }

    out = {
        "metric": f"FSS {'comparison' if cmp else 'equality'} evals/sec per party (n=32, lambda=128)",
        "value": B / (eval_ms * 1e-3),
        "unit": "evals/s/party",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": f"{'large' if B >= fss.quad_layout_below() else 'small'} batch: {kind} Gen of {B} keys + both parties' Eval, n=32, "
                               + ("uniform alpha and x" if cmp else "uniform alpha, x = alpha on a tenth of the elements")
                               + ", SoA keys resident in HBM", "batch": B, "n": n, "lambda": 128},
        "eval_ms": eval_ms, "eval_ms_median": median(ev_ms), "eval_ms_min": min(ev_ms),
        "gen_ms": gen_mean, "gen_ms_median": median(gen_ms), "gen_ms_min": min(gen_ms),
        "gen_key_pairs_per_s": B / (gen_mean * 1e-3),
        "step_evals_per_s_incl_gen": 2 * B / (wall / args.steps),
        "roofline": roofline(ek, fe, "eval"),
    }
    out["roofline"]["gen"] = roofline(gk, fg, "gen")
    out["sustained_clock_mhz"] = sustained_clock_mhz(d, dev)
    out["nominal_clock_mhz"] = 2400
    props = torch.cuda.get_device_properties(dev)
    out["device"] = {"name": props.name, "arch": getattr(props, "gcnArchName", None), "compute_units": props.multi_processor_count,
                     "lds_per_workgroup": getattr(props, "shared_memory_per_block", None)}
    if args.cpu_sample > 0:
        out["cpu_baseline"] = cpu_baseline(d, args.cpu_sample)
    del d
    torch.cuda.empty_cache()
    wanted = [] if args.configs == "none" else (list(CONFIG_NAMES) if args.configs == "all" else args.configs.split(","))
    if cmp and B == 1 << 22 and wanted:
        out["configs_legend"] = CONFIGS_LEGEND
        out["configs"] = []
        for cname in wanted:
            out["configs"].append(bench_named(cname, dev, args.config_reps, 2))
            torch.cuda.empty_cache()
    print(json.dumps(sig(out), separators=(",", ":")))


if __name__ == "__main__":
    main()
