#!/usr/bin/env python3
"""Benchmark of the FSS hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: comparison KeyGen for B
elements, then both parties' Eval.  The workload is the large-batch configuration
(B = 2^22, n = 32, uniform alpha and x), with every input and both key buffers resident in
HBM before the timed region.  Prints ONE JSON line.

  value      comparison evaluations per second per party = B / mean duration of one Eval launch
  roofline   the dominant kernel (comparison Eval) against the LDS read peak that binds it,
             with the vector-ALU and HBM fractions beside it
  cpu_baseline  the plain-C oracle timed on this host's cores on a bounded sample

Other lines on request: --batch N (small batches run the four-lanes-per-element kernels),
--workload eq (equality keys), --workload relu / maxpool (the paper's layers around the path).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# ---- work model of the comparison Eval kernel ---------------------------------------------
# (per evaluation at n = 32: 64 AES blocks of 160 four-byte table lookups each; the LDS read port,
#  128 B/clk/CU, is the unit that binds; the vector ALU and HBM are reported beside it)
N_BITS = 32
AES_BLOCKS_PER_EVAL = 2 * N_BITS            # one child block + one sigma/tau block per level
LOOKUPS_PER_BLOCK = 160                     # 16 table lookups x 10 rounds, 4 bytes each: what table-driven AES needs
LDS_BYTES_PER_EVAL = AES_BLOCKS_PER_EVAL * LOOKUPS_PER_BLOCK * 4
LDS_BYTES_ISSUED_PER_EVAL = 9282 * 4        # what the kernel issues (SQ_INSTS_LDS): coinciding lookups of the two
                                            # blocks of a level are shared, unneeded final-round ones skipped
VALU_OPS_PER_BLOCK = 257                    # vector-ALU instructions per AES block (SQ_INSTS_VALU, tree walk excluded)
TREE_OPS_PER_LEVEL = 30                     # correction-word gating, selects, accumulate
LANE_OPS_PER_EVAL = AES_BLOCKS_PER_EVAL * VALU_OPS_PER_BLOCK + N_BITS * TREE_OPS_PER_LEVEL
HBM_BYTES_PER_EVAL = 804 + 4 + 4            # key planes read by Eval + x + out
PEAK_LDS_GBS = 256 * 128 * 2.4              # 256 CUs x 128 B/clk x 2.4 GHz = 78,643 GB/s
PEAK_LANE_TOPS = 256 * 64 * 2.4e9 / 1e12    # 256 CUs x 64 lanes x 2.4 GHz = 39.3 T 32-bit lane-ops/s
PEAK_HBM_GBS = 8000.0
# HBM bytes per Eval launch at B = 2^22 from rocprofv3 FETCH_SIZE / WRITE_SIZE, scaled by a plain
# 1 GiB copy in the same run (profiles/cmp_2p22_hbm_counters.txt)
MEASURED_HBM_BYTES_2P22 = (3_309_750 + 16_384) * 1024


def cpu_baseline(sample: int):
    """The oracle as it stands, on the host cores, on the first `sample` elements of the workload."""
    import numpy as np
    import oracle
    from paper_2006_04593_amd import workloads as W
    threads = oracle.set_threads(0)
    w = W.uniform_workload("cmp", N_BITS, sample, seed=W.BASE_SEED + 5)
    g = w.gen
    t0 = time.perf_counter()
    k0, k1 = oracle.gen("cmp", N_BITS, g.alpha, g.r, g.seed0, g.seed1)
    t1 = time.perf_counter()
    o0 = oracle.eval_("cmp", 0, N_BITS, k0, w.x)
    t2 = time.perf_counter()
    o1 = oracle.eval_("cmp", 1, N_BITS, k1, w.x)
    t3 = time.perf_counter()
    assert np.array_equal(o0 + o1, (w.x <= g.alpha).astype(np.uint32))
    per_party = ((t2 - t1) + (t3 - t2)) / 2
    # the same code on one thread, on a sixteenth of the sample
    small = max(sample // 16, 1)
    oracle.set_threads(1)
    t4 = time.perf_counter()
    k0s, _ = oracle.gen("cmp", N_BITS, g.alpha[:small], g.r[:small], g.seed0[:small], g.seed1[:small])
    t5 = time.perf_counter()
    oracle.eval_("cmp", 0, N_BITS, k0s, w.x[:small])
    t6 = time.perf_counter()
    oracle.set_threads(0)
    return {
        "value": sample / per_party,
        "unit": "evals/s/party",
        "cores": threads,
        "kind": "oracle",
        "sample": f"first-seed {sample} elements of the same workload: cmp Gen {t1 - t0:.2f} s, "
                  f"Eval party0 {t2 - t1:.2f} s, party1 {t3 - t2:.2f} s",
        "gen_pairs_per_s": sample / (t1 - t0),
        "one_thread_evals_per_s": small / (t6 - t5),
        "one_thread_gen_pairs_per_s": small / (t5 - t4),
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

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    rec = (z[0] + z[1]).cpu().numpy().view(np.uint32)
    x = (masked[0] + masked[1]).cpu().numpy().view(np.uint32)
    le = (x <= g.alpha)
    assert np.array_equal(rec, np.where(le, 0, y & 0xFFFFFFFF).astype(np.uint32)), "ReLU reconstruction failed"
    ms = sum(a.elapsed_time(b) for a, b in open_ms) / len(open_ms)
    lds_gbs = B * LDS_BYTES_PER_EVAL / (ms * 1e-3) / 1e9
    return {
        "metric": "shared ReLU elements/sec per party (n=32, lambda=128)",
        "value": B / (ms * 1e-3), "unit": "elements/s/party", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": "ReLU layer 64x112x112 = 802816 fixed-point activations: Sign mask + fused comparison/open "
                               "round + finish, both parties", "batch": B, "n": n, "lambda": 128},
        "relu_open_ms": ms,
        "roofline": {"bound": "lds", "kernel": "eval_kernel<cmp, relu-open>", "achieved": lds_gbs, "peak": PEAK_LDS_GBS,
                     "unit": "GB/s", "frac": lds_gbs / PEAK_LDS_GBS, "traffic": None},
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

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    y = (out[0] + out[1]).cpu().numpy().view(np.uint32)
    win = np.lib.stride_tricks.sliding_window_view(x, (k, k), axis=(1, 2))[:, ::2, ::2].reshape(rows, m)
    agree = (y == (win.max(axis=1) & 0xFFFFFFFF).astype(np.uint32)).mean()
    assert agree > 0.99, f"max-pool agreement {agree}"       # ties and Sign wrap-arounds aside
    cmp_ms = sum(e[0].elapsed_time(e[1]) for e in marks) / len(marks)
    eq_ms = sum(e[2].elapsed_time(e[3]) for e in marks) / len(marks)
    lds_gbs = ncmp * LDS_BYTES_PER_EVAL / (cmp_ms * 1e-3) / 1e9
    return {
        "metric": "shared MaxPool windows/sec per party (3x3 stride 2, n=32, lambda=128)",
        "value": rows / ((wall / args.steps) / 2), "unit": "windows/s/party", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u32", "data": "synthetic",
        "config": {"workload": "MaxPool 3x3 stride 2 (no padding) over 64x112x112 shared activations, Algorithm 7: "
                               f"{rows} windows, {ncmp} comparisons + {neq} equalities + {neq} products per party",
                   "n": n, "lambda": 128},
        "cmp_eval_ms": cmp_ms, "cmp_evals_per_s": ncmp / (cmp_ms * 1e-3), "eq_eval_ms": eq_ms,
        "eq_evals_per_s": neq / (eq_ms * 1e-3), "agreement_with_plain_maxpool": agree,
        "roofline": {"bound": "lds", "kernel": "eval_kernel<cmp, sign>", "achieved": lds_gbs, "peak": PEAK_LDS_GBS,
                     "unit": "GB/s", "frac": lds_gbs / PEAK_LDS_GBS, "traffic": None},
    }


def dependent_rounds_bench(args, dev):
    """Benchmark configuration 4: a 3x3 stride-2 pad-1 max-pool of 64 x 112 x 112 activations as a running
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

    def T(a):
        return torch.from_numpy(a.view(np.int32) if a.dtype == np.uint32 else a).to(dev)

    d_taps = [T((taps[k] & 0xFFFFFFFF).astype(np.uint32)) for k in range(9)]
    keys, d_alpha = [], []
    for rnd in range(1, W.MAXPOOL_ROUNDS + 1):
        g = W.maxpool_round_keys(W.BASE_SEED + 4, rnd, B)
        kk = [torch.empty(fss.cmp_key_bytes(n, B), dtype=torch.uint8, device=dev) for _ in range(2)]
        fss.cmp_gen(n, B, T(g.alpha), T(g.r), T(g.seed0), T(g.seed1), kk[0], kk[1])
        keys.append(kk)
        d_alpha.append(T(g.alpha))
    torch.cuda.synchronize()
    o = [torch.empty(B, dtype=torch.int32, device=dev) for _ in range(2)]
    stream = torch.cuda.current_stream()
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

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        m = step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    got = m.cpu().numpy().astype(np.int64)
    agree = (got == taps.max(axis=0)).mean()
    assert agree > 0.9999, f"running maximum agrees with the plain max-pool on {agree} of the outputs"
    ms = [a.elapsed_time(b) for a, b in marks]
    eval_ms = sum(ms) / len(ms)
    lds_gbs = B * LDS_BYTES_PER_EVAL / (eval_ms * 1e-3) / 1e9
    return {
        "metric": "FSS comparison evals/sec per party in dependent rounds (n=32, lambda=128)",
        "value": B / (eval_ms * 1e-3), "unit": "evals/s/party", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": f"running-maximum max-pool 3x3/2 of 64x112x112: 8 dependent rounds x both parties' Eval of {B} elements",
                   "batch": B, "rounds": 8, "n": n, "lambda": 128},
        "eval_ms": eval_ms, "eval_ms_sum_of_16": eval_ms * 16, "agreement_with_plain_maxpool": agree,
        "roofline": {"bound": "lds", "kernel": "eval_kernel<cmp>", "achieved": lds_gbs, "peak": PEAK_LDS_GBS,
                     "unit": "GB/s", "frac": lds_gbs / PEAK_LDS_GBS, "traffic": None},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=1 << 22, help="elements per step (default: the 2^22 configuration)")
    ap.add_argument("--cpu-sample", type=int, default=1 << 18, help="elements for the oracle timing; 0 skips it")
    ap.add_argument("--workload", choices=["large", "eq", "relu", "maxpool", "rounds"], default="large",
                    help="large: the headline 2^22 comparison Gen+Eval step; eq: the same step with the equality keys "
                         "(Algorithms 1 and 2; --batch 1048576 is the 2^20 configuration); relu: one shared ReLU layer of "
                         "64x112x112 activations (Sign mask, fused comparison+open round, finish) per party; "
                         "maxpool: the paper's MaxPool (Algorithm 7), 3x3 stride 2 over 64x112x112; rounds: the same "
                         "pooling as a running maximum, 8 dependent comparison rounds of 200,704 elements")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also launch one plain elementwise copy over 1 GiB, so that a rocprofv3 --pmc run of this "
                         "command holds the counter's reading for a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on ONE GPU (elements are independent; more GPUs would only shard the "
              "batch with no exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2006_04593_amd as fss
    from paper_2006_04593_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload == "relu":
        print(json.dumps(relu_layer_bench(args, dev)))
        return
    if args.workload == "maxpool":
        print(json.dumps(maxpool_layer_bench(args, dev)))
        return
    if args.workload == "rounds":
        print(json.dumps(dependent_rounds_bench(args, dev)))
        return
    B, n = args.batch, N_BITS
    cmp = args.workload != "eq"
    if cmp:
        w = W.uniform_workload("cmp", n, B, seed=W.BASE_SEED + 5, name="config5")
    else:
        w = W.equality_workload(n, B, seed=W.BASE_SEED + 2)           # x = alpha on a seeded tenth of the elements
    g = w.gen
    gen_fn, eval_fn, key_bytes_fn = (fss.cmp_gen, fss.cmp_eval, fss.cmp_key_bytes) if cmp else (fss.eq_gen, fss.eq_eval, fss.eq_key_bytes)
    d_alpha, d_r, d_x = (torch.from_numpy(a.view(np.int32)).to(dev) for a in (g.alpha, g.r, w.x))
    d_s0, d_s1 = torch.from_numpy(g.seed0).to(dev), torch.from_numpy(g.seed1).to(dev)
    nbytes = key_bytes_fn(n, B)
    k0 = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    k1 = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    o0 = torch.empty(B, dtype=torch.int32, device=dev)
    o1 = torch.empty(B, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def step(marks=None):
        if marks is not None:
            e = [ev() for _ in range(4)]
            e[0].record(stream)
        gen_fn(n, B, d_alpha, d_r, d_s0, d_s1, k0, k1, stream=stream)
        if marks is not None:
            e[1].record(stream)
        eval_fn(0, n, B, k0, d_x, o0, stream=stream)
        if marks is not None:
            e[2].record(stream)
        eval_fn(1, n, B, k1, d_x, o1, stream=stream)
        if marks is not None:
            e[3].record(stream)
            marks.append(e)

    if args.pmc_calibration:
        src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    marks = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(marks)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # correctness of what was just timed: reconstruction on every element
    rec = (o0 + o1).cpu().numpy().view(np.uint32)
    truth = (w.x <= g.alpha) if cmp else (w.x == g.alpha)
    assert np.array_equal(rec, truth.astype(np.uint32)), "reconstruction failed"

    gen_ms = [e[0].elapsed_time(e[1]) for e in marks]
    ev_ms = [e[1].elapsed_time(e[2]) for e in marks] + [e[2].elapsed_time(e[3]) for e in marks]
    eval_ms = sum(ev_ms) / len(ev_ms)
    gen_mean = sum(gen_ms) / len(gen_ms)
    evals_per_s = B / (eval_ms * 1e-3)

    lane_layout = B >= fss.quad_layout_below()     # the instruction counts above belong to this layout
    blocks = AES_BLOCKS_PER_EVAL if cmp else N_BITS                 # equality: one block per level
    hbm_per_eval = HBM_BYTES_PER_EVAL if cmp else 540 + 4 + 4       # equality key planes read by Eval + x + out
    lds_gbs = B * blocks * LOOKUPS_PER_BLOCK * 4 / (eval_ms * 1e-3) / 1e9
    lane_tops = B * LANE_OPS_PER_EVAL / (eval_ms * 1e-3) / 1e12
    hbm_gbs = B * hbm_per_eval / (eval_ms * 1e-3) / 1e9
    out = {
        "metric": f"FSS {'comparison' if cmp else 'equality'} evals/sec per party (n=32, lambda=128)",
        "value": evals_per_s,
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
        "config": {"workload": f"{'large' if lane_layout else 'small'} batch: {'cmp' if cmp else 'eq'} Gen of {B} keys + both parties' Eval, n=32, "
                               + ("uniform alpha and x" if cmp else "uniform alpha, x = alpha on a tenth of the elements") + ", SoA keys resident in HBM", "batch": B, "n": n, "lambda": 128,
                   "register_layout": "one lane per element" if lane_layout else "four lanes per element"},
        "eval_ms": eval_ms,
        "eval_ms_min": min(ev_ms),
        "gen_ms": gen_mean,
        "gen_key_pairs_per_s": B / (gen_mean * 1e-3),
        "step_evals_per_s_incl_gen": 2 * B / (wall / args.steps),
        # The AES of this path is table-driven out of LDS, and the LDS read port is the unit that
        # binds: 160 four-byte lookups per AES block against 128 B/clk/CU.
        "roofline": {
            "bound": "lds",
            "kernel": "eval_kernel<cmp>" if cmp else "eval_kernel<eq>",
            "achieved": lds_gbs,
            "peak": PEAK_LDS_GBS,
            "unit": "GB/s",
            "frac": lds_gbs / PEAK_LDS_GBS,
            "traffic": MEASURED_HBM_BYTES_2P22 if (cmp and B == (1 << 22)) else None,
            "traffic_unit": "HBM bytes per Eval launch (rocprofv3 FETCH_SIZE+WRITE_SIZE, scaled)",
            "lds_issued_frac": B * LDS_BYTES_ISSUED_PER_EVAL / (eval_ms * 1e-3) / 1e9 / PEAK_LDS_GBS if (cmp and lane_layout) else None,
            "alu": {"achieved": lane_tops, "peak": PEAK_LANE_TOPS, "unit": "T 32-bit lane-ops/s",
                    "frac": lane_tops / PEAK_LANE_TOPS, "lane_ops_per_eval": LANE_OPS_PER_EVAL} if (cmp and lane_layout) else None,
            "hbm": {"achieved": hbm_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": hbm_gbs / PEAK_HBM_GBS,
                    "bytes_per_eval": hbm_per_eval},
        },
    }
    props = torch.cuda.get_device_properties(dev)
    out["device"] = {"name": props.name, "arch": getattr(props, "gcnArchName", None), "compute_units": props.multi_processor_count,
                     "lds_per_workgroup": getattr(props, "shared_memory_per_block", None)}
    if args.cpu_sample > 0 and cmp:
        out["cpu_baseline"] = cpu_baseline(args.cpu_sample)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
