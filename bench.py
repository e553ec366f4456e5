#!/usr/bin/env python3
"""Benchmark of the Beaver-multiplication hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input, every
leg the configuration names:
  configs 1, 3, 5  share X, Y -> Beaver matmul (open E, F; share update) -> trunc ->
                   elementwise Beaver mul of the result with a shared tensor -> trunc
  config 2         the same on the 1024^3 product, then share + elementwise Beaver
                   mul + trunc on the 2^24-element vectors
  config 4         Q.K^T (key matrix stored transposed, spin_beaver_matmul_nt) -> trunc ->
                   elementwise Beaver mul over the 8x8x128x128 scores -> trunc -> P.V -> trunc
Default workload: configuration 5 (5 parties, 4096^3, f = 16), the headline
configuration; --config all prints one line per configuration.  All inputs are
resident in HBM before the timed region.

Prints ONE JSON line per configuration (metric: Z_2^64 ring MACs/s of the Beaver
matmuls, counted as n*2*batch*M*N*K per product), with the roofline of the
dominant kernel and the CPU oracle timed on the host cores; the oracle's rows
are also compared with the Z the timed steps left behind.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0       # MI355X dense int8 MFMA peak, TOP/s (published 5.0 POP/s)
PEAK_HBM_GBS = 8000.0
INT8_OPS_PER_RING_MAC = 72    # 36 digit pairs x (multiply + add)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="5", choices=["1", "2", "3", "4", "5", "all"],
                    help="benchmark configuration (default 5, the headline); all: one JSON line per configuration")
    ap.add_argument("--path", default="limb", choices=["limb", "valu"])
    ap.add_argument("--workload", default="matmul", choices=["matmul", "poly", "matmul128", "matmul32", "grouped", "binary"],
                    help="matmul: the Beaver-matmul hot path (the benchmark); poly: completed-square polynomial "
                         "evaluation (Section 7.2 Eq. (4)) on the configuration's vector length; matmul128 / matmul32: the "
                         "Beaver matmul over the other two ring widths; grouped: the attention products of three "
                         "LeViT-like stages submitted as one spin_beaver_matmul_grouped call against one call per product; "
                         "binary: XOR sharing, XOR open and the AND-triple update on 2^24 packed words")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time its replays (for the launch-bound small "
                         "configurations; the per-kernel figures then come from a separate eager pass)")
    ap.add_argument("--fuse-mul-trunc", action="store_true",
                    help="run the elementwise multiplication and its truncation as the one-pass spin_beaver_mul_trunc")
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle leg (and with it the check of the timed Z against the oracle)")
    ap.add_argument("--no-mfma-ceiling", dest="mfma_ceiling", action="store_false",
                    help="skip the register-only MFMA rate probe that follows the timed steps")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def measured_traffic(kernel, cfg):
    """HBM-side bytes per launch from the committed rocprofv3 counter summaries (FETCH_SIZE and WRITE_SIZE
    passes, calibrated against a plain copy), or None where no summary covers this kernel and workload."""
    want = ["traffic_bytes_per_launch", kernel, "config%d" % cfg]
    for name in sorted(os.listdir(os.path.join(ROOT, "profiles"))) if os.path.isdir(os.path.join(ROOT, "profiles")) else []:
        try:
            for line in open(os.path.join(ROOT, "profiles", name)):
                parts = line.split()
                if len(parts) == 4 and parts[:3] == want:
                    return int(parts[3])
        except OSError:
            pass
    return None


def mfma_ceiling(kernel_tops):
    """The int8 MFMA rate this chip sustains on this machine, from a register-only loop of the GEMM's MFMA
    pattern (spin_probe_mfma): on all-zero operands and on uniformly random operand bytes, which is what the
    digits of masked shares are.  The published peak stays the roofline; these two figures say how much of
    the gap to it is the chip's clock under this data rather than the kernel."""
    import torch
    from paper_2402_02320_amd import spin
    blocks, iters = 1024, 2000
    sink = torch.empty(blocks * 256, dtype=torch.int64, device="cuda")
    res = {}
    for name, ops in (("zero_operands", torch.zeros(24 * 128, dtype=torch.int64, device="cuda")),
                      ("random_operands", spin.random(24 * 128, 0x5350494E, 99, 0))):
        spin.probe_mfma(ops, blocks, iters, sink)                # warm-up
        torch.cuda.synchronize()
        spin.profile_reset()
        spin.profile_enable(True)
        for _ in range(3):
            spin.probe_mfma(ops, blocks, iters, sink)
        torch.cuda.synchronize()
        spin.profile_enable(False)
        ms, cnt = spin.profile_read("probe")
        spin.profile_reset()
        tops = blocks * 4 * iters * spin.PROBE_OPS_PER_WAVE_ITERATION / (ms / cnt * 1e-3) / 1e12
        res[name] = {"TOP/s": tops, "frac_of_peak": tops / PEAK_INT8_TOPS}
    res["kernel_over_random_ceiling"] = kernel_tops / res["random_operands"]["TOP/s"]
    res["what"] = "register-only loop of the limb GEMM's 72-MFMA k-step, 1024 workgroups x 2000 iterations"
    return res


def cpu_baseline(cfg, target_s, gpu_rows_of_z=None):
    """The oracle, as it stands, on a bounded row sample of the first GEMM of the configuration: seeded inputs and the
    dealer's triple from oracle/ alone, timed on all host cores.  gpu_rows_of_z(rows) returns the same rows of the Z
    the timed GPU steps produced; they must equal the oracle's word for word."""
    import oracle
    from paper_2402_02320_amd import workloads
    c = workloads.CONFIGS[cfg]
    Xr, Yr = workloads.gemm_plaintexts(cfg)
    batch, M, K = Xr.shape
    N = Yr.shape[2]
    X = oracle.share(oracle.encode(Xr, c.f), c.n, c.seed, oracle.STREAM_X)
    Y = oracle.share(oracle.encode(Yr, c.f), c.n, c.seed, oracle.STREAM_Y)
    A, B, C = oracle.dealer_matmul(c.n, batch, M, N, K, seed=c.seed)        # untimed: the offline phase
    threads = oracle.threads()

    def run(rows):
        t0 = time.perf_counter()
        z = oracle.beaver_matmul(X, Y, A, B, C, rows=rows)
        return time.perf_counter() - t0, z

    def spread(nrows):
        return np.unique(np.linspace(0, M - 1, nrows).astype(np.int32))
    probe_rows = min(M, 2 * threads)
    t_probe, _ = run(spread(probe_rows))
    # the opening of E and F is paid once per call whatever the row count; estimate it from a second probe
    t_probe2, _ = run(spread(min(M, 4 * threads)))
    per_row = max((t_probe2 - t_probe) / max(1, min(M, 4 * threads) - probe_rows), 1e-9)
    nrows = int(max(probe_rows, min(M, (target_s - max(t_probe - per_row * probe_rows, 0.0)) / per_row)))
    nrows = min(M, max(threads, nrows // threads * threads))
    rows = spread(nrows)
    nrows = int(rows.size)
    t, z_rows = run(rows)
    checked = None
    if gpu_rows_of_z is not None:
        got = gpu_rows_of_z(rows)
        if got.shape != z_rows.shape or not (got == z_rows).all():
            raise SystemExit("bench.py: the Z the timed GPU steps produced differs from the oracle on the sampled rows")
        checked = nrows * batch
    macs = (2 * c.n + 1) * batch * nrows * N * K     # the oracle also forms E.F explicitly for party 0
    credited = 2 * c.n * batch * nrows * N * K
    # per-core figure: the row loop alone on one thread (the opening is subtracted through a second run)
    oracle.set_threads(1)
    r1 = max(1, nrows // (4 * threads))
    (t_a, _), (t_b, _) = run(spread(r1)), run(spread(min(M, 2 * r1)))
    oracle.set_threads(threads)
    one_core = 2 * c.n * batch * max(1, min(M, 2 * r1) - r1) * N * K / max(t_b - t_a, 1e-9)
    model = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    res = {"value": credited / t, "unit": "ring MAC/s", "cores": threads, "cpu_model": model, "kind": "oracle",
           "sample": "config %d, first GEMM, %d of %d output rows (x %d batch entries) of every party's share (%.1f s, "
                     "incl. opening E and F; %.3g ring MACs executed, %.3g credited as n*2*rows*N*K)"
                     % (cfg, nrows, M, batch, t, macs, credited),
           "one_core_value": one_core,
           "one_core_sample": "row loop on 1 thread: time of %d rows minus time of %d rows" % (min(M, 2 * r1), r1)}
    return res, checked


def bench_poly(args):
    """Side workload: f1' (completed square, two Beaver multiplications, fused (p+6)-bit truncation) on a vector."""
    import torch
    from paper_2402_02320_amd import poly, spin, workloads
    c = workloads.CONFIGS[args.config]
    n, p = c.n, 14
    count = c.vec if c.vec else c.gemms[0].batch * c.gemms[0].M * c.gemms[0].N
    t3, t2, t1, t0 = 0.96074360, 6.15066406, 24.02000383, 23.85013773      # Appendix B, f1
    z = torch.rand(count, dtype=torch.float64, device="cuda")
    x = spin.share(spin.encode(z, p), n, c.seed, 1)

    def party_random(stream):
        return torch.stack([spin.random(count, c.seed, stream, i) for i in range(n)])

    def triple(s0):
        a, b = party_random(s0), party_random(s0 + 1)
        return a, b, spin.share(spin.open(a) * spin.open(b), n, c.seed, s0 + 2)

    def trunc_tuple(f, s0):
        r_sh = party_random(s0)
        r = spin.open(r_sh)
        return r_sh, spin.share((r >> f) & ((1 << (63 - f)) - 1), n, c.seed, s0 + 1), \
            spin.share((r >> 63) & 1, n, c.seed, s0 + 2)
    triples = [triple(20), triple(30)]
    tuples = [trunc_tuple(p, 40), trunc_tuple(p + 6, 50)]

    def step():
        return poly.evaluate_completed_square(x, -6, t3, t2, t1, t0, p, triples, tuples)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    spin.profile_reset()
    spin.profile_enable(True)
    t_begin = time.perf_counter()
    for _ in range(args.steps):
        y = step()
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    spin.profile_enable(False)
    ms = (t_end - t_begin) * 1e3 / args.steps
    err = float((spin.decode(spin.open(y), p) * (0.01353417 / 2.0 ** -6) - torch.exp2(z)).abs().max())
    el = 8.0 * count
    # per step: lincomb (x+t3): 2n; mul: 6n (u read twice counts once: 5n+... u,u,a,b,c in, out) ; trunc 5n;
    # lincomb (+t2) 2n; mul 6n; lincomb+trunc (2 terms + tuple): 6n  -- element-sized transfers per party
    alg = {"lincomb": (2 * n + 2 * n + 6 * n) * el / 3, "beaver_mul": 5 * n * el, "trunc": 5 * n * el}
    kernels = {}
    for k, b in alg.items():
        tot, cnt = spin.profile_read(k)
        if cnt:
            kernels[k] = {"GB/s": b / (tot / cnt * 1e-3) / 1e9, "avg_ms": tot / cnt, "launches_per_step": cnt / args.steps}
    spin.profile_reset()
    print(json.dumps({"metric": "completed-square polynomial evaluations/s (side workload)", "value": count / (ms * 1e-3),
                      "unit": "elements/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
                      "higher_is_better": True, "vs_baseline": None, "dtype": "u64", "data": "synthetic",
                      "config": {"workload": "f1' of Section 7.2 Eq. (4) on %d elements, %d parties, p=14" % (count, n)},
                      "max_abs_error_vs_2^z": err, "stream_kernels": kernels}))


def bench_binary(args):
    """Side workload: the local work on binary shares (Section 4.1 binary sharing, Section 4.3 XOR) -- share two packed
    64-lane words per element, the AND-triple update (the GF(2) Beaver multiplication), open the result -- on 2^24
    words, 3 parties.  The opened result is checked against x & y of the inputs after the timed steps."""
    import torch
    from paper_2402_02320_amd import spin
    n, count, seed = 3, 1 << 24, 7
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    x = torch.randint(-2 ** 63, 2 ** 63 - 1, (count,), dtype=torch.int64, device="cuda", generator=g)
    y = torch.randint(-2 ** 63, 2 ** 63 - 1, (count,), dtype=torch.int64, device="cuda", generator=g)
    a = torch.stack([spin.random(count, seed, 21, i) for i in range(n)])
    b = torch.stack([spin.random(count, seed, 22, i) for i in range(n)])
    c = spin.bshare(spin.bopen(a) & spin.bopen(b), n, seed, 23)
    xs, ys, zs = torch.empty_like(a), torch.empty_like(a), torch.empty_like(a)
    z = torch.empty_like(x)

    def step():
        spin.bshare(x, n, seed, 1, out=xs)
        spin.bshare(y, n, seed, 2, out=ys)
        spin.beaver_and(xs, ys, a, b, c, out=zs)
        spin.bopen(zs, out=z)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    spin.profile_reset()
    spin.profile_enable(True)
    t_begin = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    spin.profile_enable(False)
    ms = (t_end - t_begin) * 1e3 / args.steps
    tot, cnt = spin.profile_read("binary")
    spin.profile_reset()
    if not torch.equal(z, x & y):
        raise SystemExit("bench.py: the opened AND differs from x & y")
    # words of 8 bytes per element and step: two sharings (1 in, n out each), the update (5n in, n out), the open (n in, 1 out)
    words = 2 * (1 + n) + 6 * n + (n + 1)
    print(json.dumps({"metric": "packed 64-lane binary-share AND evaluations/s (side workload)", "value": count / (ms * 1e-3),
                      "unit": "words/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
                      "higher_is_better": True, "vs_baseline": None, "dtype": "u64", "data": "synthetic",
                      "config": {"workload": "bshare x, y; beaver_and; bopen on %d words, %d parties" % (count, n)},
                      "parity": "opened result equals x & y on all words",
                      "roofline": {"bound": "hbm", "achieved": words * 8.0 * count / (tot / args.steps * 1e-3) / 1e9,
                                   "peak": 8000.0, "unit": "GB/s",
                                   "frac": words * 8.0 * count / (tot / args.steps * 1e-3) / 8e12,
                                   "kernel": "bshare, beaver_and, bopen kernels together",
                                   "kernel_ms_per_step": tot / args.steps, "launches_per_step": cnt / args.steps,
                                   "traffic": None}}))


def bench_matmul_other_ring(args, bits):
    """Side workloads: the Beaver matmul over Z_2^128 (16 digits, 136 digit pairs per ring MAC; 2 parties,
    2048^3) and over Z_2^32 (4 digits, 10 digit pairs; 2 parties, 8192^3)."""
    import torch
    from paper_2402_02320_amd import spin
    R = spin.ring128 if bits == 128 else spin.ring32
    n, M = (2, 2048) if bits == 128 else (2, 8192)
    pairs = 136 if bits == 128 else 10
    path = spin.LIMB_MFMA if args.path == "limb" else spin.VALU

    def rnd(shape):
        if bits == 128:
            return torch.empty(shape + (2,), dtype=torch.int64, device="cuda").random_(-2 ** 62, 2 ** 62)
        return torch.empty(shape, dtype=torch.int32, device="cuda").random_(-2 ** 31, 2 ** 31)
    X, Y, A, B, C = (rnd((n, 1, M, M)) for _ in range(5))
    Z = torch.empty_like(C)
    ws = torch.empty(R.beaver_matmul_workspace_bytes(n, 1, M, M, M, path), dtype=torch.uint8, device="cuda")
    for _ in range(args.warmup):
        R.beaver_matmul(X, Y, A, B, C, path=path, out=Z, workspace=ws)
    torch.cuda.synchronize()
    spin.profile_reset()
    spin.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        R.beaver_matmul(X, Y, A, B, C, path=path, out=Z, workspace=ws)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    spin.profile_enable(False)
    macs = 2.0 * n * M * M * M
    key = "gemm_limb" if path == spin.LIMB_MFMA else "gemm_valu"
    tot, cnt = spin.profile_read(key)
    pk, pc = spin.profile_read("pack")
    spin.profile_reset()
    gemm_ms = tot / cnt
    roof = None
    if path == spin.LIMB_MFMA:
        ach = macs * 2 * pairs / (cnt / args.steps) / (gemm_ms * 1e-3) / 1e12      # digit pairs x (multiply + add)
        roof = {"bound": "mfma", "kernel": "limb128_gemm_kernel" if bits == 128 else "limb_gemm_kernel<unsigned int>",
                "achieved": ach, "peak": PEAK_INT8_TOPS, "unit": "TOP/s", "frac": ach / PEAK_INT8_TOPS,
                "traffic": None, "avg_launch_ms": gemm_ms}
    ring = "u%d" % bits
    print(json.dumps({"metric": "Z_2^%d ring MACs/s for Beaver matmul (side workload)" % bits,
                      "value": macs / (ms * 1e-3), "unit": "ring MAC/s", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "vs_baseline": None,
                      "dtype": ring + " (int8 digits, int32 accumulate)" if path == spin.LIMB_MFMA else ring,
                      "data": "synthetic",
                      "config": {"workload": "%d parties, M=N=K=%d over Z_2^%d" % (n, M, bits), "gemm_path": args.path},
                      "roofline": roof, "gemm_avg_ms": gemm_ms, "pack_avg_ms": pk / pc if pc else None}))


def bench_grouped(args):
    """Side workload (Section 7.4, PMatMul): the Q.K^T and P.V products of three attention stages of different
    shapes (196, 49 and 16 tokens), 3 parties, as ONE grouped call (shared launches) and as one call per product,
    both eager on the same stream."""
    import torch
    from paper_2402_02320_amd import spin
    n = 3
    shapes = [(4, 196, 196, 64, True), (4, 196, 64, 196, False), (8, 49, 49, 32, True), (8, 49, 32, 49, False),
              (12, 16, 16, 32, True), (12, 16, 32, 16, False)]

    def rnd(shape):
        return torch.empty(shape, dtype=torch.int64, device="cuda").random_(-2 ** 62, 2 ** 62)
    groups, macs = [], 0.0
    for batch, M, N, K, yt in shapes:
        yshape = (n, batch, N, K) if yt else (n, batch, K, N)
        groups.append({"X": rnd((n, batch, M, K)), "Y": rnd(yshape), "A": rnd((n, batch, M, K)), "B": rnd(yshape),
                       "C": rnd((n, batch, M, N)), "out": torch.empty((n, batch, M, N), dtype=torch.int64, device="cuda"),
                       "y_transposed": yt})
        macs += 2.0 * n * batch * M * N * K
    ws = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")

    def grouped():
        spin.beaver_matmul_grouped(groups, workspace=ws)

    def one_by_one():
        for g in groups:
            spin.beaver_matmul(g["X"], g["Y"], g["A"], g["B"], g["C"], out=g["out"], workspace=ws,
                               y_transposed=g["y_transposed"])
    res = {}
    for name, fn in (("grouped", grouped), ("one_call_per_product", one_by_one)):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        res[name] = (time.perf_counter() - t0) * 1e3 / args.steps
    ref = [g["out"].clone() for g in groups]
    grouped()
    torch.cuda.synchronize()
    same = all(torch.equal(a, g["out"]) for a, g in zip(ref, groups))
    print(json.dumps({"metric": "Z_2^64 ring MACs/s, grouped Beaver matmuls of three attention stages (side workload)",
                      "value": macs / (res["grouped"] * 1e-3), "unit": "ring MAC/s", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "ms_per_step": res["grouped"], "higher_is_better": True, "vs_baseline": None,
                      "dtype": "u64 (int8 digits, int32 accumulate)", "data": "synthetic",
                      "config": {"workload": "3 parties, 6 products (batch, M, N, K, right operand transposed): %s" % shapes,
                                 "launch": "eager"},
                      "ms_one_call_per_product": res["one_call_per_product"],
                      "speedup_over_one_call_per_product": res["one_call_per_product"] / res["grouped"],
                      "same_words_as_one_call_per_product": same}))


def run_config(args, cfg):
    """Times the hot path on one configuration and returns the JSON record."""
    import torch
    from paper_2402_02320_amd import spin, workloads
    c = workloads.CONFIGS[cfg]
    n, f = c.n, c.f
    path = spin.LIMB_MFMA if args.path == "limb" else spin.VALU
    S = {"X": 1, "Y": 2, "A": 3, "B": 4, "C": 5, "R": 6, "RT": 7, "RM": 8, "W": 9}
    alg_bytes = {}                 # algorithmic bytes per step of the HBM-bound kernel classes

    def count_bytes(kernel, nbytes):
        alg_bytes[kernel] = alg_bytes.get(kernel, 0.0) + nbytes

    def party_random(count, stream, shape, seed):
        return torch.stack([spin.random(count, seed, stream, i) for i in range(n)]).view((n,) + shape)

    def trunc_tuple(count, seed):
        r_sh = torch.stack([spin.random(count, seed, S["R"], i) for i in range(n)])
        r = spin.open(r_sh)
        r_top = (r >> f) & ((1 << (63 - f)) - 1)
        r_msb = (r >> 63) & 1
        return r_sh, spin.share(r_top, n, seed, S["RT"]), spin.share(r_msb, n, seed, S["RM"])

    def matmul_triple(batch, M, N, K, seed):
        """A_i, B_i from the generator, C = (sum A_i).(sum B_i) through the library's own ring GEMM (one party, zero
        triple), then shared: exactly what the oracle's dealer computes.  The GEMM runs on the VALU path so that every
        limb-GEMM launch a profiler sees belongs to the workload."""
        A = party_random(batch * M * K, S["A"], (batch, M, K), seed)
        B = party_random(batch * K * N, S["B"], (batch, K, N), seed)
        ws1 = torch.empty(spin.beaver_matmul_workspace_bytes(1, batch, M, N, K, spin.VALU), dtype=torch.uint8,
                          device="cuda")
        a_open, b_open = spin.open(A)[None], spin.open(B)[None]
        zC = torch.zeros((1, batch, M, N), dtype=torch.int64, device="cuda")
        c_plain = spin.beaver_matmul(a_open, b_open, torch.zeros_like(a_open), torch.zeros_like(b_open), zC,
                                     path=spin.VALU, workspace=ws1)
        return A, B, spin.share(c_plain[0], n, seed, S["C"])

    def mul_triple(count, seed):
        ea = torch.stack([spin.random(count, seed, 11, i) for i in range(n)])
        eb = torch.stack([spin.random(count, seed, 12, i) for i in range(n)])
        return ea, eb, spin.share(spin.open(ea) * spin.open(eb), n, seed, 13)

    # ---- untimed set-up: plaintexts, triples and truncation tuples, all resident in HBM ----------------
    steps_list = []                # callables of one step, in order
    ring_macs = 0.0
    legs = []
    gemm_z = []                    # Z of every GEMM leg
    ws_bytes = 0
    gemm_plans = []
    all_rows = True
    for gi, g in enumerate(c.gemms):
        Xr, Yr = workloads.gemm_plaintexts(cfg, gi)
        batch, M, K = Xr.shape
        N = Yr.shape[2]
        transposed = g.name == "qkT"               # the key matrix is stored [N][K]: Q.K^T through spin_beaver_matmul_nt
        gemm_plans.append((gi, g, Xr, Yr, batch, M, N, K, transposed))
        ws_bytes = max(ws_bytes, spin.beaver_matmul_workspace_bytes(n, batch, M, N, K, path))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    prev_out = None                # truncated shares produced by the previous leg (config 4: the scores feed P.V)
    for gi, g, Xr, Yr, batch, M, N, K, transposed in gemm_plans:
        seed = c.seed + 0x10 * gi
        szA, szB, szC = batch * M * K, batch * K * N, batch * M * N
        A, B, C = matmul_triple(batch, M, N, K, seed)
        y_plain = spin.encode(torch.from_numpy(Yr).cuda(), f)
        if transposed:
            y_plain = y_plain.transpose(1, 2).contiguous()
            B = B.transpose(2, 3).contiguous()
        Ys = torch.empty((n,) + tuple(y_plain.shape), dtype=torch.int64, device="cuda")
        Z = torch.empty((n, batch, M, N), dtype=torch.int64, device="cuda")
        T = torch.empty((n, szC), dtype=torch.int64, device="cuda")
        tup = trunc_tuple(szC, seed + 0x100)
        chained = cfg == 4 and gi == 1 and prev_out is not None
        if chained:
            Xs = prev_out.view(n, batch, M, K)     # P = the multiplied, truncated scores of the previous legs
            x_plain = None
        else:
            x_plain = spin.encode(torch.from_numpy(Xr).cuda(), f)
            Xs = torch.empty((n, batch, M, K), dtype=torch.int64, device="cuda")

        def leg(x_plain=x_plain, y_plain=y_plain, Xs=Xs, Ys=Ys, A=A, B=B, C=C, Z=Z, T=T, tup=tup, seed=seed,
                transposed=transposed):
            if x_plain is not None:
                spin.share(x_plain, n, seed, S["X"], out=Xs)
            spin.share(y_plain, n, seed, S["Y"], out=Ys)
            spin.beaver_matmul(Xs, Ys, A, B, C, path=path, out=Z, workspace=ws, y_transposed=transposed)
            spin.trunc(Z.view(n, -1), tup[0], tup[1], tup[2], f, out=T)
        steps_list.append(leg)
        gemm_z.append(Z)
        ring_macs += 2.0 * n * batch * M * N * K
        count_bytes("share", (1 + n) * 8.0 * (szB + (0 if chained else szA)))
        count_bytes("trunc", 5 * n * 8.0 * szC)
        # left fragments built inside the GEMM (the library's own rule also weighs a cost model; these shapes pass it)
        fused_left = path == spin.LIMB_MFMA and n <= 3 and K % 2 == 0 and (N <= 64 or (N <= 128 and K <= 128))
        all_rows = all_rows and fused_left
        count_bytes("pack", 8.0 * (3 * n + 1) * (szB + (0 if fused_left else szA)))
        legs.append("%sBeaver matmul %s batch %d M=%d N=%d K=%d (%s) + trunc"
                    % ("" if chained else "share X, ", g.name, batch, M, N, K,
                       "share Y, spin_beaver_matmul_nt" if transposed else "share Y, spin_beaver_matmul"))
        prev_out = T
        # elementwise leg on this GEMM's truncated output (configs without vectors of their own; config 4: the scores)
        if (c.vec == 0 and gi == 0) or (cfg == 4 and gi == 0):
            count = szC
            ea, eb, ec = mul_triple(count, seed)
            w = spin.share(spin.encode(torch.from_numpy(workloads.vec_plaintexts(cfg, count)[0]).cuda(), f), n, seed, S["W"])
            V = torch.empty((n, count), dtype=torch.int64, device="cuda")
            tup2 = trunc_tuple(count, seed + 0x200)

            def mul_leg(T=T, w=w, ea=ea, eb=eb, ec=ec, V=V, tup2=tup2):
                if args.fuse_mul_trunc:
                    spin.beaver_mul_trunc(T, w, ea, eb, ec, tup2[0], tup2[1], tup2[2], f, out=V)
                else:
                    spin.beaver_mul(T, w, ea, eb, ec, out=V)
                    spin.trunc(V, tup2[0], tup2[1], tup2[2], f, out=V)
            steps_list.append(mul_leg)
            if args.fuse_mul_trunc:
                count_bytes("beaver_mul_trunc", 9 * n * 8.0 * count)
            else:
                count_bytes("beaver_mul", 6 * n * 8.0 * count)
                count_bytes("trunc", 5 * n * 8.0 * count)
            legs.append("elementwise Beaver mul of the result with a shared tensor (%d elements) + trunc" % count)
            prev_out = V
    if c.vec and cfg != 4:
        # the configuration's own vectors (config 2: 2^24 elements): share both, multiply, truncate
        L = c.vec
        xr, yr = workloads.vec_plaintexts(cfg)
        xv = spin.encode(torch.from_numpy(xr).cuda(), f)
        yv = spin.encode(torch.from_numpy(yr).cuda(), f)
        Xv = torch.empty((n, L), dtype=torch.int64, device="cuda")
        Yv = torch.empty((n, L), dtype=torch.int64, device="cuda")
        ea, eb, ec = mul_triple(L, c.seed + 0x40)
        tupv = trunc_tuple(L, c.seed + 0x300)
        Vv = torch.empty((n, L), dtype=torch.int64, device="cuda")

        def vec_leg():
            spin.share(xv, n, c.seed, S["X"] + 20, out=Xv)
            spin.share(yv, n, c.seed, S["Y"] + 20, out=Yv)
            if args.fuse_mul_trunc:
                spin.beaver_mul_trunc(Xv, Yv, ea, eb, ec, tupv[0], tupv[1], tupv[2], f, out=Vv)
            else:
                spin.beaver_mul(Xv, Yv, ea, eb, ec, out=Vv)
                spin.trunc(Vv, tupv[0], tupv[1], tupv[2], f, out=Vv)
        steps_list.append(vec_leg)
        count_bytes("share", 2 * (1 + n) * 8.0 * L)
        if args.fuse_mul_trunc:
            count_bytes("beaver_mul_trunc", 9 * n * 8.0 * L)
        else:
            count_bytes("beaver_mul", 6 * n * 8.0 * L)
            count_bytes("trunc", 5 * n * 8.0 * L)
        legs.append("share + elementwise Beaver mul + trunc on %d-element vectors" % L)

    def step():
        for leg in steps_list:
            leg()

    # one plain copy of known size (open of a single share: out[k] = shares[0][k]); the HBM byte counters
    # of a profiler run are calibrated against what they read for this launch (1 GiB in, 1 GiB out)
    calib = torch.empty((1, 1 << 27), dtype=torch.int64, device="cuda").fill_(3)
    calib_out = spin.open(calib)
    del calib, calib_out

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    spin.profile_reset()
    if args.graph:
        # event pairs cannot be recorded into a captured graph: per-kernel durations come from an eager pass
        # first, the timed region replays the captured step
        spin.profile_enable(True)
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        spin.profile_enable(False)
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        step_ms = None
    else:
        spin.profile_enable(True)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks[0].record()
        for i in range(args.steps):
            step()
            marks[i + 1].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        spin.profile_enable(False)
        step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kernels = {k: spin.profile_read(k) for k in spin.KERNELS}
    spin.profile_reset()
    gemm_key = "gemm_limb" if path == spin.LIMB_MFMA else "gemm_valu"
    gemm_ms, gemm_launches = kernels[gemm_key]
    pack_ms = kernels["pack"][0] if path == spin.LIMB_MFMA else kernels["open"][0]
    launches_per_step = gemm_launches / args.steps
    gemm_avg_ms = gemm_ms / gemm_launches
    gemm_ms_per_step = gemm_ms / args.steps
    if path == spin.LIMB_MFMA:
        # all GEMM launches of a step together: algorithmic int8 operations / their summed kernel time
        achieved = ring_macs * INT8_OPS_PER_RING_MAC / (gemm_ms_per_step * 1e-3) / 1e12
        with_pack = ring_macs * INT8_OPS_PER_RING_MAC / ((gemm_ms + pack_ms) / args.steps * 1e-3) / 1e12
        # which GEMM kernel the library picks: the row-streaming one for products of few column tiles, at most
        # three parties and an even inner dimension (it builds the left fragments itself), else the tile kernel
        kernel_name = "limb_gemm_rows_kernel" if all_rows else "limb_gemm_kernel"
        traffic = measured_traffic(kernel_name, cfg)
        roofline = {"bound": "mfma", "kernel": kernel_name, "achieved": achieved, "peak": PEAK_INT8_TOPS,
                    "unit": "TOP/s", "frac": achieved / PEAK_INT8_TOPS, "traffic": traffic,
                    "traffic_source": ("profiles/ (config %d): rocprofv3 FETCH_SIZE / WRITE_SIZE of an earlier run of "
                                       "this command, not measured in this run" % cfg) if traffic else None,
                    "avg_launch_ms": gemm_avg_ms, "launches_per_step": launches_per_step,
                    "ring_mac_per_s": ring_macs / (gemm_ms_per_step * 1e-3),
                    "frac_with_pack": with_pack / PEAK_INT8_TOPS,
                    "note": "frac = int8 operations of all limb-GEMM launches of a step / their kernel time; frac_with_pack "
                            "also counts the pack kernels that open E, F and split the operands into digits"}
    else:
        # 64-bit multiply-add on the vector ALU: 256 CUs x 4 SIMDs x 16 lanes per clock at 2.4 GHz; the compiled
        # inner loop spends four VALU instructions per ring MAC (v_mad_u64_u32, 2 x v_mul_lo_u32, v_add3_u32),
        # each taken at full rate
        peak = 256 * 4 * 16 * 2.4e9 / 4 / 1e12
        achieved = ring_macs / (gemm_ms_per_step * 1e-3) / 1e12
        roofline = {"bound": "alu", "kernel": "valu_gemm_kernel", "achieved": achieved, "peak": peak,
                    "unit": "T ring MAC/s", "frac": achieved / peak, "traffic": None, "traffic_source": None,
                    "avg_launch_ms": gemm_avg_ms, "launches_per_step": launches_per_step}
    # HBM-bound side kernels: algorithmic bytes of all their launches in a step / their summed event time
    streams = {}
    for k, b in alg_bytes.items():
        ms, cnt = kernels[k]
        if cnt:
            rate = b * args.steps / (ms * 1e-3) / 1e9
            streams[k] = {"GB/s": rate, "frac_hbm": rate / PEAK_HBM_GBS, "avg_ms": ms / cnt,
                          "launches_per_step": cnt / args.steps, "algorithmic_bytes_per_step": b}
    g0 = c.gemms[0]
    out = {
        "metric": "Z_2^64 ring MACs/s for Beaver matmul (1 GPU)", "value": ring_macs / (ms_per_step * 1e-3),
        "unit": "ring MAC/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64 (int8 digits, int32 accumulate)" if path == spin.LIMB_MFMA else "u64",
        "data": "synthetic",
        "config": {"workload": "config %d: %d parties, f=%d, %s; step = %s" % (cfg, n, f, c.dist, "; then ".join(legs)),
                   "gemm_path": args.path, "parties": n, "launch": "hip graph replay" if args.graph else "eager",
                   "mul_trunc": "one pass" if args.fuse_mul_trunc else "two calls",
                   "ring_macs_per_step": ring_macs},
        "roofline": roofline, "stream_kernels": streams,
        "step_ms_median": step_ms[len(step_ms) // 2] if step_ms else None, "step_ms_min": step_ms[0] if step_ms else None,
        "limb_roofline_ring_mac_per_s": PEAK_INT8_TOPS * 1e12 / INT8_OPS_PER_RING_MAC,
        # the protocol's view: one secure product of the plaintext shapes per step, whatever n
        "secure_matmul_mac_per_s": ring_macs / (2 * n) / (ms_per_step * 1e-3),
    }
    if path == spin.LIMB_MFMA and args.mfma_ceiling:
        out["mfma_ceiling"] = mfma_ceiling(roofline["achieved"])
    if not args.no_cpu_baseline:
        Z0 = gemm_z[0]

        def gpu_rows(rows):
            idx = torch.from_numpy(np.asarray(rows, dtype=np.int64)).cuda()
            return Z0.index_select(2, idx).cpu().numpy().view(np.uint64)
        steps_list.clear()
        torch.cuda.empty_cache()
        out["cpu_baseline"], out["parity_rows_checked"] = cpu_baseline(cfg, args.cpu_seconds, gpu_rows)
        out["parity"] = ("rows of the first GEMM's Z, as left by the timed steps, equal the oracle's word for word "
                         "(rows x batch entries, every party)")
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (all parties' shares live on one MI355X); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2402_02320_amd import spin
    if not os.path.exists(spin.LIB_PATH):
        from paper_2402_02320_amd import build
        build.build()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.workload == "poly":
        args.config = 5 if args.config == "all" else int(args.config)
        return bench_poly(args)
    if args.workload in ("matmul128", "matmul32"):
        return bench_matmul_other_ring(args, 128 if args.workload == "matmul128" else 32)
    if args.workload == "grouped":
        return bench_grouped(args)
    if args.workload == "binary":
        return bench_binary(args)
    configs = [1, 2, 3, 4, 5] if args.config == "all" else [int(args.config)]
    for cfg in configs:
        print(json.dumps(run_config(args, cfg)), flush=True)
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
