#!/usr/bin/env python3
"""Benchmark of the potq hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extras] [--no-cpu]

Headline ("step"): one stand-alone PoT dequant pass over a Llama-2-70B-shaped
decoder layer (q/o 8192x8192, k/v 1024x8192, gate/up 28672x8192, down
8192x28672: 855.6 M weights), 2-bit codes, group 128, all seven matrices in one
pot_dequant_batch launch, inputs resident in HBM: the steps rotate through
three layers' worth of codes and scales (0.68 GB) so that they are read from
HBM, not from the 256 MB last-level cache.  `value` is algorithmic bytes (codes
+ scales in, fp16 out) per second.  The same JSON line carries the roofline of
the dominant kernel, the CPU oracle timed on the host cores, and (unless
--no-extras) one row per workload of the benchmark description: the 3-bit pass
over the same layer, the 7B layer with its uniform-INT baseline, the single
4096x4096 matrix, the fused GEMV on the 7B and 70B shapes at 2 and 3 bits, the
fused MFMA GEMM on the 13B shapes, each with its fraction of the roof that
bounds it and its speed-up over the INT path.

All inputs are seeded synthetic tensors from workloads.py.  This run uses one
GPU; --gpus above 1 is refused.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_F16_PEAK_TFLOPS = 2500.0   # dense fp16 MFMA, published
CONFIG_INDEX = 3                # the Llama-2-70B layer workload (workloads.CONFIGS)
CODE_SETS = 3                   # layers' worth of codes and scales the timed steps rotate through (3 x 227 MB)
RAMP_UP = 100                   # untimed launches before the timed region (the first ~10 ms after idling run slow)

# HBM bytes per launch of the headline kernel by code width, from rocprofv3 FETCH_SIZE (x 2.000) + WRITE_SIZE
# (x 1.000), factors calibrated on a 256 MiB copy: measured once with the commands in the file named here, not
# re-measured by this script
PROFILED_TRAFFIC = {"bytes_per_launch": {2: 1938671360, 3: 2045564477},
                    "source": "profiles/pot_dequant_batch_llama70b_layer.md"}


def _events(torch):
    return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)


def _time_steps(torch, step, steps, warmup):
    """Average milliseconds per call of `step` over `steps` calls, HIP events on the launch stream."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = _events(torch)
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def _time_pair(torch, step_a, step_b, steps, warmup, reps=5):
    """Median milliseconds per call of two alternatives measured alternately (a, b, a, b, ...): the first
    measurement after an idle phase runs a few per cent slow, which a single a-then-b pass would charge to a."""
    ta, tb = [], []
    for _ in range(reps):
        ta.append(_time_steps(torch, step_a, steps, warmup))
        tb.append(_time_steps(torch, step_b, steps, warmup))
    ta.sort()
    tb.sort()
    return ta[len(ta) // 2], tb[len(tb) // 2]


def _hbm(nbytes, us):
    """Row fields of a launch bound by HBM: algorithmic bytes over time against the 8 TB/s peak."""
    gbps = nbytes / us / 1e3
    return {"us": round(us, 2), "GBps": round(gbps, 1), "bound": "hbm", "frac": round(gbps / HBM_PEAK_GBPS, 4)}


def _gemm_roof(M, N, K, nbytes, us):
    """Row fields of a fused GEMM: the roof is whichever of HBM time and fp16 MFMA time is longer."""
    flops = 2.0 * M * N * K
    t_hbm, t_mfma = nbytes / HBM_PEAK_GBPS / 1e3, flops / MFMA_F16_PEAK_TFLOPS / 1e6      # microseconds
    bound = "mfma" if t_mfma > t_hbm else "hbm"
    return {"us": round(us, 2), "TFLOPs": round(flops / us / 1e6, 1), "GBps": round(nbytes / us / 1e3, 1),
            "bound": bound, "frac": round(max(t_hbm, t_mfma) / us, 4),
            "pct_mfma_peak": round(flops / us / 1e6 / MFMA_F16_PEAK_TFLOPS * 100, 2)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--bits", type=int, default=2, choices=(2, 3), help="code width of the headline pass")
    ap.add_argument("--workload", default="70b", choices=("70b", "7b"),
                    help="layer of the headline pass: Llama-2-70B (default) or Llama-2-7B (ten rotating code sets; "
                         "for profiling runs, use with --no-extras)")
    ap.add_argument("--no-extras", action="store_true", help="headline only (used for profiling runs)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy a few times (reference kernel for byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import __graft_entry__
    __graft_entry__.ensure_built()          # loads what is built; builds only if the tree holds no library
    import paper_2507_11959_amd as potq     # raises if libpotq.so is still missing: there is no fallback path
    from paper_2507_11959_amd import binding
    import workloads

    lib = binding.raw()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream().cuda_stream
    G = workloads.GROUP
    gen = torch.Generator(device=dev)
    gen.manual_seed(workloads.seed_of(CONFIG_INDEX, 0, 9))
    turn = [0]

    def to_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    def check(status):
        if status != 0:
            raise RuntimeError(f"potq status {status}: {potq.strerror(status)}")

    def random_codes(N, K, bits):        # uniformly random bytes are uniformly random codes
        return torch.randint(0, 256, (N, K * bits // 8), dtype=torch.uint8, device=dev, generator=gen)

    def permuted(t):                      # same values, other places: same distribution, other bytes
        perm = torch.randperm(t.numel(), device=dev, generator=gen)
        return t.flatten()[perm].reshape(t.shape).contiguous()

    class Layer:
        """A decoder layer's matrices for the stand-alone dequant: `sets` rotating sets of codes and scales
        (set 0 is the seeded workload of the parity tests, the others are device-side random bytes and
        permutations of the seeded scales) that all write the same output buffers."""

        def __init__(self, config, shapes, bits, sets, with_int=False, keep_host=False):
            self.shapes, self.bits, self.n_sets = shapes, bits, sets
            self.outs = [torch.empty((N, K), dtype=torch.float16, device=dev) for _, N, K in shapes]
            self.host = []
            first = []
            for i, (_, N, K) in enumerate(shapes):
                codes, scales = workloads.pot_matrix(config, i, N, K, bits, G)
                if keep_host:
                    self.host.append((codes, scales, K))
                S = Z = None
                if with_int:
                    S, Z = (to_dev(a) for a in workloads.int_scales_zeros(workloads.seed_of(config, i, 3), N, K, bits, G))
                first.append((to_dev(codes), to_dev(scales), S, Z))
            self.sets = [first]
            for _ in range(1, sets):
                self.sets.append([(random_codes(N, K, bits), permuted(f[1]),
                                   permuted(f[2]) if with_int else None, permuted(f[3]) if with_int else None)
                                  for f, (_, N, K) in zip(first, shapes)])
            self.pot_items = [binding.make_batch([(c, s, None, o, K, bits) for (c, s, _, _), o, (_, _, K)
                                                  in zip(layer, self.outs, shapes)]) for layer in self.sets]
            self.int_items = [binding.make_batch([(c, S, Z, o, K, bits) for (c, _, S, Z), o, (_, _, K)
                                                  in zip(layer, self.outs, shapes)], is_int=True)
                              for layer in self.sets] if with_int else None
            self.pot_bytes = sum(workloads.algorithmic_bytes_dequant(N, K, bits, G) for _, N, K in shapes)
            self.int_bytes = sum(workloads.algorithmic_bytes_dequant(N, K, bits, G, True) for _, N, K in shapes)
            self.weights = sum(N * K for _, N, K in shapes)

        def pot_step(self):                # the whole layer in one launch, the next set's codes every step
            turn[0] += 1
            check(lib.pot_dequant_batch(self.pot_items[turn[0] % self.n_sets], len(self.shapes), self.bits, G, stream))

        def int_step(self):
            turn[0] += 1
            check(lib.int_dequant_batch(self.int_items[turn[0] % self.n_sets], len(self.shapes), self.bits, G, stream))

        def ramp_up(self, n=RAMP_UP):
            for _ in range(n):
                self.pot_step()
            torch.cuda.synchronize()

    # ---------------------------------------------------------------- headline: 70B layer dequant
    # The codes and scales of one layer (227 MB at 2 bits) would partly stay in the 256 MB last-level cache if
    # every step re-read the same buffers; a decoder walks distinct layers, so the steps rotate through
    # CODE_SETS layers' worth.  Whatever --warmup says, RAMP_UP untimed launches come first so that the timed
    # region sees the steady state (clock ramp-up, cold address translation).
    bits = args.bits
    if args.workload == "7b":
        head_cfg, head_shapes, head_sets, head_ramp = 1, workloads.LLAMA2_7B_LAYER, 10, 200
        head_name = "Llama-2-7B decoder layer (q,k,v,o 4096x4096; gate,up 11008x4096; down 4096x11008)"
    else:
        head_cfg, head_shapes, head_sets, head_ramp = CONFIG_INDEX, workloads.LLAMA2_70B_LAYER, CODE_SETS, RAMP_UP
        head_name = ("Llama-2-70B decoder layer (q,o 8192x8192; k,v 1024x8192; gate,up 28672x8192; "
                     "down 8192x28672)")
    head = Layer(head_cfg, head_shapes, bits, head_sets, keep_host=not args.no_cpu)
    head.ramp_up(head_ramp)
    ms = _time_steps(torch, head.pot_step, args.steps, args.warmup)
    value = head.pot_bytes / (ms * 1e-3) / 1e9
    result = {
        "metric": "PoT dequant GB/s (algorithmic bytes: codes + scales in, fp16 out)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u16",
        "data": "synthetic",
        "config": {"workload": f"{head_name}, {bits}-bit PoT codes, group 128, stand-alone dequant of all "
                               "seven matrices",
                   "bits": bits, "group": G, "weights": head.weights, "launches_per_step": 1,
                   "entry_point": "pot_dequant_batch", "layout": "canonical",
                   "code_sets_rotated": head_sets, "untimed_ramp_up_launches": head_ramp},
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "roofline": {
            "kernel": f"potq::dequant_batch_kernel<{bits}, false>",
            "bound": "hbm",
            "achieved": round(value, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(value / HBM_PEAK_GBPS, 4),
            "bytes_per_launch": head.pot_bytes,
            "us_per_launch": round(ms * 1e3, 3),
            "traffic": PROFILED_TRAFFIC["bytes_per_launch"][bits] if args.workload == "70b" else None,
            "traffic_source": PROFILED_TRAFFIC["source"],
        },
    }

    if args.copy_calibration:
        # a kernel whose HBM traffic is known exactly: 256 MiB read + 256 MiB written per launch
        a = torch.empty(128 * 1024 * 1024, dtype=torch.float16, device=dev).normal_()
        b = torch.empty_like(a)
        for _ in range(10):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    # ---------------------------------------------------------------- CPU oracle on the host cores
    if not args.no_cpu:
        import oracle
        cores = len(os.sched_getaffinity(0))
        threads = min(cores, oracle.max_threads())
        passes = 0
        t0 = time.perf_counter()
        while passes < 64 and (passes == 0 or time.perf_counter() - t0 < 12.0):
            for codes_h, scales_h, K in head.host:
                oracle.pot_dequant(codes_h, scales_h, K, bits, G, nthreads=threads)
            passes += 1
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {
            "value": round(passes * head.pot_bytes / dt / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"{passes} full passes over the same seven matrices ({head.weights / 1e6:.1f} M weights each), "
                      "oracle/potq_oracle.c pot_dequant, OpenMP over rows",
            "seconds": round(dt, 2),
        }
    head.host = []

    if args.no_extras or args.workload != "70b":
        print(json.dumps(result))
        return 0

    # ---------------------------------------------------------------- extras
    extras = {}
    head.ramp_up()                       # the GPU idled during the CPU baseline: ramp up again, untimed

    # value-independence of the (branch-free) kernel: the same pass over all-zero codes
    zero_items = []
    zero_keep = []
    for _ in range(CODE_SETS):
        layer = [(torch.zeros_like(c), s) for (c, s, _, _) in head.sets[0]]
        zero_keep.append(layer)
        zero_items.append(binding.make_batch([(c, s, None, o, K, bits) for (c, s), o, (_, _, K)
                                              in zip(layer, head.outs, head.shapes)]))

    def zero_step():
        turn[0] += 1
        check(lib.pot_dequant_batch(zero_items[turn[0] % CODE_SETS], len(head.shapes), bits, G, stream))

    ms_rand, ms_zero = _time_pair(torch, head.pot_step, zero_step, 30, 5)
    extras["value_independence"] = {
        "random_codes_us": round(ms_rand * 1e3, 1), "all_zero_codes_us": round(ms_zero * 1e3, 1),
        "ratio": round(ms_zero / ms_rand, 4), "independent_within_3pct": bool(abs(ms_zero / ms_rand - 1.0) < 0.03)}
    del zero_items, zero_keep

    # ceilings of this machine: a plain device copy and a plain fill (torch kernels, 512 MiB buffers)
    ca = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
    cb = torch.empty_like(ca)
    ms_copy = _time_steps(torch, lambda: cb.copy_(ca), 20, 5)
    ms_fill = _time_steps(torch, lambda: cb.zero_(), 20, 5)
    extras["box_ceilings"] = {"device_copy_GBps": round(2 * ca.numel() / ms_copy / 1e6, 1),
                              "fill_GBps": round(ca.numel() / ms_fill / 1e6, 1),
                              "note": "torch copy_ / zero_ on 512 MiB: what plain streaming kernels reach here"}
    del ca, cb

    # the other code width on the same layer
    other = 5 - bits
    del head
    torch.cuda.empty_cache()
    lay = Layer(CONFIG_INDEX, workloads.LLAMA2_70B_LAYER, other, CODE_SETS)
    lay.ramp_up()
    ms_o = _time_steps(torch, lay.pot_step, args.steps, args.warmup)
    extras[f"pot_dequant_70b_layer_{other}bit"] = dict(_hbm(lay.pot_bytes, ms_o * 1e3), kernel=f"dequant_batch_kernel<{other}, false>")
    del lay
    torch.cuda.empty_cache()

    # Llama-2-7B layer, 2 bits, with the uniform-INT baseline (ten rotating sets: 538 MB)
    l7 = Layer(1, workloads.LLAMA2_7B_LAYER, 2, 10, with_int=True)
    l7.ramp_up(200)
    ms_p7, ms_i7 = _time_pair(torch, l7.pot_step, l7.int_step, 200, 20)
    extras["pot_dequant_7b_layer_2bit"] = dict(_hbm(l7.pot_bytes, ms_p7 * 1e3), int_us=round(ms_i7 * 1e3, 2),
                                                int_GBps=round(l7.int_bytes / ms_i7 / 1e6, 1),
                                                pot_speedup_vs_int=round(ms_i7 / ms_p7, 4),
                                                note="PoT and INT measured alternately, five times each, medians")
    one = l7.pot_items[0]
    ms_res = _time_steps(torch, lambda: check(lib.pot_dequant_batch(one, 7, 2, G, stream)), 200, 20)
    extras["pot_dequant_7b_layer_2bit_cache_resident_codes"] = dict(
        _hbm(l7.pot_bytes, ms_res * 1e3),
        note="one set of code buffers re-read every step: the 53.8 MB of codes and scales come from the 256 MB "
             "last-level cache, only the writes reach HBM")
    del l7, one
    torch.cuda.empty_cache()

    # single 4096 x 4096 matrix, 3 bits (pot_dequant): rotating through 27 buffer sets (1.08 GB), and re-using one
    N1 = K1 = 4096
    nb1 = workloads.algorithmic_bytes_dequant(N1, K1, 3, G)
    c1, s1 = (to_dev(a) for a in workloads.pot_matrix(0, 0, N1, K1, 3, G))
    sets1 = [(c1, s1, torch.empty((N1, K1), dtype=torch.float16, device=dev))]
    for _ in range(26):
        sets1.append((random_codes(N1, K1, 3), permuted(s1), torch.empty((N1, K1), dtype=torch.float16, device=dev)))
    calls1 = [(c.data_ptr(), s.data_ptr(), o.data_ptr(), N1, K1, 3, G, stream) for c, s, o in sets1]

    def single_rot():
        for c in calls1:
            check(lib.pot_dequant(*c))

    def single_res():
        check(lib.pot_dequant(*calls1[0]))

    single_rot()
    us_rot = _time_steps(torch, single_rot, 10, 3) * 1e3 / len(calls1)
    us_res = _time_steps(torch, single_res, 200, 20) * 1e3
    extras["pot_dequant_4096x4096_3bit"] = dict(_hbm(nb1, us_rot), buffers_rotated=len(calls1),
                                                 cache_resident=dict(_hbm(nb1, us_res),
                                                                     note="one 40 MB buffer set re-used: inputs and "
                                                                          "outputs stay in the 256 MB last-level cache"))
    del sets1, calls1, c1, s1
    torch.cuda.empty_cache()

    def rotate(nbytes_per_set):
        return max(2, min(64, (1 << 30) // max(1, nbytes_per_set) + 1))

    def gemv_pairs(shapes, bb, seed_cfg):
        """PoT and INT GEMV per shape, measured alternately, weight buffers rotating through HBM."""
        rows_ = []
        for j, (N, K) in enumerate(shapes):
            nbytes = workloads.algorithmic_bytes_gemm(1, N, K, bb, G)
            R = rotate(nbytes)
            cs = [random_codes(N, K, bb) for _ in range(R)]
            sc_ = to_dev(workloads.pot_scales(workloads.seed_of(seed_cfg, j, 1), N, K, G))
            S_h, Z_h = workloads.int_scales_zeros(workloads.seed_of(seed_cfg, j, 3), N, K, bb, G)
            Sd_, Zd_ = to_dev(S_h), to_dev(Z_h)
            x = to_dev(workloads.activations(workloads.seed_of(seed_cfg, j, 2), 1, K)[0])
            y = torch.empty((N,), dtype=torch.float16, device=dev)
            pc = [(c.data_ptr(), sc_.data_ptr(), x.data_ptr(), y.data_ptr(), N, K, bb, G, 1, stream) for c in cs]
            ic = [(c.data_ptr(), Sd_.data_ptr(), Zd_.data_ptr(), x.data_ptr(), y.data_ptr(), N, K, bb, G, 1, stream)
                  for c in cs]

            def pot_rot():
                for c in pc:
                    check(lib.pot_gemv(*c))

            def int_rot():
                for c in ic:
                    check(lib.int_gemv(*c))

            reps = max(2, 128 // R)
            us_p, us_i = (t * 1e3 / R for t in _time_pair(torch, pot_rot, int_rot, reps, 2))
            rows_.append(dict(_hbm(nbytes, us_p), shape=f"{N}x{K}", bits=bb, TFLOPs=round(2.0 * N * K / us_p / 1e6, 2),
                              int_us=round(us_i, 2), pot_speedup_vs_int=round(us_i / us_p, 3), buffers_rotated=R,
                              exponent_form=bool(potq.potq_gemv_exponent_form(N, K, bb))))
            del cs, pc, ic
            torch.cuda.empty_cache()
        return rows_

    b3 = 3
    shapes7 = [(N, K) for _, N, K in workloads.GEMV_7B_SHAPES]
    shapes70 = [(8192, 8192), (1024, 8192), (28672, 8192), (8192, 28672)]
    extras["pot_gemv_7b_shapes"] = gemv_pairs(shapes7, 3, 2) + gemv_pairs(shapes7, 2, 2)
    extras["pot_gemv_70b_shapes"] = gemv_pairs(shapes70, 3, 3) + gemv_pairs(shapes70, 2, 3)
    # the vocabulary projection of a decoder (32000 or 128256 rows): the largest matrix of a decode step
    extras["pot_gemv_3bit_vocabulary_projection"] = gemv_pairs(((32000, 4096), (128256, 4096), (128256, 8192)), 3, 3)

    # the same product on the canonical layout (the boundary's own format, no repack) next to the tiled one
    canon = []
    for (N, K) in ((11008, 4096), (28672, 8192), (8192, 28672)):
        nbytes = workloads.algorithmic_bytes_gemm(1, N, K, b3, G)
        R = rotate(nbytes)
        cs = [random_codes(N, K, b3) for _ in range(R)]
        sc_ = to_dev(workloads.pot_scales(workloads.seed_of(3, 0, 1), N, K, G))
        x = to_dev(workloads.activations(workloads.seed_of(3, 0, 2), 1, K)[0])
        y = torch.empty((N,), dtype=torch.float16, device=dev)
        calls = {lay: [(c.data_ptr(), sc_.data_ptr(), x.data_ptr(), y.data_ptr(), N, K, b3, G, lay, stream) for c in cs]
                 for lay in (binding.LAYOUT_CANONICAL, binding.LAYOUT_TILE16)}

        def canon_rot():
            for c in calls[binding.LAYOUT_CANONICAL]:
                check(lib.pot_gemv(*c))

        def tiled_rot():
            for c in calls[binding.LAYOUT_TILE16]:
                check(lib.pot_gemv(*c))

        reps = max(2, 128 // R)
        us_c, us_t = (t * 1e3 / R for t in _time_pair(torch, canon_rot, tiled_rot, reps, 2))
        canon.append(dict(_hbm(nbytes, us_c), shape=f"{N}x{K}", bits=b3, layout="canonical",
                          tiled_us=round(us_t, 2), buffers_rotated=R))
        del cs, calls
        torch.cuda.empty_cache()
    extras["pot_gemv_3bit_canonical_layout"] = canon

    # shared-activation batches: q/k/v (3 x 4096x4096) and gate/up (2 x 11008x4096) in one launch each
    shared = []
    for label, (N, K), copies in (("qkv 3x4096x4096", (4096, 4096), 3), ("gate_up 2x11008x4096", (11008, 4096), 2)):
        nbytes = copies * workloads.algorithmic_bytes_gemm(1, N, K, b3, G)
        R = rotate(nbytes)
        scales_h = workloads.pot_scales(workloads.seed_of(2, 7, 1), N, K, G)
        x = to_dev(workloads.activations(workloads.seed_of(2, 7, 2), 1, K)[0])
        keep, batches, singles = [], [], []
        for r in range(R):
            ms_ = [(random_codes(N, K, b3), to_dev(scales_h), None,
                    torch.empty((N,), dtype=torch.float16, device=dev)) for _ in range(copies)]
            keep.append(ms_)
            batches.append(binding.make_gemv_batch(ms_, K, b3))
            singles.append([(m_[0].data_ptr(), m_[1].data_ptr(), x.data_ptr(), m_[3].data_ptr(), N, K, b3, G, 1,
                             stream) for m_ in ms_])

        def batch_rot():
            for arr in batches:
                check(lib.pot_gemv_batch(arr, copies, x.data_ptr(), K, b3, G, 1, stream))

        def single_rot2():
            for calls in singles:
                for c in calls:
                    check(lib.pot_gemv(*c))

        reps = max(2, 128 // R)
        us_b, us_s = (t * 1e3 / R for t in _time_pair(torch, batch_rot, single_rot2, reps, 2))
        shared.append(dict(_hbm(nbytes, us_b), batch=label, us_separate_launches=round(us_s, 2), buffers_rotated=R))
        del keep, batches, singles
    extras["pot_gemv_batch_3bit_shared_activation"] = shared
    torch.cuda.empty_cache()

    # the seven projections of one decoder layer at batch 1 as a decoder issues them: q/k/v in one launch,
    # o, gate/up in one launch, down (four launches), rotating through enough layers' worth of weights to
    # exceed the last-level cache; random bytes are valid codes, the activations are unrelated vectors
    def decoder_layer_batch1(hidden, kv_rows, ffn, layers):
        shapes = [(hidden, hidden), (kv_rows, hidden), (kv_rows, hidden), (hidden, hidden),
                  (ffn, hidden), (ffn, hidden), (hidden, ffn)]
        layer_bytes = sum(workloads.algorithmic_bytes_gemm(1, N, K, b3, G) for N, K in shapes)
        xh = to_dev(workloads.activations(workloads.seed_of(2, 8, 2), 1, hidden)[0])
        xf = to_dev(workloads.activations(workloads.seed_of(2, 9, 2), 1, ffn)[0])
        keep, steps_ = [], []
        for _ in range(layers):
            def mat(N, K):
                sc_ = to_dev(workloads.pot_scales(workloads.seed_of(2, 8, 1), N, K, G))
                return (random_codes(N, K, b3), sc_, None, torch.empty((N,), dtype=torch.float16, device=dev))
            qkv = [mat(hidden, hidden), mat(kv_rows, hidden), mat(kv_rows, hidden)]
            o = mat(hidden, hidden)
            gu = [mat(ffn, hidden) for _ in range(2)]
            dn = mat(hidden, ffn)
            keep.append((qkv, o, gu, dn))
            steps_.append((binding.make_gemv_batch(qkv, hidden, b3), binding.make_gemv_batch(gu, hidden, b3),
                           (o[0].data_ptr(), o[1].data_ptr(), xh.data_ptr(), o[3].data_ptr(), hidden, hidden, b3, G,
                            1, stream),
                           (dn[0].data_ptr(), dn[1].data_ptr(), xf.data_ptr(), dn[3].data_ptr(), hidden, ffn, b3, G,
                            1, stream)))

        def layer_rot():
            for b_qkv, b_gu, c_o, c_dn in steps_:
                check(lib.pot_gemv_batch(b_qkv, 3, xh.data_ptr(), hidden, b3, G, 1, stream))
                check(lib.pot_gemv(*c_o))
                check(lib.pot_gemv_batch(b_gu, 2, xh.data_ptr(), hidden, b3, G, 1, stream))
                check(lib.pot_gemv(*c_dn))

        us_layer = _time_steps(torch, layer_rot, max(2, 128 // layers), 2) * 1e3 / layers
        # the same launches recorded once into a HIP graph and replayed (the stream passed to the library
        # inside the capture is the capturing one): what a decoder that replays its step would see
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            cs = torch.cuda.current_stream().cuda_stream
            for b_qkv, b_gu, c_o, c_dn in steps_:
                check(lib.pot_gemv_batch(b_qkv, 3, xh.data_ptr(), hidden, b3, G, 1, cs))
                check(lib.pot_gemv(*c_o[:-1], cs))
                check(lib.pot_gemv_batch(b_gu, 2, xh.data_ptr(), hidden, b3, G, 1, cs))
                check(lib.pot_gemv(*c_dn[:-1], cs))
        us_graph = _time_steps(torch, graph.replay, max(2, 128 // layers), 2) * 1e3 / layers
        del graph, keep, steps_
        torch.cuda.empty_cache()
        return dict(_hbm(layer_bytes, us_layer), launches_per_layer=4, layers_rotated=layers,
                    hip_graph_replay=_hbm(layer_bytes, us_graph))

    extras["pot_gemv_3bit_7b_decoder_layer_batch1"] = decoder_layer_batch1(4096, 4096, 11008, 16)
    extras["pot_gemv_3bit_70b_decoder_layer_batch1"] = decoder_layer_batch1(8192, 1024, 28672, 3)

    # fused MFMA GEMM, 3-bit, 13B shapes; the calls rotate through enough copies of the weight codes
    # (random bytes are valid codes) that they are read from HBM, not from the 256 MB last-level cache
    gemm = []
    for i, (name, N, K) in enumerate(workloads.GEMM_13B_SHAPES):
        codes_h, scales_h = workloads.pot_matrix(4, i, N, K, b3, G)
        S_h, Z_h = workloads.int_scales_zeros(workloads.seed_of(4, i, 3), N, K, b3, G)
        tiled = [potq.potq_repack(to_dev(codes_h), K, b3)]
        R = max(2, int(640e6 // tiled[0].numel()) + 1)
        for _ in range(1, R):
            tiled.append(torch.randint(0, 256, tiled[0].shape, dtype=torch.uint8, device=dev, generator=gen))
        sc, Sd, Zd = to_dev(scales_h), to_dev(S_h), to_dev(Z_h)
        # context: the vendor library's fp16 GEMM (torch.matmul) on the same weights already de-quantised to
        # fp16 (what Sec. 1 describes: de-quantise, then GEMM), three rotating copies so that they come from HBM
        W16 = [potq.pot_dequant(to_dev(codes_h), sc, K, b3, G)]
        W16 += [W16[0].clone() for _ in range(2)]
        for M in workloads.GEMM_TOKENS:
            X = to_dev(workloads.activations(workloads.seed_of(4, i, 2) + M, M, K))
            Y = torch.empty((M, N), dtype=torch.float16, device=dev)
            ws = potq.gemm_workspace(M, N, K, b3)
            wp, wn = (ws.data_ptr(), ws.numel()) if ws is not None else (None, 0)
            pas = [(t.data_ptr(), sc.data_ptr(), X.data_ptr(), Y.data_ptr(), M, N, K, b3, G, 1, wp, wn, stream)
                   for t in tiled]
            ias = [(t.data_ptr(), Sd.data_ptr(), Zd.data_ptr(), X.data_ptr(), Y.data_ptr(), M, N, K, b3, G, 1,
                    wp, wn, stream) for t in tiled]

            def pot_rot():
                turn[0] += 1
                check(lib.pot_gemm(*pas[turn[0] % R]))

            def int_rot():
                turn[0] += 1
                check(lib.int_gemm(*ias[turn[0] % R]))

            us_p, us_i = (t * 1e3 for t in _time_pair(torch, pot_rot, int_rot, 2 * R, 3))

            def lib_rot():
                turn[0] += 1
                torch.matmul(X, W16[turn[0] % 3].t(), out=Y)

            us_lib = _time_steps(torch, lib_rot, 30, 5) * 1e3
            gemm.append(dict(_gemm_roof(M, N, K, workloads.algorithmic_bytes_gemm(M, N, K, b3, G), us_p),
                             shape=f"{N}x{K}", M=M, int_us=round(us_i, 2), pot_speedup_vs_int=round(us_i / us_p, 3),
                             buffers_rotated=R, torch_fp16_matmul_on_dequantised_weights_us=round(us_lib, 2)))
        del tiled, W16
        torch.cuda.empty_cache()
    extras["pot_gemm_3bit_13b_shapes"] = gemm
    del sc, Sd, Zd
    torch.cuda.empty_cache()

    # the same kernel family at prefill size (2048 tokens), 13B and 70B projection shapes: bound by the
    # matrix cores, so one set of weights is enough; the vendor fp16 GEMM on de-quantised weights beside it
    prefill = []
    M = 2048
    for i, (N, K) in enumerate([(13824, 5120), (5120, 13824), (8192, 8192), (28672, 8192), (8192, 28672)]):
        codes_h, scales_h = workloads.pot_matrix(5, i, N, K, b3, G)
        sc = to_dev(scales_h)
        tiled = potq.potq_repack(to_dev(codes_h), K, b3)
        W16 = potq.pot_dequant(to_dev(codes_h), sc, K, b3, G)
        X = to_dev(workloads.activations(workloads.seed_of(5, i, 2), M, K))
        Y = torch.empty((M, N), dtype=torch.float16, device=dev)
        ws = potq.gemm_workspace(M, N, K, b3)
        wp, wn = (ws.data_ptr(), ws.numel()) if ws is not None else (None, 0)
        pa = (tiled.data_ptr(), sc.data_ptr(), X.data_ptr(), Y.data_ptr(), M, N, K, b3, G, 1, wp, wn, stream)
        us_p = _time_steps(torch, lambda: check(lib.pot_gemm(*pa)), 10, 3) * 1e3
        us_lib = _time_steps(torch, lambda: torch.matmul(X, W16.t(), out=Y), 10, 3) * 1e3
        prefill.append(dict(_gemm_roof(M, N, K, workloads.algorithmic_bytes_gemm(M, N, K, b3, G), us_p),
                            shape=f"{N}x{K}", M=M, torch_fp16_matmul_on_dequantised_weights_us=round(us_lib, 2)))
        del tiled, W16, X, Y, ws
        torch.cuda.empty_cache()
    extras["pot_gemm_3bit_2048_tokens"] = prefill

    # Step 1 scale search (Algorithm 1) on one 4096x4096 fp16 matrix, 3-bit, group 128: plain vector-ALU
    # work, about eight lane operations per weight and multiplier (200 multipliers)
    Wq = to_dev(workloads.weights_f16(workloads.seed_of(0, 0, 4), 4096, 4096))
    qc = torch.empty((4096, 4096 * b3 // 8), dtype=torch.uint8, device=dev)
    qs = torch.empty((4096, 4096 // G), dtype=torch.float16, device=dev)
    qa = (Wq.data_ptr(), qc.data_ptr(), qs.data_ptr(), 4096, 4096, b3, G, stream)
    ms_q = _time_steps(torch, lambda: check(lib.pot_quantize(*qa)), 10, 2)
    lane_ops = 4096.0 * 4096 * 200 * 8
    extras["pot_quantize_3bit_4096x4096"] = {
        "ms": round(ms_q, 4), "Mweights_per_s": round(4096 * 4096 / ms_q / 1e3, 1),
        "bound": "alu", "T_lane_ops_per_s": round(lane_ops / ms_q / 1e9, 2),
        "frac": round(lane_ops / ms_q / 1e9 / 39.3, 4), "peak_T_lane_ops_per_s": 39.3}
    # Step 2 weight path (Sec. 3.3) on one 7B MLP matrix: streaming kernels, 4 bytes per weight each way
    fN, fK = 11008, 4096
    fW = to_dev(workloads.weights_f16(workloads.seed_of(0, 1, 4), fN, fK))
    fS = to_dev(workloads.pot_scales(workloads.seed_of(0, 1, 1), fN, fK, G))
    fG = torch.zeros((fN, fK // G), dtype=torch.float32, device=dev)
    fdG = torch.empty_like(fG)
    fD = to_dev(workloads.weights_f16(workloads.seed_of(0, 1, 5), fN, fK))
    fO = torch.empty_like(fW)
    fa = (fW.data_ptr(), fS.data_ptr(), fG.data_ptr(), fO.data_ptr(), fN, fK, b3, G, stream)
    ba = (fW.data_ptr(), fS.data_ptr(), fG.data_ptr(), fD.data_ptr(), fdG.data_ptr(), fN, fK, b3, G, stream)
    ms_f = _time_steps(torch, lambda: check(lib.pot_fakequant_forward(*fa)), 50, 5)
    ms_b = _time_steps(torch, lambda: check(lib.pot_fakequant_backward(*ba)), 50, 5)
    fbytes = fN * fK * 4 + fN * (fK // G) * 6
    extras["pot_fakequant_3bit_11008x4096"] = {
        "forward": _hbm(fbytes, ms_f * 1e3), "backward": _hbm(fbytes + fN * (fK // G) * 4, ms_b * 1e3),
        "note": "single buffer set (180 MB per pass: partly served by the 256 MB last-level cache)"}
    result["extras"] = extras

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
