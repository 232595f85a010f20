#!/usr/bin/env python3
"""Benchmark of the DCT hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input:
  dct_select_threshold + dct_threshold_compact (exactly-k) on the c4 gradient
  (embedding-shaped, N = 2^28 fp32, keep 0.5 %), then
  dct_rowtopk_fwd + dct_rowtopk_bwd on the c5 activations
  (65536 x 4096 bf16, k = 204).
Inputs are resident in HBM before the timed region; two copies of every input
alternate so that no step re-reads what the previous one left in cache.

Prints ONE JSON line: whole-step throughput in elements/s; per-call times, elements/s and
HBM fractions for all five configurations (c1 and c2 are a few MB and run out of cache: latency,
not bandwidth; c3 is the reuse loop, the threshold selected once and applied to 1000 fresh draws);
the roofline entry of the dominant kernel; the calls of the further rows (error feedback,
decompression, other encodings, many tensors per call; none is part of the step); and the CPU
oracle timed on the same step's input, on one thread and spread over the host's cores.
The last lines on stderr repeat the figures that matter in short form.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import synth_inputs as si  # noqa: E402

HBM_PEAK_GBPS = 8000.0

# kernels behind each timed call (names as rocprofv3 prints them) and launches per call
CALL_KERNELS = {
    "dct_select_threshold[c4]": [("dct::select_sample_kernel<0, false>", 1),
                                 ("dct::select_partition_kernel<0, false, 8>", 1),
                                 ("dct::select_tail_kernel<0, false>", 1)],
    "dct_threshold_compact[c4,exact_k]": [("dct::compact_kernel<0, true, false, true>", 1)],
    "dct_rowtopk_fwd[c5]": [("dct::fast::rowtopk_fwd_onchip_kernel<8, 0, false, 16>", 1)],
    "dct_rowtopk_bwd[c5]": [("dct::rowtopk_bwd_rows_kernel<unsigned short, int>", 1)],
    "dct_ef_select_threshold[c4]": [("dct::select_sample_kernel<0, true>", 1),
                                    ("dct::select_partition_kernel<0, true, 8>", 1),
                                    ("dct::select_tail_kernel<0, true>", 1)],
    "dct_ef_threshold_compact[c4,ge_tau]": [("dct::compact_kernel<0, false, true, false>", 1)],
    "dct_scatter[c4,assign]": [("dct::scatter_assign_kernel<unsigned int>", 1)],
    "dct_scatter[c4,add]": [("dct::scatter_add4_kernel", 1)],
    "dct_rowtopk_scatter[c5]": [("dct::rowscatter_lds_kernel<unsigned short, int>", 1)],
    "dct_rowtopk_fwd_bitmask[c5]": [("dct::fast::rowtopk_fwd_onchip_kernel<8, 1, false, 16>", 1)],
    "dct_rowtopk_bwd_bitmask[c5]": [("dct::rowtopk_bwd_rows_bitmask_kernel<unsigned short>", 1)],
    "dct_rowtopk_scatter_bitmask[c5]": [("dct::rowtopk_bitmask_lanes_kernel<unsigned short, false>", 1)],
    "dct_rowtopk_fwd_idx16[c5]": [("dct::fast::rowtopk_fwd_onchip_kernel<8, 2, false, 16>", 1)],
    "dct_rowtopk_bwd_idx16[c5]": [("dct::rowtopk_bwd_rows_kernel<unsigned short, unsigned short>", 1)],
    "dct_rowtopk_scatter_idx16[c5]": [("dct::rowscatter_lds_kernel<unsigned short, unsigned short>", 1)],
}


TRAFFIC_FILE = os.path.join("profiles", "hbm_traffic_per_launch.txt")


def traffic_table():
    """{kernel name: HBM bytes per launch} from the committed rocprofv3 counter summary, and where it came from."""
    path = os.path.join(ROOT, TRAFFIC_FILE)
    table = {}
    with open(path) as f:
        text = f.read()
    for line in text.splitlines():
        if line.startswith("#") or not line.strip():
            continue
        name, fb, wb = line.split("\t")
        table[name] = float(fb) + float(wb)
    return table, f"{TRAFFIC_FILE}#sha1:{hashlib.sha1(text.encode()).hexdigest()[:12]}"


def measured_traffic(call, table):
    """HBM bytes per call: scaled FETCH_SIZE + WRITE_SIZE of its kernels.  A kernel the summary does not know
    (renamed since the counters were collected) is an error, not a silent null."""
    missing = [k for k, _ in CALL_KERNELS[call] if k not in table]
    if missing:
        sys.exit(f"bench.py: {TRAFFIC_FILE} has no entry for {missing} (call {call}): collect the counters again "
                 f"(rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this benchmark) and refresh the summary")
    return int(sum(table[k] * n for k, n in CALL_KERNELS[call]))


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_calls(fn, reps, warmup=2, per_call=False):
    """Average duration in microseconds of fn(i) over `reps` back-to-back calls: two HIP events around the
    whole region, on the stream the kernels are launched on (torch's current stream).  per_call=True brackets
    every call with events instead and returns the median interval (each event adds about 2.5 us)."""
    for i in range(warmup):
        fn(i)
    if per_call:
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        torch.cuda.synchronize()
        ev[0].record()
        for i in range(reps):
            fn(i)
            ev[i + 1].record()
        torch.cuda.synchronize()
        return float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(reps)])) * 1e3
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(reps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--reps", type=int, default=30, help="launches per kernel for the per-call timings")
    ap.add_argument("--c3-draws", type=int, default=1000, help="distinct resident draws for the c3 reuse loop")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-batched", action="store_true",
                    help="skip the small-tensor comparison (its per-tensor calls launch the same kernels as the "
                         "large configurations, which blurs per-kernel profiles)")
    ap.add_argument("--small", action="store_true", help="shrink c4/c5 by 16x (debugging only, not a valid number)")
    ap.add_argument("--no-small-configs", action="store_true",
                    help="skip c1 and c2 (they launch the same kernels as the large configurations, which blurs "
                         "per-kernel profiles)")
    ap.add_argument("--no-traffic", action="store_true",
                    help="leave roofline.traffic null instead of looking it up in profiles/ (for the rocprofv3 runs "
                         "that collect the counters the lookup is made from)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (every box has one); --gpus N with N > 1 is not supported. "
                 "Every worker runs this same path on its own data with no communication; value is the one GPU's throughput.")
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")

    import paper_2010_08899_amd as dct
    from paper_2010_08899_amd import bench_probes
    dct.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    shrink = 16 if args.small else 1

    # ------------------------------------------------------------ inputs (resident)
    t0 = time.time()
    c4_rows = si.C4_ROWS // shrink
    g4 = [None, None]
    g4[0], k4 = si.config_c4(dev, rows=c4_rows)
    g4[1] = si.embedding_gradient(c4_rows, si.C4_DIM, (c4_rows * 5) // 100, dev, si.BASE_SEED + 40)
    n4 = g4[0].numel()
    c5_b = si.C5_B // shrink
    x5 = [None, None]
    dy5 = [None, None]
    x5[0], dy5[0], k5 = si.config_c5(dev, b=c5_b)
    x5[1] = si.relu_activations(c5_b, si.C5_D, dev, si.BASE_SEED + 50, dtype=torch.bfloat16)
    dy5[1] = si.normal_matrix(c5_b, si.C5_D, dev, si.BASE_SEED + 51, dtype=torch.bfloat16)
    B5, D5 = x5[0].shape
    def checksum(t):
        """64-bit sum of the tensor's words (wraps): identifies the generated bytes."""
        w = t.reshape(-1).view(torch.int32 if t.element_size() == 4 else torch.int16)
        return int(w.sum(dtype=torch.int64).item()) & ((1 << 64) - 1)

    inputs = {"torch": torch.__version__, "base_seed": si.BASE_SEED,
              "checksums": {"c4_g": [checksum(g4[0]), checksum(g4[1])], "c5_x": [checksum(x5[0]), checksum(x5[1])],
                            "c5_dy": [checksum(dy5[0]), checksum(dy5[1])]},
              "c4_nonzero_rows": (c4_rows * 5) // 100}
    torch.cuda.synchronize()
    log(f"[bench] inputs resident in {time.time() - t0:.1f}s: c4 N={n4} k={k4}; c5 {B5}x{D5} bf16 k={k5}")

    thr = torch.zeros(4, dtype=torch.int32, device=dev)
    sel_ws = dct.new_select_workspace(g4[0])
    cmp_ws = dct.new_compact_workspace(g4[0])
    cap4 = k4
    idx4 = torch.zeros(cap4, dtype=torch.int32, device=dev)
    val4 = torch.zeros(cap4, dtype=torch.float32, device=dev)
    cnt4 = torch.zeros(1, dtype=torch.int64, device=dev)
    idx5 = torch.zeros(B5, k5, dtype=torch.int32, device=dev)
    val5 = torch.zeros(B5, k5, dtype=torch.bfloat16, device=dev)
    dval5 = torch.zeros(B5, k5, dtype=torch.bfloat16, device=dev)

    def call_select(i):
        dct.dct_select_threshold(g4[i & 1], k4, thr, sel_ws)

    def call_compact(i):
        dct.dct_threshold_compact(g4[i & 1], thr, dct.DCT_EXACT_K, idx4, val4, cnt4, cmp_ws)

    def call_fwd(i):
        dct.dct_rowtopk_fwd(x5[i & 1], k5, idx5, val5, None)

    def call_bwd(i):
        dct.dct_rowtopk_bwd(dy5[i & 1], idx5, dval5)

    def step(i):
        call_select(i)
        call_compact(i)
        call_fwd(i)
        call_bwd(i)

    # ------------------------------------------------------------ the timed steps
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    assert dct.read_count(cnt4, capacity=cap4) == k4
    elems_per_step = n4 + B5 * D5
    ms_per_step = elapsed * 1e3 / args.steps
    value = elems_per_step * args.steps / elapsed
    log(f"[bench] {args.steps} steps: {ms_per_step:.3f} ms/step, {value:.4g} elements/s")

    # ------------------------------------------------------------ per-call timings and rooflines
    def entry(name, us, alg_bytes, elems, launches=1, extra=None):
        gbps = alg_bytes / (us * 1e-6) / 1e9
        e = {"call": name, "us": round(us, 2), "elements_per_s": elems / (us * 1e-6), "algorithmic_bytes": alg_bytes,
             "GBps": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4), "launches": launches}
        if extra:
            e.update(extra)
        return e

    calls = []
    us = time_calls(call_select, args.reps)
    sel_launches = sum(n for _, n in CALL_KERNELS["dct_select_threshold[c4]"])
    calls.append(entry("dct_select_threshold[c4]", us, n4 * 4 + 16, n4, launches=sel_launches))
    call_select(0)
    us = time_calls(call_compact, args.reps)
    calls.append(entry("dct_threshold_compact[c4,exact_k]", us, n4 * 4 + k4 * 8 + 8, n4))
    us = time_calls(call_fwd, args.reps)
    calls.append(entry("dct_rowtopk_fwd[c5]", us, B5 * D5 * 2 + B5 * k5 * 6, B5 * D5))
    us = time_calls(call_bwd, args.reps)
    # touched-sector floor of the gather (128-byte lines and 64-byte sectors), from the indices themselves
    idx_h = idx5[: min(B5, 2048)].cpu().numpy().astype(np.int64)
    lines128 = np.mean([np.unique(r // 64).size for r in idx_h]) * 128
    sect64 = np.mean([np.unique(r // 32).size for r in idx_h]) * 64
    strict = B5 * k5 * (4 + 2 * 2)
    gran128 = int(B5 * lines128) + B5 * k5 * 6
    gran64 = int(B5 * sect64) + B5 * k5 * 6
    calls.append(entry("dct_rowtopk_bwd[c5]", us, gran128, B5 * D5, extra={
        "frac_of_hbm_peak_strict": round(strict / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes_strict": strict, "GBps_strict": round(strict / (us * 1e-6) / 1e9, 1),
        "algorithmic_bytes_64B_sectors": gran64, "GBps_64B_sectors": round(gran64 / (us * 1e-6) / 1e9, 1),
        "note": "frac_of_hbm_peak counts the 128-byte lines the gather touches (a 5 % gather of bf16 touches 96 % of them: "
                "the memory moves whole lines); frac_of_hbm_peak_strict counts B*k*(4+2e) bytes only"}))

    # ------------------------------------------------------------ the small configurations (parity cases; latency-bound)
    # c1 (4 MiB) and c2 (8 MiB) live in the caches and take a microsecond of memory traffic: what is measured
    # is launch latency.  Reported because the metric asks for every configuration's elements/s.
    small_calls = []
    if not args.small and not args.no_small_configs:
        g1, k1 = si.config_c1(dev)
        ws1s, ws1c = dct.new_select_workspace(g1), dct.new_compact_workspace(g1)
        thr1 = torch.zeros(4, dtype=torch.int32, device=dev)
        idx1 = torch.zeros(k1, dtype=torch.int32, device=dev)
        val1 = torch.zeros(k1, dtype=torch.float32, device=dev)
        us = time_calls(lambda i: dct.dct_select_threshold(g1, k1, thr1, ws1s), 200)
        small_calls.append(entry("dct_select_threshold[c1]", us, si.C1_N * 4 + 16, si.C1_N, launches=2))
        us = time_calls(lambda i: dct.dct_threshold_compact(g1, thr1, dct.DCT_EXACT_K, idx1, val1, cnt4, ws1c), 200)
        small_calls.append(entry("dct_threshold_compact[c1,exact_k]", us, si.C1_N * 4 + k1 * 8 + 8, si.C1_N))
        x2, dy2, k2 = si.config_c2(dev)
        idx2 = torch.zeros(si.C2_B, k2, dtype=torch.int32, device=dev)
        val2 = torch.zeros(si.C2_B, k2, dtype=torch.float32, device=dev)
        dval2 = torch.zeros_like(val2)
        us = time_calls(lambda i: dct.dct_rowtopk_fwd(x2, k2, idx2, val2, None), 200)
        small_calls.append(entry("dct_rowtopk_fwd[c2]", us, si.C2_B * si.C2_D * 4 + si.C2_B * k2 * 8, si.C2_B * si.C2_D))
        us = time_calls(lambda i: dct.dct_rowtopk_bwd(dy2, idx2, dval2), 200)
        small_calls.append(entry("dct_rowtopk_bwd[c2]", us, si.C2_B * k2 * 12, si.C2_B * si.C2_D,
                                 extra={"note": "strict bytes (idx, gathered values, output); the input sits in cache"}))
        for c in small_calls:
            c["note"] = (c.get("note", "") + " cache-resident input, repeated calls: launch latency, not HBM bandwidth").strip()
        del g1, x2, dy2
    call_select(0)

    # ------------------------------------------------------------ error feedback fused in (not part of the step)
    # Same c4 gradients plus a resident residual per copy; the new residual goes to a third buffer so
    # that every repetition sees the same sums.
    ef_calls = []
    e4 = [si.residual_vector(n4, dev, si.BASE_SEED + 60 + j) for j in range(2)]
    e4_out = torch.empty(n4, dtype=torch.float32, device=dev)
    cap4e = 2 * k4
    idx4e = torch.zeros(cap4e, dtype=torch.int32, device=dev)
    val4e = torch.zeros(cap4e, dtype=torch.float32, device=dev)
    us = time_calls(lambda i: dct.dct_ef_select_threshold(g4[i & 1], e4[i & 1], k4, thr, sel_ws), args.reps)
    ef_calls.append(entry("dct_ef_select_threshold[c4]", us, 2 * n4 * 4 + 16, n4, launches=sel_launches))
    dct.dct_ef_select_threshold(g4[0], e4[0], k4, thr, sel_ws)
    us = time_calls(lambda i: dct.dct_ef_threshold_compact(g4[0], e4[0], e4_out, thr, dct.DCT_GE_TAU, idx4e, val4e,
                                                           cnt4, cmp_ws), args.reps)
    c4e = dct.read_count(cnt4, capacity=cap4e)
    ef_calls.append(entry("dct_ef_threshold_compact[c4,ge_tau]", us, 3 * n4 * 4 + c4e * 12 + 8, n4,
                          extra={"survivors": c4e}))
    del e4, e4_out, idx4e, val4e
    call_select(0)

    # ------------------------------------------------------------ receiver side: decompression (not part of the step)
    # The messages of the step (c4 pairs with their device-side count, c5 row lists) put back into
    # dense tensors; two output buffers alternate.
    call_compact(0)
    rx_calls = []
    d4 = [torch.empty(n4, dtype=torch.float32, device=dev) for _ in range(2)]
    us = time_calls(lambda i: dct.dct_scatter(idx4, val4, cnt4, d4[i & 1]), args.reps)
    rx_calls.append(entry("dct_scatter[c4,assign]", us, n4 * 4 + k4 * 8 + 8, n4))
    d4[0].zero_()
    us = time_calls(lambda i: dct.dct_scatter(idx4, val4, cnt4, d4[0], dct.DCT_SCATTER_ADD), args.reps)
    rx_calls.append(entry("dct_scatter[c4,add]", us, k4 * 16 + 8, k4, extra={
        "note": "strict bytes (idx, val, read-modify-write of the touched floats); the touched sectors are larger"}))
    del d4
    d5 = [torch.empty(B5, D5, dtype=torch.bfloat16, device=dev) for _ in range(2)]
    call_fwd(0)
    us = time_calls(lambda i: dct.dct_rowtopk_scatter(idx5, val5, d5[i & 1]), args.reps)
    rx_calls.append(entry("dct_rowtopk_scatter[c5]", us, B5 * D5 * 2 + B5 * k5 * 6, B5 * D5))

    # ------------------------------------------------------------ the mask as a bitmap (not part of the step)
    bm_calls = []
    mask5 = torch.zeros(B5, D5 // 32, dtype=torch.int32, device=dev)
    us = time_calls(lambda i: dct.dct_rowtopk_fwd_bitmask(x5[i & 1], k5, mask5, val5, None), args.reps)
    bm_calls.append(entry("dct_rowtopk_fwd_bitmask[c5]", us, B5 * D5 * 2 + B5 * (D5 // 8 + k5 * 2), B5 * D5))
    us = time_calls(lambda i: dct.dct_rowtopk_bwd_bitmask(dy5[i & 1], mask5, dval5), args.reps)
    bm_calls.append(entry("dct_rowtopk_bwd_bitmask[c5]", us, int(B5 * lines128) + B5 * (D5 // 8 + k5 * 2), B5 * D5,
                          extra={"note": "algorithmic_bytes counts the 128-byte lines the gather touches"}))
    us = time_calls(lambda i: dct.dct_rowtopk_scatter_bitmask(mask5, val5, d5[i & 1]), args.reps)
    bm_calls.append(entry("dct_rowtopk_scatter_bitmask[c5]", us, B5 * D5 * 2 + B5 * (D5 // 8 + k5 * 2), B5 * D5))
    del mask5

    # ------------------------------------------------------------ the mask as 16-bit indices (not part of the step)
    i16_calls = []
    idx16 = torch.zeros(B5, k5, dtype=torch.int16, device=dev)
    us = time_calls(lambda i: dct.dct_rowtopk_fwd_idx16(x5[i & 1], k5, idx16, val5, None), args.reps)
    i16_calls.append(entry("dct_rowtopk_fwd_idx16[c5]", us, B5 * D5 * 2 + B5 * k5 * 4, B5 * D5))
    us = time_calls(lambda i: dct.dct_rowtopk_bwd_idx16(dy5[i & 1], idx16, dval5), args.reps)
    i16_calls.append(entry("dct_rowtopk_bwd_idx16[c5]", us, int(B5 * lines128) + B5 * k5 * 4, B5 * D5,
                           extra={"note": "algorithmic_bytes counts the 128-byte lines the gather touches"}))
    us = time_calls(lambda i: dct.dct_rowtopk_scatter_idx16(idx16, val5, d5[i & 1]), args.reps)
    i16_calls.append(entry("dct_rowtopk_scatter_idx16[c5]", us, B5 * D5 * 2 + B5 * k5 * 4, B5 * D5))
    del d5, idx16
    call_fwd(0)

    # ------------------------------------------------------------ the paper's own MP widths (not part of the step)
    # Sec. 3.1 / 3.2: DLRM MLP layers of 512 and 256 units, Transformer FFN of 1024: 512 MiB of bf16 rows each
    narrow = []
    if not args.no_batched:
        for Dn in (256, 512, 1024):
            Bn = max(1, ((512 << 20) // shrink) // (Dn * 2))
            kn = Dn // 20
            xn = [si.relu_activations(Bn, Dn, dev, si.BASE_SEED + 60 + j, dtype=torch.bfloat16) for j in range(2)]
            idxn = torch.zeros(Bn, kn, dtype=torch.int32, device=dev)
            valn = torch.zeros(Bn, kn, dtype=torch.bfloat16, device=dev)
            dvaln = torch.zeros_like(valn)
            outn = torch.empty_like(xn[0])
            uf = time_calls(lambda i: dct.dct_rowtopk_fwd(xn[i & 1], kn, idxn, valn, None), 30)
            ub = time_calls(lambda i: dct.dct_rowtopk_bwd(xn[i & 1], idxn, dvaln), 10)
            us_ = time_calls(lambda i: dct.dct_rowtopk_scatter(idxn, valn, outn), 10)
            fb = Bn * Dn * 2 + Bn * kn * 6
            # the same traffic and nothing else: four rows (one group of the narrow-row kernel) read by a wavefront,
            # their outputs' bytes written
            chunk = 4 * Dn * 2
            out_b = (4 * kn * 6 + 15) // 16 * 16
            snk = torch.zeros(16384, dtype=torch.uint8, device=dev)
            dstn = torch.empty((Bn // 4) * out_b + 16, dtype=torch.uint8, device=dev)
            ut = time_calls(lambda i: bench_probes.probe_rows(xn[i & 1].view(torch.uint8).reshape(-1), chunk, dstn, out_b, snk), 10)
            narrow.append({"B": Bn, "D": Dn, "k": kn, "dtype": "bf16", "fwd_us": round(uf, 1),
                           "fwd_frac_of_hbm_peak": round(fb / (uf * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                           "traffic_only_us": round(ut, 1), "fwd_frac_of_traffic_only": round(ut / uf, 4),
                           "bwd_us": round(ub, 1), "scatter_us": round(us_, 1)})
            log(f"[bench] MP {Bn}x{Dn} bf16 k={kn}: fwd {uf:.1f} us ({narrow[-1]['fwd_frac_of_hbm_peak'] * 100:.1f}% of peak, "
                f"traffic only {ut:.1f} us), bwd {ub:.1f} us, scatter {us_:.1f} us")
            del xn, idxn, valn, dvaln, outn, dstn

    # ------------------------------------------------------------ many small tensors per call (not part of the step)
    # 24 tensors from 64 to 2^20 elements (the largest is c1-sized), 1 % kept: one batched select +
    # one batched compaction against one pair of calls per tensor.
    batched = None
    bt_sizes = [] if args.no_batched else [1 << 20, 512 * 1024, 512 * 256, 256 * 64, 1024, 512, 256, 64] * 3
    if bt_sizes:
        bt_segs, off_b, out_b = [], 0, 0
        for n_b in bt_sizes:
            k_b = max(1, n_b // 100)
            bt_segs.append((off_b, n_b, k_b, out_b, 2 * k_b))
            off_b += n_b
            out_b += 2 * k_b
        gb = si.gaussian_gradient(off_b, dev, si.BASE_SEED + 70)
        bt_table = dct.segment_table(bt_segs)
        bt_ws = dct.new_batched_workspace(gb, bt_table)
        bt_thr = torch.zeros(len(bt_segs), 4, dtype=torch.int32, device=dev)
        bt_idx = torch.zeros(out_b, dtype=torch.int32, device=dev)
        bt_val = torch.zeros(out_b, dtype=torch.float32, device=dev)
        bt_cnt = torch.zeros(len(bt_segs), dtype=torch.int64, device=dev)
        one_sws = dct.new_select_workspace(gb[: bt_sizes[0]])
        one_cws = dct.new_compact_workspace(gb[: bt_sizes[0]])
        one_cnt = torch.zeros(1, dtype=torch.int64, device=dev)

        def batched_pair(i):
            dct.dct_select_threshold_batched(gb, bt_table, bt_thr, bt_ws)
            dct.dct_threshold_compact_batched(gb, bt_table, bt_thr, dct.DCT_GE_TAU, bt_idx, bt_val, bt_cnt, bt_ws)

        def per_tensor_pairs(i):
            for (o, n_b, k_b, oo, cap_b) in bt_segs:
                dct.dct_select_threshold(gb[o:o + n_b], k_b, thr, one_sws)
                dct.dct_threshold_compact(gb[o:o + n_b], thr, dct.DCT_GE_TAU, bt_idx[oo:oo + cap_b],
                                          bt_val[oo:oo + cap_b], one_cnt, one_cws)

        us_bt = time_calls(batched_pair, 10)
        us_pt = time_calls(per_tensor_pairs, 10)
        batched = {"tensors": len(bt_segs), "elements": off_b, "kept_fraction": 0.01,
                   "batched_select_plus_compact_us": round(us_bt, 1), "one_call_pair_per_tensor_us": round(us_pt, 1),
                   "elements_per_s_batched": off_b / (us_bt * 1e-6)}
        log(f"[bench] batched: {batched}")
    call_select(0)

    # plain streaming kernels: the achievable HBM rate measured in the same run
    probe_bytes = (4 << 30) // shrink
    probe_src = torch.empty(probe_bytes, dtype=torch.uint8, device=dev).random_(0, 255)
    probe_dst = torch.empty(probe_bytes // 2, dtype=torch.uint8, device=dev)
    sink = torch.zeros(16384, dtype=torch.uint8, device=dev)
    us_read = time_calls(lambda i: bench_probes.probe_read(probe_src, sink), 10)
    us_copy = time_calls(lambda i: bench_probes.probe_copy(probe_dst, probe_src[: probe_bytes // 2]), 10)
    probes = {"read_GBps": round(probe_bytes / (us_read * 1e-6) / 1e9, 1),
              "copy_GBps": round(probe_bytes / (us_copy * 1e-6) / 1e9, 1)}
    # the traffic of the forward row kernel with none of its work: 8 KiB rows read by one wavefront each (the next
    # row in flight), k (index, value) pairs' worth of bytes written per row.  Even a few per cent of writes mixed
    # into a read stream cost this chip far more than their bytes (see the rows_* figures against read_GBps).
    rows5 = (512 << 20) // shrink // 8192
    out5 = (k5 * 6 + 15) // 16 * 16
    row_src = probe_src[: rows5 * 8192]
    us_rows0 = time_calls(lambda i: bench_probes.probe_rows(row_src, 8192, probe_dst, 0, sink), 10)
    us_rows = time_calls(lambda i: bench_probes.probe_rows(row_src, 8192, probe_dst, out5, sink), 10)
    probes["rows_c5_read_only_us"] = round(us_rows0, 2)
    probes["rows_c5_read_write_us"] = round(us_rows, 2)
    probes["rows_c5_write_bytes_per_row"] = out5
    del probe_src, probe_dst, row_src
    for c in calls + ef_calls + rx_calls + bm_calls:
        c["frac_of_probe_read"] = round(c["GBps"] / probes["read_GBps"], 4)
        log(f"[bench] {c['call']}: {c['us']} us, {c['GBps']} GB/s = {c['frac_of_hbm_peak']:.1%} of 8 TB/s")
    log(f"[bench] probes: {probes}")

    # ------------------------------------------------------------ c3: select once, reuse on fresh draws
    c3 = None
    free_b, _ = torch.cuda.mem_get_info()
    n3 = si.C3_N // shrink
    draws = max(3, min(args.c3_draws, int(free_b * 0.8) // (n3 * 4) - 2))
    try:
        t0 = time.time()
        bank = torch.empty(draws, n3, dtype=torch.float32, device=dev)
        for j in range(draws):
            bank[j] = si.config_c3_draw(dev, j + 1, n3)
        g0 = si.config_c3_draw(dev, 0, n3)
        k3 = si.ceil_frac(n3, 1, 1000)
        cap3 = 2 * k3
        thr3 = torch.zeros(4, dtype=torch.int32, device=dev)
        ws3s = dct.new_select_workspace(g0)
        ws3 = dct.new_compact_workspace(g0)
        idx3 = torch.zeros(cap3, dtype=torch.int32, device=dev)
        val3 = torch.zeros(cap3, dtype=torch.float32, device=dev)
        cnt3 = torch.zeros(1, dtype=torch.int64, device=dev)
        torch.cuda.synchronize()
        log(f"[bench] c3: {draws} draws resident in {time.time() - t0:.1f}s")
        # the selection runs once per threshold life-span; timed over distinct draws as well
        us_sel3 = time_calls(lambda i: dct.dct_select_threshold(bank[i % draws], k3, thr3, ws3s), 50)
        dct.dct_select_threshold(g0, k3, thr3, ws3s)
        iters = si.C3_DRAWS
        # the loop as a training run issues it: iterations back to back, two events around all of them
        us_c3 = time_calls(lambda i: dct.dct_threshold_compact(bank[i % draws], thr3, dct.DCT_GE_TAU, idx3, val3,
                                                               cnt3, ws3), iters, warmup=5)
        last = dct.read_count(cnt3, capacity=cap3)
        us_c3_events = time_calls(lambda i: dct.dct_threshold_compact(bank[i % draws], thr3, dct.DCT_GE_TAU, idx3,
                                                                      val3, cnt3, ws3), min(iters, 200), warmup=5, per_call=True)
        alg3 = n3 * 4 + k3 * 8 + 8
        calls.append(entry("dct_select_threshold[c3]", us_sel3, n3 * 4 + 16, n3, launches=sel_launches))
        calls.append(entry("dct_threshold_compact[c3,ge_tau,reuse]", us_c3, alg3, n3, extra={
            "note": f"per iteration of {iters} back-to-back calls over {draws} distinct resident draws"}))
        c3 = {"n": n3, "k": k3, "distinct_draws": draws, "iterations": iters, "select_us": round(us_sel3, 2),
              "compact_us_per_iteration": round(us_c3, 2),
              "compact_us_median_with_an_event_per_call": round(us_c3_events, 2),
              "elements_per_s": n3 / (us_c3 * 1e-6),
              "GBps": round(alg3 / (us_c3 * 1e-6) / 1e9, 1),
              "frac_of_hbm_peak": round(alg3 / (us_c3 * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
              "amortised_us_per_iteration_L1000": round(us_c3 + us_sel3 / 1000.0, 2), "last_count": last}
        log(f"[bench] c3 reuse: {c3}")
        del bank
    except torch.cuda.OutOfMemoryError:
        log("[bench] c3 reuse loop skipped: not enough free HBM")

    # The dominant KERNEL of the step: among the step's calls that are one launch each, the longest.  (The
    # selection call is three launches; its largest kernel, the partition pass, is shorter than the
    # compaction kernel -- see profiles/bench_kernel_trace.txt -- and the call as a whole is reported
    # in `calls` and, flat, below.)
    with_traffic = not (args.no_traffic or args.small)
    table, traffic_source = traffic_table() if with_traffic else ({}, None)
    by_name = {c["call"]: c for c in calls}
    dom = max((c for c in calls[:4] if c["launches"] == 1), key=lambda c: c["us"])
    roofline = {"bound": "hbm", "kernel": CALL_KERNELS[dom["call"]][0][0], "call": dom["call"],
                "achieved": dom["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(dom["GBps"] / HBM_PEAK_GBPS, 4),
                "traffic": measured_traffic(dom["call"], table) if with_traffic else None,
                "traffic_source": traffic_source,
                "algorithmic_bytes": dom["algorithmic_bytes"], "launch_us": dom["us"],
                "note": "achieved = algorithmic bytes of one launch / average launch time (HIP events); traffic = scaled "
                        "FETCH_SIZE + WRITE_SIZE per launch"}
    # the other calls of the metric, flat (a reader of a trimmed record still sees them)
    for key, name in (("select_c4", "dct_select_threshold[c4]"), ("fwd_c5", "dct_rowtopk_fwd[c5]"),
                      ("bwd_c5", "dct_rowtopk_bwd[c5]"), ("select_c3", "dct_select_threshold[c3]"),
                      ("compact_c3_reuse", "dct_threshold_compact[c3,ge_tau,reuse]")):
        if name in by_name:
            roofline[key + "_us"] = by_name[name]["us"]
            roofline[key + "_frac"] = by_name[name]["frac_of_hbm_peak"]
    roofline["bwd_c5_frac_strict"] = by_name["dct_rowtopk_bwd[c5]"]["frac_of_hbm_peak_strict"]
    # the forward call against a kernel that only moves its bytes (probes: rows_c5_read_write_us)
    roofline["fwd_c5_traffic_only_us"] = probes["rows_c5_read_write_us"]
    roofline["fwd_c5_frac_of_traffic_only"] = round(probes["rows_c5_read_write_us"] / by_name["dct_rowtopk_fwd[c5]"]["us"], 4)
    for w in narrow:  # the paper's MP widths, flat as well
        roofline[f"fwd_d{w['D']}_us"] = w["fwd_us"]
        roofline[f"fwd_d{w['D']}_frac"] = w["fwd_frac_of_hbm_peak"]
    for c in calls[:4] + ef_calls + rx_calls + bm_calls + i16_calls:
        c["traffic"] = measured_traffic(c["call"], table) if with_traffic else None

    # ------------------------------------------------------------ CPU oracle on the same step's input
    cpu = None
    if not args.no_cpu:
        import oracle
        n_s = min(n4, 1 << 28)   # at the benchmark's sizes this is the whole step: about 15 s on one core
        b_s = min(B5, 65536)
        k_s = si.ceil_frac(n_s, 5, 1000)
        gs = g4[0][:n_s].cpu().numpy()
        xs = oracle.as_numpy(x5[0][:b_s].cpu())
        dys = oracle.as_numpy(dy5[0][:b_s].cpu())
        t = {}
        t0 = time.perf_counter(); thr_s = oracle.select_threshold(gs, k_s); t["select_full_sort"] = time.perf_counter() - t0
        t0 = time.perf_counter(); ci, cv, cc = oracle.threshold_compact(gs, thr_s, oracle.EXACT_K, capacity=k_s); t["compact"] = time.perf_counter() - t0
        t0 = time.perf_counter(); ei, ev, _ = oracle.rowtopk_fwd(xs, k5); t["rowtopk_fwd"] = time.perf_counter() - t0
        t0 = time.perf_counter(); ed = oracle.rowtopk_bwd(dys, ei); t["rowtopk_bwd"] = time.perf_counter() - t0
        total = sum(t.values())
        t0 = time.perf_counter(); oracle.select_threshold(gs, k_s, method="nth"); t_nth = time.perf_counter() - t0

        # The same oracle spread trivially over the host's cores where the work is independent: rows for the
        # row top-k, chunks + ordered concatenation for the compaction (the mask of Algorithm 1 per chunk; the
        # ties beyond the quota are dropped afterwards).  The selection stays ONE full sort: its time is the
        # single-thread one.  (The oracle's C routines release the interpreter lock, so threads do.)
        cores = max(1, min(16, os.cpu_count() or 1))
        tp = {}
        with ThreadPoolExecutor(cores) as pool:
            bounds = [n_s * j // cores for j in range(cores + 1)]
            t0 = time.perf_counter()
            parts = list(pool.map(lambda j: oracle.threshold_compact(gs[bounds[j]:bounds[j + 1]], thr_s, oracle.GE_TAU),
                                  range(cores)))
            pidx = np.concatenate([p_[0].astype(np.int64) + bounds[j] for j, p_ in enumerate(parts)])
            pval = np.concatenate([p_[1] for p_ in parts])
            tie = (pval.view(np.uint32) & 0x7FFFFFFF) == thr_s.tau_key
            keep = ~tie | (np.cumsum(tie) <= thr_s.tie_quota)
            pidx, pval = pidx[keep], pval[keep]
            tp["compact"] = time.perf_counter() - t0
            rb = [b_s * j // cores for j in range(cores + 1)]
            t0 = time.perf_counter()
            fparts = list(pool.map(lambda j: oracle.rowtopk_fwd(xs[rb[j]:rb[j + 1]], k5), range(cores)))
            pei = np.concatenate([f_[0] for f_ in fparts])
            tp["rowtopk_fwd"] = time.perf_counter() - t0
            t0 = time.perf_counter()
            ped = np.concatenate(list(pool.map(lambda j: oracle.rowtopk_bwd(dys[rb[j]:rb[j + 1]], pei[rb[j]:rb[j + 1]]),
                                               range(cores))))
            tp["rowtopk_bwd"] = time.perf_counter() - t0
        assert np.array_equal(pidx, ci[:cc].astype(np.int64)) and np.array_equal(pei, ei) and np.array_equal(ped, ed)
        total_par = t["select_full_sort"] + sum(tp.values())
        model = ""
        try:
            with open("/proc/cpuinfo") as f:
                model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), "")
        except OSError:
            pass
        elems = n_s + b_s * D5
        cpu = {"value": elems / total, "unit": "elements/s", "cores": 1, "kind": "oracle",
               "sample": f"one whole step: {n_s} elements of c4 (k={k_s}), {b_s} rows of c5; full-sort select + scalar "
                         f"compact + partial-sort row top-k + gather",
               "seconds_select_full_sort": round(t["select_full_sort"], 3), "seconds_compact": round(t["compact"], 3),
               "seconds_rowtopk_fwd": round(t["rowtopk_fwd"], 3), "seconds_rowtopk_bwd": round(t["rowtopk_bwd"], 3),
               "select_nth_element_seconds": round(t_nth, 3),
               "all_cores_value": elems / total_par, "all_cores": cores,
               "all_cores_seconds_compact": round(tp["compact"], 3), "all_cores_seconds_rowtopk_fwd": round(tp["rowtopk_fwd"], 3),
               "all_cores_seconds_rowtopk_bwd": round(tp["rowtopk_bwd"], 3),
               "all_cores_without_select_value": elems / sum(tp.values()),
               "all_cores_note": "rows / chunks over threads; the selection stays one full sort on one core",
               "host_cpus": os.cpu_count(), "cpu_model": model}
        log(f"[bench] cpu oracle: {cpu}")

    out = {
        "metric": "elements/s and % of HBM peak: DP threshold+compact, MP row top-k fwd/bwd",
        "value": value, "unit": "elements/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 keys of fp32 (DP) / u16 keys of bf16 (MP); integer compare and bit copy only",
        "data": "synthetic",
        "config": {"workload": "c4 DP select+compact (N=2^28 fp32, keep 0.5%) + c5 MP row top-k fwd+bwd "
                               "(65536x4096 bf16, k=204)" + (" [SHRUNK 16x: not a valid number]" if args.small else ""),
                   "elements_per_step": elems_per_step, "dp_n": n4, "dp_k": k4, "mp_B": B5, "mp_D": D5, "mp_k": k5},
        "roofline": roofline, "calls": calls, "small_config_calls": small_calls, "error_feedback_calls": ef_calls,
        "decompression_calls": rx_calls, "bitmask_calls": bm_calls, "idx16_calls": i16_calls,
        "paper_mp_widths": narrow, "batched_small_tensors": batched, "probes": probes, "c3_reuse": c3, "cpu_baseline": cpu,
        "inputs": inputs,
    }
    print(json.dumps(out), flush=True)

    # ------------------------------------------------------------ the short form, last on stderr
    log("[bench] ---- summary (us, fraction of the 8 TB/s peak, elements/s)")
    for c in calls + small_calls:
        log(f"[bench] {c['call']}: {c['us']} us {c['frac_of_hbm_peak']:.3f} {c['elements_per_s']:.3g}")
    for w in narrow:
        log(f"[bench] MP bf16 D={w['D']} k={w['k']} B={w['B']}: fwd {w['fwd_us']} us {w['fwd_frac_of_hbm_peak']:.3f} "
            f"(traffic only {w['traffic_only_us']} us), bwd {w['bwd_us']} us, scatter {w['scatter_us']} us")
    log(f"[bench] step {ms_per_step:.4f} ms = {value:.4g} elements/s; probes {probes}")
    if cpu:
        log(f"[bench] cpu oracle: 1 core {cpu['value']:.3g} el/s; {cpu['all_cores']} cores {cpu['all_cores_value']:.3g} el/s "
            f"(without the one-core sort {cpu['all_cores_without_select_value']:.3g})")


if __name__ == "__main__":
    main()
