#!/usr/bin/env python3
"""Benchmark of the pQuant decoupled linear on one MI355X.

A step is one forward + STE backward of the whole hot path on the 1.3B-shaped attention projection
(tokens=8192, 2048x2048 1-bit branch, rank-128 high-precision branch, bf16 I/O, fp32 weight
gradients): weight statistics, binarise+pack, activation quantiser, int8 MFMA GEMM, hp branch,
and the backward GEMMs with the alpha/beta reductions.  Inputs are synthetic, seeded, and already
resident in HBM when the timed region starts.

Prints ONE JSON line (see the keys below).  `value` comes from a timed region of exactly `--steps` steps
between synchronisations.  `roofline` is for the dominant kernel: its duration is measured with HIP events
recorded by the library around each launch, on the launch stream, in a second pass over the same steps
(the events open gaps between launches, so they stay out of the region that is timed as a whole);
`cpu_baseline` is the NumPy oracle timed on a bounded sample of the same workload.

Defaults: 50 warm-up and 200 timed steps (0.1 s of GPU time).  Short runs measure the clock ramp of a GPU that
has just been idle rather than the kernels: 5 + 20 steps read 8 % slower than the steady state on the same box.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16 = 2.5e15      # dense MFMA bf16, FLOP/s
PEAK_I8 = 5.0e15        # dense MFMA int8, OP/s
PREWARM_S = 0.25        # seconds of the headline step run before its warm-up steps (reported as "prewarm_s")

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
# kernel-name fragments of the three large GEMMs of the default workload (template arguments: ..., whole tiles, int8,
# operand kinds of A and B, kinds of the fused second contraction, streaming loop)
TRAFFIC_KERNELS = {"gemm_dW": "gemm_tn_w4_kernel", "gemm_dX": "128, true, false, 0, 4, 0, 1, true>",
                   "gemm_onebit_fwd": "128, true, true, 2, 3, 0, 0, true>", "decode_main_B1": "decode_gemv_tiled_kernel<1, false>",
                   "decode_main_B8": "decode_gemm16_tiled_kernel<8, false>", "decode_prep_B1": "decode_prep_h_kernel<false>",
                   "decode_prep_B8": "decode_prep_kernel", "decode_h_B8": "decode_h_grouped_kernel<8>"}


def csrc_sha():
    """Digest of the kernel sources the loaded library was built from: measured traffic figures are only quoted for the
    sources they were measured on."""
    import hashlib
    d = os.path.join(ROOT, "paper_2602_22592_amd", "csrc")
    h = hashlib.sha256()
    for fn in sorted(os.listdir(d)):
        if fn.endswith((".hip", ".h")):
            h.update(fn.encode()); h.update(open(os.path.join(d, fn), "rb").read())
    return h.hexdigest()[:16]


def load_traffic():
    """{label: HBM bytes per launch} from profiles/hbm_traffic.json (written by `bench.py --traffic-from`), or {} when the
    file is missing or was measured on other kernel sources."""
    try:
        t = json.load(open(TRAFFIC_FILE))
        if t.get("csrc_sha") != csrc_sha():
            return {}
        return {k: v["bytes"] for k, v in t["kernels"].items()}
    except Exception:
        return {}


def write_traffic(fetch_csv, write_csv):
    """Turns two rocprofv3 --pmc counter CSVs (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch) of a `--calibrate` run of this
    script into profiles/hbm_traffic.json.  Each counter is scaled by what it reads for the calibration copy of known size."""
    import collections
    import csv

    def avg(path):
        agg = collections.defaultdict(list)
        for r in csv.DictReader(open(path)):
            agg[r["Kernel_Name"]].append(float(r["Counter_Value"]))
        return {k: sum(v) / len(v) for k, v in agg.items()}
    F, W = avg(fetch_csv), avg(write_csv)
    cal_f = next(v for k, v in F.items() if "gather_rows_kernel" in k)
    cal_w = next(v for k, v in W.items() if "gather_rows_kernel" in k)
    rows, cols = 65536, 2048
    ff, fw = (rows * cols * 2 + rows * 4) / 1024.0 / cal_f, (rows * cols * 2) / 1024.0 / cal_w
    out = {"csrc_sha": csrc_sha(), "fetch_factor": round(ff, 4), "write_factor": round(fw, 4),
           "calibration": "gather_rows_kernel copy of 65536 x 2048 bf16", "kernels": {}}
    for label, frag in TRAFFIC_KERNELS.items():
        kf = [v for k, v in F.items() if frag in k]
        kw = [v for k, v in W.items() if frag in k]
        if kf and kw:
            out["kernels"][label] = {"kernel": frag, "fetch_kib": round(kf[0], 1), "write_kib": round(kw[0], 1),
                                     "bytes": int((kf[0] * ff + kw[0] * fw) * 1024)}
    json.dump(out, open(TRAFFIC_FILE, "w"), indent=1)
    print(json.dumps(out, indent=1))


def gemm_flops(T, K, N, r):
    """Algorithmic flops of one launch of each GEMM label (2 * M * N * K each)."""
    return {
        "gemm_onebit_fwd": 2.0 * T * K * N,
        "gemm_hp_H": 2.0 * T * r * K, "gemm_hp_Y": 2.0 * T * N * r,
        "gemm_dH": 2.0 * T * r * N, "gemm_dX": 2.0 * T * K * N, "gemm_dX_hp": 2.0 * T * K * r,
        "gemm_dW": 2.0 * T * K * N,
        "gemm_dB": 2.0 * T * N * r + 2.0 * T * r * K,      # dB and dA share one launch, timed under this label
    }


def cpu_baseline(sample_tokens):
    """The oracle as it stands, on the host cores, on the first `sample_tokens` tokens of the workload."""
    from oracle import pquant_oracle as po
    from paper_2602_22592_amd import workloads as wl
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    c = wl.config2(tokens=sample_tokens)
    t0 = time.perf_counter()
    f = po.linear_fwd(c["X"], c["W"], c["alpha"], c["beta"], A=c["A"], B=c["B"])
    po.linear_bwd(c["dY"], c["X"], c["W"], c["alpha"], c["beta"], f, A=c["A"], B=c["B"])
    dt = time.perf_counter() - t0
    return {"value": sample_tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {sample_tokens} tokens of the workload, fwd+bwd, {dt:.1f} s"}


def decode_bench(pq, torch, batch, n_layers=64, steps=100, warmup=20, int8_experts=False):
    """Packed-1-bit decode product, 4096 -> 11008 with E=8 top-2 rank-64 experts (bf16, or their INT8 form), over
    `n_layers` distinct weight sets per launch (361 MB of bits: larger than the Infinity Cache)."""
    K, N, E, r, k = 4096, 11008, 8, 64, 2
    g = torch.Generator(device="cuda").manual_seed(4)
    bf = torch.bfloat16
    P = torch.randint(-2**31, 2**31 - 1, (n_layers, N, K // 32), dtype=torch.int32, device="cuda", generator=g)
    X = torch.randn((n_layers, batch, K), device="cuda", generator=g).to(bf)
    A = (torch.randn((n_layers, E, r, K), device="cuda", generator=g) * 0.02).to(bf)
    Bm = (torch.randn((n_layers, E, N, r), device="cuda", generator=g) * 0.02).to(bf)
    Wr = (torch.randn((n_layers, E, K), device="cuda", generator=g) * 0.02).to(bf)
    scale = torch.from_numpy(np.full(n_layers, np.float16(0.2 * 0.016)).view(np.int16)).cuda()
    Y = torch.empty((n_layers, batch, N), dtype=bf, device="cuda")
    tiled = True              # the decode kernels stream the row-interleaved packing (re-tiled offline)
    if tiled:
        P = torch.stack([pq.pack_retile64(P[l], K) for l in range(n_layers)]).contiguous()
    desc = pq.DecodeDesc(batch, K, N, r, E, k, n_layers, pq.PQ_PACKED_TILED64 if tiled else pq.PQ_PACKED_ROWMAJOR, 2.0)
    ws = pq.decode_workspace(desc)
    run = lambda: pq.decode_gemv(desc, X, P, scale, Y, ws, A=A, B=Bm, Wr=Wr)
    eb = 2                                                  # bytes per expert weight
    if int8_experts:
        Aq, gA = pq.quant_rows(A)
        Bq, gB = pq.quant_rows(Bm)
        del A, Bm
        run = lambda: pq.decode_gemv_int8(desc, X, P, scale, Y, ws, Aq, gA, Bq, gB, Wr)
        eb = 1
    _warm(torch, run)
    total_us = 1e3 * _time_steps(torch, run, steps, warmup)        # whole calls, no per-launch events
    pq.prof_reset(); pq.prof_enable(True)                          # second pass: per-kernel durations
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    pq.prof_enable(False)
    prof = pq.prof_read(); pq.prof_reset()
    main_us = 1e3 * prof["decode_main"][0] / prof["decode_main"][1]
    prep_us = 1e3 * prof["decode_prep"][0] / prof["decode_prep"][1]
    h_us = 1e3 * prof["decode_h"][0] / prof["decode_h"][1] if "decode_h" in prof else 0.0   # batch 1: fused into prep
    # algorithmic bytes: packed bits + the rows of the DISTINCT experts a layer's tokens selected (read back from the
    # routing decisions of the last call, outside every timed region) + router + x, y
    idx = pq.decode_ws_idx(desc, ws).cpu().numpy().reshape(n_layers, -1)
    n_sel = sum(len(set(row.tolist())) for row in idx)      # summed over the layers
    main_bytes = n_layers * (N * K // 8 + batch * (K + 2 * N)) + n_sel * N * (r * eb + (4 if int8_experts else 0))
    prep_bytes = n_layers * (batch * 2 * K + E * K * 2) + n_sel * r * K * eb    # x, router, the selected experts' A
    whole = (main_bytes + prep_bytes) / total_us / 1e3
    return {"batch": batch, "experts": "int8" if int8_experts else "bf16", "layers_per_launch": n_layers,
            "distinct_experts_per_layer": round(n_sel / n_layers, 3), "main_kernel_us": round(main_us, 2),
            "prep_kernel_us": round(prep_us, 2), "h_kernel_us": round(h_us, 2), "launch_us": round(total_us, 2),
            "whole_call_GBps": round(whole, 1), "whole_call_frac_hbm": round(whole / 8000.0, 4),
            "main_kernel_GBps": round(main_bytes / main_us / 1e3, 1), "main_kernel_frac_hbm": round(main_bytes / main_us / 1e3 / 8000.0, 4),
            "us_per_layer": round(total_us / n_layers, 3), "bytes_per_layer": (main_bytes + prep_bytes) // n_layers}


def decode_ffn_bench(pq, torch, n_layers=32, steps=100, warmup=20, batch=1):
    """The decoupled FFN at inference, `batch` tokens per layer: 4096 -> 11008 -> 4096 packed 1-bit matrices with E=8
    top-2 experts of hidden width 64, `n_layers` distinct FFNs per call (541 MB of bits)."""
    D, F, E, r, k = 4096, 11008, 8, 64, 2
    g = torch.Generator(device="cuda").manual_seed(9)
    bf = torch.bfloat16
    rnd = lambda *s: torch.randint(-2**31, 2**31 - 1, s, dtype=torch.int32, device="cuda", generator=g)
    Pug = rnd(n_layers, 2, ((F + 63) // 64) * 64 * (D // 32))     # random bits, already in the row-interleaved order
    Pd = rnd(n_layers, ((D + 63) // 64) * 64 * (F // 32))
    X = torch.randn((n_layers, batch, D), device="cuda", generator=g).to(bf)
    UpGate = (torch.randn((n_layers, E, 2 * r, D), device="cuda", generator=g) * 0.02).to(bf)
    Down = (torch.randn((n_layers, E, D, r), device="cuda", generator=g) * 0.02).to(bf)
    Wr = (torch.randn((n_layers, E, D), device="cuda", generator=g) * 0.02).to(bf)
    sug = torch.from_numpy(np.full((n_layers, 2), np.float16(0.016)).view(np.int16)).cuda()
    sd = torch.from_numpy(np.full(n_layers, np.float16(0.4 * 0.016)).view(np.int16)).cuda()
    Y = torch.empty((n_layers, batch, D), dtype=bf, device="cuda")
    desc = pq.DecodeFFNDesc(D, F, r, E, k, n_layers, 1.5, batch)
    ws = pq.decode_ffn_workspace(desc)
    run = lambda: pq.decode_ffn(desc, X, Pug, sug, Pd, sd, UpGate, Down, Wr, Y, ws)
    _warm(torch, run)
    total_us = 1e3 * _time_steps(torch, run, steps, warmup)
    prof = _profile_steps(pq, torch, run, steps)
    # algorithmic bytes per layer: three packed matrices, the distinct selected experts (2r x D and D x r bf16; the
    # expected number of distinct experts over the batch's independent top-k choices), router, x, y
    distinct = E * (1.0 - (1.0 - k / E) ** batch) if batch > 1 else k
    per_layer = int(3 * D * F // 8 + distinct * (2 * r * D + D * r) * 2 + E * D * 2 + batch * 4 * D)
    return {"batch": batch, "layers_per_call": n_layers, "call_us": round(total_us, 2), "us_per_layer": round(total_us / n_layers, 3),
            "bytes_per_layer": per_layer, "whole_call_GBps": round(per_layer * n_layers / total_us / 1e3, 1),
            "frac_hbm": round(per_layer * n_layers / total_us / 1e3 / 8000.0, 4),
            "kernels_us_total_per_call": {k_: round(1e3 * ms / steps, 2) for k_, (ms, n) in sorted(prof.items())}}


def _warm(torch, fn, seconds=0.2):
    """Run fn back to back for `seconds` of wall time: the first measurement of a bandwidth-bound section in a process
    otherwise reads 5-15 % slow (the first hundred milliseconds of a new access pattern)."""
    t_end = time.time() + seconds
    while time.time() < t_end:
        for _ in range(50):
            fn()
        torch.cuda.synchronize()


def _time_steps(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def _profile_steps(pq, torch, fn, steps):
    """A separate pass with the library's per-launch HIP events on (they cost launch gaps, so the pass that is
    timed as a whole runs without them).  Returns {label: (total ms, launches)}."""
    torch.cuda.synchronize()
    pq.prof_reset(); pq.prof_enable(True)
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    pq.prof_enable(False)
    prof = pq.prof_read(); pq.prof_reset()
    return prof


def norm_quant_bench(pq, torch, T=8192, K=2048, sets=4, steps=100, warmup=20):
    """RMSNorm fused with the AbsMax quantiser at the config-2 activation shape (bf16), forward (all outputs)
    and backward, against HBM bandwidth.  The calls rotate over `sets` buffer sets so that the working set
    (sets x 112 MB forward) is larger than the 256 MB last-level cache.  Algorithmic bytes per element:
    forward 2 (x) + 2 (x_hat) + 1 (codes) + 2 (q / gamma) = 7; backward 2 (dx_hat) + 2 (x) + 2 (dx) = 6."""
    g = torch.Generator(device="cuda").manual_seed(6)
    bf = torch.bfloat16
    Xs = [torch.randn((T, K), device="cuda", generator=g).to(bf) for _ in range(sets)]
    dXs = [torch.randn((T, K), device="cuda", generator=g).to(bf) for _ in range(sets)]
    gain = (1.0 + 0.1 * torch.randn((K,), device="cuda", generator=g)).to(bf)
    outs = [dict(Xn=torch.empty_like(Xs[0]), Xq=torch.empty((T, K), dtype=torch.int8, device="cuda"),
                 gamma=torch.empty((T,), dtype=torch.float32, device="cuda"), Xt=torch.empty_like(Xs[0]),
                 rstd=torch.empty((T,), dtype=torch.float32, device="cuda"), dX=torch.empty_like(Xs[0]),
                 dg=torch.empty((K,), dtype=torch.float32, device="cuda")) for _ in range(sets)]
    ws = torch.empty(pq.lib().pq_rmsnorm_bwd_workspace_bytes(T, K), dtype=torch.uint8, device="cuda")
    it = [0]

    def fwd():
        i = it[0] % sets; it[0] += 1
        o = outs[i]
        pq.rmsnorm_quant_fwd_into(Xs[i], gain, 1e-6, o["Xn"], o["Xq"], o["gamma"], o["Xt"], o["rstd"])

    def bwd():
        i = it[0] % sets; it[0] += 1
        o = outs[i]
        pq.rmsnorm_bwd_into(dXs[i], Xs[i], gain, o["rstd"], o["dX"], o["dg"], ws)

    def unfused():
        i = it[0] % sets; it[0] += 1
        o = outs[i]
        pq.quant_act_into(Xs[i], o["Xq"], o["gamma"])

    for _ in range(sets):
        fwd()
    ms_f = _time_steps(torch, fwd, steps, warmup)
    ms_b = _time_steps(torch, bwd, steps, warmup)
    ms_q = _time_steps(torch, unfused, steps, warmup)
    n = T * K
    fb, bb, qb = 7 * n + 8 * T, 6 * n + 4 * T + 4 * K, 3 * n + 4 * T
    return {"workload": "tokens=%d, d=%d, bf16; buffers rotate over %d sets" % (T, K, sets),
            "fwd_us": round(ms_f * 1e3, 2), "fwd_GBps": round(fb / ms_f / 1e6, 1), "fwd_frac_hbm": round(fb / ms_f / 1e6 / 8000.0, 4),
            "bwd_us": round(ms_b * 1e3, 2), "bwd_GBps": round(bb / ms_b / 1e6, 1), "bwd_frac_hbm": round(bb / ms_b / 1e6 / 8000.0, 4),
            "plain_quantiser_us": round(ms_q * 1e3, 2), "plain_quantiser_GBps": round(qb / ms_q / 1e6, 1)}


def hp_int8_bench(pq, torch, T=8192, K=2048, N=2048, r=128, steps=100, warmup=20):
    """INT8 form of the high-precision branch at the config-2 shape: forward (weight-row quantisers, two int8
    GEMMs with the de-quantising epilogue, hidden-state quantiser) and STE backward (four bf16 GEMMs)."""
    g = torch.Generator(device="cuda").manual_seed(8)
    bf = torch.bfloat16
    X = torch.randn((T, K), device="cuda", generator=g).to(bf)
    A = (0.02 * torch.randn((r, K), device="cuda", generator=g)).to(bf)
    B = (0.02 * torch.randn((N, r), device="cuda", generator=g)).to(bf)
    dY = torch.randn((T, N), device="cuda", generator=g).to(bf)
    gain = torch.ones((K,), dtype=bf, device="cuda")
    _, Xq, gx, Xt, _ = pq.rmsnorm_quant_fwd(X, gain, 1e-6, want_xn=False, want_rstd=False)
    bufs = pq.HpInt8Buffers(T, K, N, r)
    Y = torch.zeros((T, N), dtype=bf, device="cuda")
    dX = torch.empty((T, K), dtype=bf, device="cuda")
    dA = torch.empty((r, K), dtype=torch.float32, device="cuda")
    dB = torch.empty((N, r), dtype=torch.float32, device="cuda")
    fwd = lambda: pq.hp_int8_fwd(Xq, gx, A, B, 1.0, Y, bufs)
    bwd = lambda: pq.hp_int8_bwd(dY, Xt, 1.0, bufs, dX, dA, dB)
    ms_f = _time_steps(torch, fwd, steps, warmup)
    ms_b = _time_steps(torch, bwd, steps, warmup)
    prof = _profile_steps(pq, torch, lambda: (fwd(), bwd()), steps)
    ops_f = 2.0 * T * r * (K + N)
    return {"workload": "tokens=%d, d_in=%d, d_out=%d, r=%d, bf16 I/O" % (T, K, N, r),
            "fwd_us": round(ms_f * 1e3, 2), "fwd_int8_TOPs": round(ops_f / ms_f / 1e9, 1),
            "bwd_us": round(ms_b * 1e3, 2), "bwd_bf16_TFLOPs": round(2.0 * ops_f / ms_b / 1e9, 1),
            "kernels_us": {k: round(1e3 * ms / n, 2) for k, (ms, n) in sorted(prof.items())}}


def fp32_io_bench(pq, torch, c, steps=5, warmup=2):
    """The config-2 step with fp32 activations and gradients: every GEMM except the int8 one runs on the fp64 matrix
    instructions (the path the tight-tolerance parity tests use).  Reported so that its cost is known; fp64 MFMA peak
    78.6 TFLOP/s."""
    T, K, N, r = c["tokens"], c["d_in"], c["d_out"], c["hp_rank"]
    to = lambda x: torch.from_numpy(x).cuda().float()
    X, W, dY, A, B = to(c["X"]), to(c["W"]), to(c["dY"]), to(c["A"]), to(c["B"])
    desc = pq.make_desc(T, K, N, hp_rank=r, io_dtype=pq.PQ_F32, alpha=c["alpha"], beta=c["beta"])
    bufs = pq.LinearBuffers(desc)
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    Y, dX, dW, dA, dB, dab = f32(T, N), f32(T, K), f32(N, K), f32(r, K), f32(N, r), f32(2)

    def step():
        pq.linear_fwd(desc, X, W, Y, bufs, A=A, B=B)
        pq.linear_bwd(desc, dY, X, W, bufs, dX, dW, dab, A=A, B=B, dA=dA, dB=dB)

    ms = _time_steps(torch, step, steps, warmup)
    prof = _profile_steps(pq, torch, step, steps)
    k_us = {k: round(1e3 * t / n, 1) for k, (t, n) in sorted(prof.items())}
    big = 2.0 * T * K * N
    return {"workload": "tokens=%d, d_in=%d, d_out=%d, r=%d, fp32 I/O, fwd+bwd" % (T, K, N, r), "ms_per_step": round(ms, 3),
            "tokens_per_s": round(T / (ms * 1e-3), 1),
            "gemm_dX_fp64_TFLOPs": round(big / (k_us["gemm_dX"] * 1e-6) / 1e12, 1) if "gemm_dX" in k_us else None,
            "gemm_dW_fp64_TFLOPs": round(big / (k_us["gemm_dW"] * 1e-6) / 1e12, 1) if "gemm_dW" in k_us else None,
            "kernels_us": k_us}


def ffn_bench(pq, torch, T=8192, D=2048, F=5504, E=8, r=32, steps=20, warmup=5, int8_experts=False):
    """Config 3: the 1.3B-shaped decoupled FFN (three 1-bit projections + E=8 top-1 experts of width 32), fwd+bwd.
    With F=5076, r=384 and E in {1, 2, 4, 8} it is the paper's own 1.3B FFN (Table 1) and its branch sweep (Sec. 4.4)."""
    g = torch.Generator(device="cuda").manual_seed(3)
    bf = torch.bfloat16
    rn = lambda *s, std=0.02: (torch.randn(s, device="cuda", generator=g) * std).to(bf)
    X = rn(T, D, std=1.0); dY = rn(T, D, std=1.0)
    W_up, W_gate, W_down = rn(F, D), rn(F, D), rn(D, F)
    Up, Gate, Down, Wr = rn(E, r, D), rn(E, r, D), rn(E, D, r), rn(E, D)
    desc = pq.FFNDesc(T, D, F, r, E, 1, pq.PQ_BF16, 2.0, 0.2, pq.PQ_HP_LOWRANK_INT8 if int8_experts else pq.PQ_HP_LOWRANK_BF16)
    bufs = pq.FFNBuffers(desc)
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    Y = torch.empty((T, D), dtype=bf, device="cuda"); dX = torch.empty((T, D), dtype=bf, device="cuda")
    gr = (f32(F, D), f32(F, D), f32(D, F), f32(E, r, D), f32(E, r, D), f32(E, D, r), f32(E, D), f32(2))

    def step():
        pq.ffn_fwd(desc, X, W_up, W_gate, W_down, Up, Gate, Down, Wr, Y, bufs)
        pq.ffn_bwd(desc, dY, X, Up, Gate, Down, Wr, bufs, dX, *gr)
    ms = _time_steps(torch, step, steps, warmup)
    prof = _profile_steps(pq, torch, step, steps)
    # one active expert per token: 3 projections of width r forward, 6 GEMMs backward (bf16)
    t_mfma = 3 * 2.0 * T * D * F / PEAK_I8 + 6 * 2.0 * T * D * F / PEAK_BF16 + 9 * 2.0 * T * D * r / PEAK_BF16
    # roofline of the label with the largest total time: its launches are GEMMs of 2 T D F flops each
    big = {k: v for k, v in prof.items() if k in ("gemm_dW", "gemm_dX", "gemm_onebit_fwd")}
    dom = max(big, key=lambda k: big[k][0])
    peak = PEAK_I8 if dom == "gemm_onebit_fwd" else PEAK_BF16
    ach = 2.0 * T * D * F * big[dom][1] / (big[dom][0] * 1e-3)
    return {"workload": f"tokens={T}, d_model={D}, d_ffn={F}, E={E} {'INT8' if int8_experts else 'bf16'} experts of width {r}, top-1, "
                        "bf16 I/O, fwd+bwd",
            "ms_per_step": round(ms, 4), "tokens_per_s": round(T / ms * 1e3, 1), "mfma_frac_of_step": round(t_mfma / (ms * 1e-3), 4),
            "roofline": {"bound": "mfma", "kernel": dom, "achieved": round(ach / 1e12, 2), "peak": peak / 1e12,
                         "unit": "TOP/s" if dom == "gemm_onebit_fwd" else "TFLOP/s", "frac": round(ach / peak, 4),
                         "avg_us": round(1e3 * big[dom][0] / big[dom][1], 2), "traffic": None},
            "kernels_us_total_per_step": {k: round(1e3 * v[0] / steps, 1) for k, v in sorted(prof.items())}}


def stack_bench(pq, torch, L=24, T=16384, D=2048, F=5504, E=8, r=32, steps=2, warmup=1):
    """Config 5: 24 layers of {q,k,v,o pure 1-bit 2048^2 linears + the config-3 FFN}, one fwd+bwd over 16384 tokens."""
    from paper_2602_22592_amd import workloads as wl
    from paper_2602_22592_amd.stack import Stack
    g = torch.Generator(device="cuda").manual_seed(5)
    bf = torch.bfloat16
    rn = lambda *s, std=0.02: (torch.randn(s, device="cuda", generator=g) * std).to(bf)
    shapes = dict(Wq=(D, D), Wk=(D, D), Wv=(D, D), Wo=(D, D), W_up=(F, D), W_gate=(F, D), W_down=(D, F), Up=(E, r, D),
                  Gate=(E, r, D), Down=(E, D, r), Wr=(E, D))
    weights = [{n: rn(*s) for n, s in shapes.items()} for _ in range(L)]
    grads = [dict({n: torch.empty(s, dtype=torch.float32, device="cuda") for n, s in shapes.items()},
                  dab=torch.empty(2, dtype=torch.float32, device="cuda")) for _ in range(L)]
    table = rn(32000, D, std=1.0)
    ids = torch.randint(0, 32000, (T,), dtype=torch.int32, device="cuda", generator=g)
    dY = rn(T, D, std=1.0)
    st = Stack(L, T, D, F, E, r, 1, [wl.TRAINED_ALPHA[l % 16] for l in range(L)], [wl.TRAINED_BETA[l % 16] for l in range(L)])
    h0 = torch.empty((T, D), dtype=bf, device="cuda")

    def step():
        pq.glue_gather_rows(table, ids, h0)
        st.forward(h0, weights)
        st.backward(dY, weights, grads)
    ms = _time_steps(torch, step, steps, warmup)
    prof = _profile_steps(pq, torch, step, 1)
    glue_ms = prof.get("glue", (0.0, 1))[0]
    ops_i8 = L * (4 * 2.0 * T * D * D + 3 * 2.0 * T * D * F)
    t_mfma = ops_i8 / PEAK_I8 + 2 * ops_i8 / PEAK_BF16
    return {"workload": f"{L} layers x (4 pure 1-bit {D}x{D} linears + FFN d_ffn={F}, E={E}x{r} top-1), tokens={T}, bf16, fwd+bwd",
            "ms_per_step": round(ms, 3), "ms_per_layer": round(ms / L, 3), "tokens_per_s": round(T / ms * 1e3, 1),
            "glue_ms_per_step": round(glue_ms, 3), "linears_ms_per_step": round(ms - glue_ms, 3),
            "mfma_frac_of_step": round(t_mfma / (ms * 1e-3), 4)}


def vendor_gemm_context(torch, X, W, dY, steps=100, warmup=10):
    """Context, not product: what the vendor GEMM library (through torch.matmul, bf16) needs on this machine for plain GEMMs
    of the step's three shapes on the same operands, and for a large square GEMM on normal and on all-zero operands.
    With real operand data the chip runs matrix work against its power limit (the shader clock falls with the toggling
    of the data), so the nominal 2.5 PFLOP/s is not what any kernel is measured against in practice."""
    T, K = X.shape
    N = W.shape[0]
    def t(f, n=steps):
        for _ in range(warmup):
            f()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n
    out = {}
    for name, f in (("fwd_X_Wt", lambda: torch.matmul(X, W.t())), ("dX_dY_W", lambda: torch.matmul(dY, W)),
                    ("dW_dYt_X", lambda: torch.matmul(dY.t(), X))):
        us = t(f)
        out[name] = {"us": round(us, 1), "TFLOP/s": round(2.0 * T * K * N / us / 1e6, 0)}
    n = 8192
    for data in ("normal", "zero"):
        a = torch.randn((n, n), device="cuda").to(torch.bfloat16) if data == "normal" else torch.zeros((n, n), dtype=torch.bfloat16, device="cuda")
        b = a.clone()
        us = t(lambda: torch.matmul(a, b.t()), 20)
        out[f"square_8192_{data}"] = {"us": round(us, 1), "TFLOP/s": round(2.0 * n ** 3 / us / 1e6, 0)}
        del a, b
    return out


def groupwise_contrast(pq, torch, X, W, steps=50, warmup=10):
    """Sec. 4.6's group-wise(64) weight scales against the per-tensor scale, both in the contrast kernel (forward only:
    quantiser, statistics, packing, group scales, GEMM), plus the GEMM launch alone from the library's events."""
    out = {"workload": f"tokens={X.shape[0]}, d_in={X.shape[1]}, d_out={W.shape[0]}, bf16 in, fp32 out, forward only"}
    for group, key in ((64, "group64"), (0, "per_tensor_same_kernel")):
        Y = pq.groupwise_fwd(X, W, 1.0, group=group)
        fn = lambda: pq.groupwise_fwd(X, W, 1.0, group=group, Y=Y)
        ms = _time_steps(torch, fn, steps, warmup)
        prof = _profile_steps(pq, torch, fn, steps)
        gemm = prof.get("gemm_onebit_fwd")
        out[key] = {"call_us": round(1e3 * ms, 1), "gemm_us": round(1e3 * gemm[0] / gemm[1], 1) if gemm else None}
    g, p = out["group64"]["gemm_us"], out["per_tensor_same_kernel"]["gemm_us"]
    out["gemm_ratio_group_over_per_tensor"] = round(g / p, 2) if g and p else None
    out["scale_bytes_per_weight_bit"] = {"group64": 16 / 64, "per_tensor": 0.0}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--tokens", type=int, default=8192)
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="counter run for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE: the default workload, batch-1 and batch-8 "
                         "decode, and a 256 MiB copy kernel of known size that scales the byte counters; nothing else")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-ffn", action="store_true")
    ap.add_argument("--no-stack", action="store_true")
    ap.add_argument("--no-norm", action="store_true")
    ap.add_argument("--no-hp8", action="store_true")
    ap.add_argument("--no-fp32-io", action="store_true", help="skip the fp32 I/O step at the config-2 shape (fp64 matrix instructions)")
    ap.add_argument("--no-groupwise", action="store_true", help="skip the group-wise(64) scale contrast (Sec. 4.6)")
    ap.add_argument("--no-vendor-context", action="store_true", help="skip the vendor-library GEMM timings (context only)")
    ap.add_argument("--no-paper-ffn", action="store_true", help="skip the paper-exact 1.3B FFN (Table 1) and its branch sweep")
    ap.add_argument("--no-decode-layer-sweep", action="store_true",
                    help="skip batch-1 decode at 128 and 256 weight sets per launch (shows the rate does not lean on the last-level cache)")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="no GPU work: turn two rocprofv3 --pmc counter CSVs of a --calibrate run into profiles/hbm_traffic.json")
    args = ap.parse_args()
    if args.traffic_from:
        write_traffic(*args.traffic_from)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_22592_amd import binding as pq
    from paper_2602_22592_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if not os.path.exists(pq.LIB_PATH):
        from paper_2602_22592_amd.build import build
        build(verbose=False)

    # The sections next to the headline step; one of them failing must not cost the line its headline numbers, so a
    # failure is recorded in its place (and on stderr) instead of propagating.
    extra = {}

    def section(key, fn):
        try:
            extra[key] = fn()
        except Exception as exc:                      # noqa: BLE001
            extra[key] = {"error": f"{type(exc).__name__}: {exc}"}
            print(f"bench.py: section {key} failed: {exc!r}", file=sys.stderr, flush=True)

    # The bandwidth-bound sections run first: straight after 0.15 s of back-to-back MFMA work the same kernels read
    # 8-10 % slower (the chip's power management), which says nothing about them.
    if args.calibrate:
        # a counter run: only the workloads whose kernels are looked up in the counter files, so that a kernel name
        # stands for one workload (the INT8-expert decode variants and the FFN stack launch the same kernels on other sizes)
        args.no_ffn = args.no_stack = args.no_hp8 = args.no_paper_ffn = args.no_cpu_baseline = True
        section("decode_gemv", lambda: {"B1": decode_bench(pq, torch, 1), "B8": decode_bench(pq, torch, 8)})
    elif not args.no_decode:
        section("decode_gemv", lambda: {"metric": "1-bit decode GEMV HBM GB/s (4096->11008, E=8 top-2 r=64 experts)",
                                        "B1": decode_bench(pq, torch, 1), "B8": decode_bench(pq, torch, 8),
                                        "B1_int8_experts": decode_bench(pq, torch, 1, int8_experts=True),
                                        "B8_int8_experts": decode_bench(pq, torch, 8, int8_experts=True)})
        if not args.no_decode_layer_sweep:
            section("decode_layer_sweep", lambda: {str(n): decode_bench(pq, torch, 1, n_layers=n, steps=50, warmup=10)
                                                   for n in (128, 256)})
        section("decode_ffn", lambda: decode_ffn_bench(pq, torch))
        section("decode_ffn_B8", lambda: decode_ffn_bench(pq, torch, batch=8))
    if not args.no_norm:
        section("rmsnorm_quant", lambda: norm_quant_bench(pq, torch))
    torch.cuda.empty_cache()

    c = wl.config2(tokens=args.tokens)
    T, K, N, r = c["tokens"], c["d_in"], c["d_out"], c["hp_rank"]
    bf = torch.bfloat16
    to = lambda x: torch.from_numpy(x).cuda().to(bf)
    X, W, dY, A, B = to(c["X"]), to(c["W"]), to(c["dY"]), to(c["A"]), to(c["B"])
    desc = pq.make_desc(T, K, N, hp_rank=r, io_dtype=pq.PQ_BF16, alpha=c["alpha"], beta=c["beta"])
    bufs = pq.LinearBuffers(desc)
    Y = torch.empty((T, N), dtype=bf, device="cuda")
    dX = torch.empty((T, K), dtype=bf, device="cuda")
    dW = torch.empty((N, K), dtype=torch.float32, device="cuda")
    dA = torch.empty((r, K), dtype=torch.float32, device="cuda")
    dB = torch.empty((N, r), dtype=torch.float32, device="cuda")
    dab = torch.empty((2,), dtype=torch.float32, device="cuda")

    def step():
        pq.linear_fwd(desc, X, W, Y, bufs, A=A, B=B)
        pq.linear_bwd(desc, dY, X, W, bufs, dX, dW, dab, A=A, B=B, dA=dA, dB=dB)

    # The clocks of a GPU that has just run bandwidth-bound work (or none) take some tens of milliseconds of matrix work
    # to settle: the same step is run back to back for `PREWARM_S` first, so that short timed regions (a handful of
    # steps is 2 ms) measure the kernels and not that ramp.  Then the contract: `warmup` untimed steps, and exactly
    # `steps` steps between synchronisations, no per-launch events.
    _warm(torch, step, PREWARM_S)
    ms_per_step = _time_steps(torch, step, args.steps, args.warmup)
    # per-kernel durations: the same `steps` steps again with the library's HIP events around every launch (on the
    # launch stream); those events open gaps between launches, which is why they stay out of the timed region
    prof = _profile_steps(pq, torch, step, args.steps)

    kernels = {k: {"avg_us": 1e3 * ms / n, "launches": n} for k, (ms, n) in prof.items()}
    fl = gemm_flops(T, K, N, r)
    dom = max((k for k in kernels if k in fl), key=lambda k: kernels[k]["avg_us"] * kernels[k]["launches"])
    is_i8 = dom == "gemm_onebit_fwd"
    # the rank-r product dH A runs inside the dX launch (a second contraction into the same tile) when no launch carries
    # the gemm_dX_hp label: its flops are part of that launch's algorithmic work
    dom_flops = fl[dom] + (fl["gemm_dX_hp"] if dom == "gemm_dX" and "gemm_dX_hp" not in kernels and r > 0 else 0.0)
    achieved = dom_flops / (kernels[dom]["avg_us"] * 1e-6) / 1e12
    peak = (PEAK_I8 if is_i8 else PEAK_BF16) / 1e12
    # HBM traffic of that kernel per launch: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch) scaled by what
    # the same counters read for a 256 MiB copy of known size (`--calibrate`), see profiles/; keyed by GEMM label
    # at the default workload, null for anything that was not profiled
    traffic = load_traffic().get(dom) if (T, K, N, r) == (8192, 2048, 2048, 128) else None
    roofline = {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 2), "peak": peak,
                "unit": "TOP/s" if is_i8 else "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": traffic,
                "avg_us": round(kernels[dom]["avg_us"], 2)}
    # whole-step MFMA utilisation: int8 ops at the int8 peak + bf16 flops at the bf16 peak
    t_mfma = fl["gemm_onebit_fwd"] / PEAK_I8 + sum(v for k, v in fl.items() if k != "gemm_onebit_fwd") / PEAK_BF16
    out = {
        "metric": "decoupled-linear fwd+bwd tokens/s", "value": round(T / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "prewarm_s": PREWARM_S,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8 (1-bit branch fwd) + bf16 (hp branch, backward), fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"1.3B-shaped attention projection: tokens={T}, d_in=d_out={K}, hp rank {r}, "
                               "bf16 master weights, fwd + STE bwd (dX, dW, dA, dB, dalpha, dbeta)"},
        "mfma_frac_of_step": round(t_mfma / (ms_per_step * 1e-3), 4),
        "roofline": roofline,
        "kernels_us": {k: round(v["avg_us"], 2) for k, v in sorted(kernels.items())},
    }
    if args.calibrate:
        # a plain copy of known size through the library's row-gather kernel (identity indices), so that a
        # rocprofv3 --pmc run of this command carries its own scale for FETCH_SIZE / WRITE_SIZE
        rows, cols = 65536, 2048
        src = torch.randn((rows, cols), device="cuda").to(bf)
        dst = torch.empty_like(src)
        ids = torch.arange(rows, dtype=torch.int32, device="cuda")
        for _ in range(3):
            pq.glue_gather_rows(src, ids, dst)
        torch.cuda.synchronize()
        out["calibration_copy"] = {"kernel": "gather_rows_kernel", "read_bytes": rows * cols * 2 + rows * 4,
                                   "write_bytes": rows * cols * 2}
        del src, dst, ids
    if not args.no_vendor_context and not args.calibrate:
        section("vendor_gemm_context", lambda: vendor_gemm_context(torch, X, W, dY))
    if not args.calibrate and not args.no_groupwise:
        section("groupwise_contrast", lambda: groupwise_contrast(pq, torch, X, W))
    if not args.no_hp8:
        section("hp_int8_branch", lambda: hp_int8_bench(pq, torch))
    if not args.no_fp32_io and not args.calibrate:
        section("fp32_io_config2_shape", lambda: fp32_io_bench(pq, torch, c))
    if not args.no_ffn:
        section("ffn_config3", lambda: ffn_bench(pq, torch))
        # the same FFN with its experts in the INT8 form of the FFN equation (Sec. 3.2)
        section("ffn_config3_int8_experts", lambda: ffn_bench(pq, torch, int8_experts=True))
    if not args.no_paper_ffn:
        # Table 1's 1.3B model: D_model 2048, D_ff - r = 5076 one-bit hidden units, r = 384 per high-precision branch;
        # Sec. 4.4 / App. D scale the number of branches N (one active per token)
        section("ffn_paper_1p3b", lambda: {f"N{n}": ffn_bench(pq, torch, F=5076, E=n, r=384, steps=10, warmup=3) for n in (1, 2, 4, 8)})
        section("ffn_paper_1p3b_int8_experts", lambda: {f"N{n}": ffn_bench(pq, torch, F=5076, E=n, r=384, steps=10, warmup=3, int8_experts=True)
                                                         for n in (1, 8)})
    if not args.no_stack:
        del X, W, dY, A, B, Y, dX, dW, bufs
        torch.cuda.empty_cache()
        section("stack_config5", lambda: stack_bench(pq, torch))
    if not args.no_cpu_baseline:
        section("cpu_baseline", lambda: cpu_baseline(args.cpu_sample_tokens))
    out.update(extra)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
