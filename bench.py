#!/usr/bin/env python3
"""Benchmark of the variance-based gradient compression hot path on one MI355X.

Workload (default): the flat 1e9-parameter fp32 stream (Student-t(3) per-sample gradients,
batch 16, squared sums precomputed), 8 simulated workers on the one GPU, groups of 2^24,
alpha 1, zeta 0.999.  One step = one training iteration's compression work for all workers:
for each worker vgc_accumulate_select + vgc_pack on its (r, v) state, then the dense buffer is
overwritten with the sum of the 8 decoded messages (vgc_unpack_add_batch; `--decode per-message`
clears it and calls vgc_unpack_add once per message instead).  Inputs (g, s for
every worker and step) are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` = parameters compressed per second (workers x N x steps / time).
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--n", type=int, default=1_000_000_000, help="parameters per worker")
    ap.add_argument("--workers", type=int, default=8)
    ap.add_argument("--alpha", type=float, default=1.0)
    ap.add_argument("--decode", choices=["batch", "per-message"], default="batch",
                    help="batch: all messages in one pass over the dense buffer; per-message: one launch each")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sqgrad", action="store_true")
    ap.add_argument("--core-only", action="store_true",
                    help="only the timed steps of the flat workload (what the kernel-trace summary under profiles/ is taken with: "
                         "every launch then has the benchmark's size)")
    ap.add_argument("--cpu-sample", type=int, default=1 << 27, help="upper bound on the parameters of the oracle-timed sample")
    return ap.parse_args()


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1802_06058_amd import vgc, workloads as W

    if not os.path.exists(vgc.LIB_PATH):
        from paper_1802_06058_amd import build
        build.build()
    vgc.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg = W.CONFIGS["C5"]
    N, P = a.n, a.workers
    zeta, batch, nu = cfg["zeta"], cfg["batch"], cfg["nu"]
    groups = W.flat_groups(N, cfg["group"])
    plan = vgc.Plan(groups, dev)

    # ---- inputs: a pool of P (g, s) pairs; worker w uses pair (w + step) % P at a step, so no worker
    # sees a pair twice within P steps and every pair is resident before timing starts
    t0 = time.time()
    pool = [student_stream(W, N, batch, nu, cfg["seed"] + 1000 * i, dev) for i in range(P)]
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    r = [torch.zeros(N, dtype=torch.float32, device=dev) for _ in range(P)]
    v = [torch.zeros(N, dtype=torch.float32, device=dev) for _ in range(P)]
    scratch = plan.new_scratch()
    cap = N
    words = [torch.empty(cap, dtype=torch.int32, device=dev) for _ in range(P)]
    hdrs = [plan.new_headers() for _ in range(P)]
    status = [plan.new_status() for _ in range(P)]
    dense = torch.zeros(N, dtype=torch.float32, device=dev)
    scale = 1.0 / P

    ev = lambda: torch.cuda.Event(enable_timing=True)
    sel_ms, pack_ms, dec_ms, sent_words = [], [], [], []

    def step(k, record):
        marks = []
        for w in range(P):
            g, s = pool[(w + k) % P]
            e0, e1, e2 = ev(), ev(), ev()
            e0.record()
            vgc.accumulate_select(g, s, r[w], v[w], plan, a.alpha, zeta, scratch)
            e1.record()
            vgc.pack(plan, scratch, words[w], hdrs[w], status[w])
            e2.record()
            marks.append((e0, e1, e2))
        torch.cuda.synchronize()                       # a receiver learns the message sizes from the transfer
        counts = [vgc.read_status(status[w]) for w in range(P)]
        d0, d1 = ev(), ev()
        d0.record()
        if a.decode == "batch":
            vgc.unpack_add_batch(words, [c[0] for c in counts], hdrs, plan, scale, dense, overwrite=True)
        else:
            dense.zero_()
            for w in range(P):
                vgc.unpack_add(words[w], counts[w][0], hdrs[w], plan, scale, dense)
        d1.record()
        if record:
            torch.cuda.synchronize()
            for e0, e1, e2 in marks:
                sel_ms.append(e0.elapsed_time(e1))
                pack_ms.append(e1.elapsed_time(e2))
            dec_ms.append(d0.elapsed_time(d1))
            sent_words.append([c[0] for c in counts])
            assert not any(c[1] for c in counts), "word buffer overflow"

    for k in range(a.warmup):
        step(k, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(a.warmup, a.warmup + a.steps):
        step(k, True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms_per_step = elapsed * 1e3 / a.steps
    value = P * N * a.steps / elapsed / 1e9
    rho = float(np.mean(sent_words)) / N
    sel = float(np.mean(sel_ms))
    pk = float(np.mean(pack_ms))
    dec = float(np.mean(dec_ms))
    sel_gbs = 24.0 * N / (sel * 1e-3) / 1e9
    sp_gbs = (24.0 + 4.0 * rho) * N / ((sel + pk) * 1e-3) / 1e9
    dec_gbs = 12.0 * rho * N * P / (dec * 1e-3) / 1e9

    traffic, traffic_source = measured_traffic(N)
    out = {
        "metric": "compressed params/sec", "value": round(value, 3), "unit": "Gparams/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "C5: flat 1e9-param fp32 stream, Student-t(3) per-sample gradients, batch 16, "
                               "8 simulated workers, groups of 2^24, alpha 1, zeta 0.999",
                   "n_params_per_worker": N, "workers": P, "alpha": a.alpha, "zeta": zeta,
                   "n_groups": len(groups), "tile": vgc.tile_size(), "sent_fraction": round(rho, 5)},
        "roofline": {"bound": "hbm", "kernel": "k_accumulate_select", "achieved": round(sel_gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(sel_gbs / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": 24.0 * N, "avg_launch_ms": round(sel, 4),
                     "median_launch_ms": round(float(np.median(sel_ms)), 4), "min_launch_ms": round(float(np.min(sel_ms)), 4),
                     "launches": len(sel_ms)},
        "stages": {
            "select_ms": round(sel, 4), "pack_ms": round(pk, 4), "decode_all_workers_ms": round(dec, 4),
            "select_plus_pack": {"algorithmic_GBs": round(sp_gbs, 1), "frac_of_peak": round(sp_gbs / HBM_PEAK_GBS, 4),
                                 "bytes_per_param": round(24.0 + 4.0 * rho, 3),
                                 "Gparams_per_s": round(N / ((sel + pk) * 1e-3) / 1e9, 2)},
            "decode": {"algorithmic_GBs": round(dec_gbs, 1), "frac_of_peak": round(dec_gbs / HBM_PEAK_GBS, 4),
                       "bytes_per_word": 12, "mode": a.decode},
        },
        "input_generation_s": round(gen_s, 1),
    }

    if a.core_only:
        print(json.dumps(out))
        return

    # the compressed index format on worker 0's next message (steady state: its state after the timed steps)
    out["stages"]["compressed_indexes"] = bench_compact(vgc, plan, pool, r[0], v[0], a.alpha, zeta, scratch, words, hdrs, status, dense, N, P, scale)

    # hybrid algorithm (Alg. 2): same kernels with the threshold rule, tau = 0.05, on every worker's buffers from a
    # fresh state, queued like the timed steps above (the time of a select call moves by several per cent with where
    # its six arrays lie relative to each other, so one worker's buffers alone would measure their placement)
    for w in range(P):
        r[w].zero_(); v[w].zero_()
    hy_marks, hy_status = [], [plan.new_status() for _ in range(3 * P)]
    hy_buf, hy_hdrs = torch.empty(cap, dtype=torch.int32, device=dev), plan.new_headers()   # (the Alg. 1 messages stay for the stages below)
    for k in range(3):
        for w in range(P):
            g, s = pool[(w + k) % P]
            e0, e1 = ev(), ev()
            e0.record()
            vgc.accumulate_select_hybrid(g, s, r[w], v[w], plan, 2.0, zeta, 0.05, scratch)
            vgc.pack(plan, scratch, hy_buf, hy_hdrs, hy_status[k * P + w])
            e1.record()
            hy_marks.append((e0, e1))
        torch.cuda.synchronize()
    hy_ms = [e0.elapsed_time(e1) for e0, e1 in hy_marks[P:]]
    hy_words = [vgc.read_status(x)[0] for x in hy_status[P:]]
    hy, hrho = float(np.mean(hy_ms)), float(np.mean(hy_words)) / N
    del hy_buf
    out["stages"]["hybrid_select_plus_pack"] = {
        "alpha": 2.0, "tau": 0.05, "ms": round(hy, 4), "sent_fraction": round(hrho, 5),
        "algorithmic_GBs": round((24.0 + 4.0 * hrho) * N / (hy * 1e-3) / 1e9, 1),
        "frac_of_peak": round((24.0 + 4.0 * hrho) * N / (hy * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    # decode fused with the parameter update: the last step's 8 messages, one Momentum SGD / Adam step on N parameters
    out["stages"]["decode_plus_update"] = bench_update(vgc, plan, words, hdrs, status, dense, N, P, scale)

    # the sparse regime, one worker of the flat workload on a fresh state
    out["stages"]["sparse_regime_fresh_state"] = alpha_sweep(vgc, plan, pool[0][0], pool[0][1], r[0], v[0], zeta, scratch,
                                                             words[0], hdrs[0], status[0], (8.0, 16.0), dense=dense)
    out["stages"]["model_parameter_sets"] = bench_model_sets(dev, a.alpha, zeta)
    out["stages"]["fused_fc_statistic_select"] = bench_fused_fc(dev, zeta)
    if not a.no_sqgrad:
        out["stages"]["sqgrad"] = bench_sqgrad(dev)
        out["stages"]["vgg16_iteration"] = bench_vgg_iteration(dev, zeta)
        out["stages"]["resnet50_iteration"] = bench_resnet_iteration(dev, zeta)
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(pool[0], a, cfg, min(a.cpu_sample, N))
    print(json.dumps(out))


def bench_compact(vgc, plan, pool, r, v, alpha, zeta, scratch, words, hdrs, status, dense, N, P, scale):
    """The compressed index format on the flat workload: worker 0's steady-state message (its state after the timed
    steps) packed both ways, sizes compared; then P copies of that message decoded in one pass, plain against compact."""
    import torch
    dev = dense.device
    g, s = pool[0]
    vgc.accumulate_select(g, s, r, v, plan, alpha, zeta, scratch)
    stream = torch.empty(N, dtype=torch.uint8, device=dev)
    tile_bytes = torch.empty(plan.n_tiles, dtype=torch.int16, device=dev)
    run_offsets = torch.empty(plan.n_runs, dtype=torch.int64, device=dev)
    chdrs, cstatus = plan.new_headers(), plan.new_status()
    t_plain = _timed(lambda: vgc.pack(plan, scratch, words[0], hdrs[0], status[0]), 30.0, 60.0)
    t_comp = _timed(lambda: vgc.pack_compact(plan, scratch, stream, tile_bytes, run_offsets, chdrs, cstatus), 30.0, 60.0)
    n_words, n_bytes = vgc.read_status(status[0])[0], vgc.read_status(cstatus)[0]
    plain_bytes = 4.0 * n_words + 16.0 * plan.n_groups
    comp_bytes = n_bytes + 2.0 * plan.n_tiles + 8.0 * plan.n_runs + 16.0 * plan.n_groups
    t_dp = _timed(lambda: vgc.unpack_add_batch([words[0]] * P, [n_words] * P, [hdrs[0]] * P, plan, scale, dense, overwrite=True), 30.0, 60.0)
    t_dc = _timed(lambda: vgc.unpack_compact_add_batch([stream] * P, [n_bytes] * P, [tile_bytes] * P, [run_offsets] * P, [chdrs] * P,
                                                      plan, scale, dense, overwrite=True), 30.0, 60.0)
    return {"sent_fraction": round(n_words / N, 5), "plain_message_bytes": plain_bytes, "compact_message_bytes": comp_bytes,
            "size_ratio": round(plain_bytes / comp_bytes, 3), "bits_per_element_compact": round(8.0 * comp_bytes / max(n_words, 1), 3),
            "pack_plain_ms": round(t_plain, 4), "pack_compact_ms": round(t_comp, 4),
            "decode_plain_ms": round(t_dp, 4), "decode_compact_ms": round(t_dc, 4), "messages_decoded": P}


def student_stream(W, n, batch, nu, seed, device, chunk=1 << 24):
    """The flat workload's inputs ("squared sums precomputed"): per parameter `batch` Student-t(nu) per-sample
    gradients y_z from a seeded generator on the device, reduced to the two inputs of a step,
    g = sum_z y_z / batch and s = sum_z (y_z / batch)^2.  Not timed."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    g = torch.empty(n, dtype=torch.float32, device=device)
    s = torch.empty(n, dtype=torch.float32, device=device)
    for lo in range(0, n, chunk):
        m = min(chunk, n - lo)
        gacc = torch.zeros(m, dtype=torch.float32, device=device)
        sacc = torch.zeros(m, dtype=torch.float32, device=device)
        for _ in range(batch):
            y = W.device_student_draw(m, nu, gen, device) / batch
            gacc += y
            sacc += y * y
        g[lo:lo + m] = gacc
        s[lo:lo + m] = sacc
    return g, s


def bench_update(vgc, plan, words, hdrs, status, param, N, P, scale):
    """vgc_unpack_apply on the messages left by the last timed step.  Algorithmic bytes: parameters and optimizer
    state read and written once (16 B per parameter for Momentum SGD, 24 for Adam) + 4 B per word."""
    import torch
    counts = [vgc.read_status(status[w])[0] for w in range(P)]
    n_words = float(sum(counts))
    res = {}
    m = torch.zeros_like(param)
    v = torch.zeros_like(param)
    for name, kind, per_param in (("momentum_sgd", vgc.MOMENTUM_SGD, 16.0), ("adam", vgc.ADAM, 24.0)):
        ms = []
        for k in range(4):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            vgc.unpack_apply(words, counts, hdrs, plan, scale, param, m, v if kind == vgc.ADAM else None, kind=kind,
                             lr=1e-3, momentum=0.9, step=k + 1)
            e1.record(); torch.cuda.synchronize()
            if k:
                ms.append(e0.elapsed_time(e1))
        t = float(np.mean(ms))
        gbs = (per_param * N + 4.0 * n_words) / (t * 1e-3) / 1e9
        res[name] = {"ms": round(t, 4), "algorithmic_GBs": round(gbs, 1), "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4),
                     "bytes_per_param": per_param, "messages": P}
    del m, v
    return res


def measured_traffic(N):
    """(HBM bytes per k_accumulate_select launch, where the figure comes from) from the committed counter runs
    (profiles/), which were taken at N = 1e9 and a sent fraction of about 0.2; (None, None) for any other size."""
    path = os.path.join(ROOT, "profiles", "traffic_c5_microbench_pmc.txt")
    if N != 1_000_000_000 or not os.path.exists(path):
        return None, None
    traffic, taken = None, None
    for line in open(path):
        if line.startswith("# taken:"):
            taken = line.split(":", 1)[1].strip()
        if line.startswith("k_accumulate_select_traffic_bytes_per_launch_n1e9:"):
            traffic = float(line.split(":")[1])
    return traffic, {"file": "profiles/traffic_c5_microbench_pmc.txt", "taken": taken}


def bench_model_sets(dev, alpha, zeta):
    """select + pack on the ResNet-50-shaped (161 groups, 25.6 M) and VGG-16-shaped (32 groups, 138 M)
    parameter sets: many groups of very different sizes in one launch."""
    import torch
    from paper_1802_06058_amd import vgc, workloads as W
    res = {}
    for name in ("C3", "C4"):
        cfg = W.CONFIGS[name]
        layers = cfg["layers"]
        plan = vgc.Plan(W.groups_from_sizes([L["size"] for L in layers]), dev)
        n, B = plan.n, cfg["batch"]
        sig = torch.from_numpy(np.repeat(W.layer_sigmas(cfg["seed"], len(layers)), [L["size"] for L in layers]).astype(np.float32)).to(dev)
        gen = torch.Generator(device=dev); gen.manual_seed(3)
        r = torch.zeros(n, dtype=torch.float32, device=dev); v = torch.zeros(n, dtype=torch.float32, device=dev)
        scratch, hdrs, status = plan.new_scratch(), plan.new_headers(), plan.new_status()
        words = torch.empty(n, dtype=torch.int32, device=dev)
        ms, sent = [], []
        for k in range(6):
            z = torch.randn(n, generator=gen, device=dev)
            chi = torch.zeros(n, device=dev)
            for _ in range(B - 1):
                w = torch.randn(n, generator=gen, device=dev); chi += w * w
            g = sig * z / B ** 0.5
            s = sig * sig * (chi + z * z) / (B * B)
            del z, chi
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            vgc.accumulate_select(g, s, r, v, plan, alpha, zeta, scratch)
            vgc.pack(plan, scratch, words, hdrs, status)
            e1.record(); torch.cuda.synchronize()
            if k:
                ms.append(e0.elapsed_time(e1)); sent.append(vgc.read_status(status)[0])
        t, rho = float(np.mean(ms)), float(np.mean(sent)) / n
        res[name] = {"n_params": n, "n_groups": plan.n_groups, "select_plus_pack_ms": round(t, 4),
                     "sent_fraction": round(rho, 4), "Gparams_per_s": round(n / (t * 1e-3) / 1e9, 1),
                     "algorithmic_GBs": round((24 + 4 * rho) * n / (t * 1e-3) / 1e9, 1),
                     "frac_of_peak": round((24 + 4 * rho) * n / (t * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        if name == "C4":
            # the last (g, s) on a fresh state, across alpha: from half of the elements sent down to the
            # sparse regime the method is meant for
            res[name]["alpha_sweep_fresh_state"] = alpha_sweep(vgc, plan, g, s, r, v, zeta, scratch, words, hdrs, status,
                                                               (0.5, 1.0, 2.0, 4.0, 8.0, 16.0))
    return res


def bench_fused_fc(dev, zeta):
    """The two large FC layers of the VGG-16-shaped configuration (bf16, batch 64): statistic + accumulate pass as two
    calls (vgc_sqgrad writes g and s, vgc_accumulate_select reads them back: 32 bytes per parameter) against the fused
    call (vgc_sqgrad_accumulate_select: g and s stay on chip, 16 bytes per parameter: r and v read and written).  Both
    are followed by the same vgc_pack, not timed here."""
    import torch
    from paper_1802_06058_amd import vgc, workloads as W
    res = {}
    for name, B, J, C in (("vgg_fc6_25088x4096_B64_bf16", 64, 25088, 4096), ("vgg_fc7_4096x4096_B64_bf16", 64, 4096, 4096)):
        plan = vgc.Plan(W.groups_from_sizes([J * C]), dev)
        n = plan.n
        gen = torch.Generator(device=dev); gen.manual_seed(2)
        X = torch.randn((B, J), generator=gen, device=dev).to(torch.bfloat16)
        D = (torch.randn((B, C), generator=gen, device=dev) * 1e-3).to(torch.bfloat16)
        r = torch.zeros(n, device=dev); v = torch.zeros(n, device=dev)
        g = torch.empty(J, C, device=dev); s = torch.empty(J, C, device=dev)
        scratch, hdrs, status = plan.new_scratch(), plan.new_headers(), plan.new_status()
        words = torch.empty(n, dtype=torch.int32, device=dev)
        ws = torch.empty(vgc.sqgrad_accumulate_select_workspace_bytes(vgc.BF16, B, J, C), dtype=torch.uint8, device=dev)

        def two_calls():
            vgc.sqgrad(vgc.FC, X, D, 1.0 / B, s, g)
            vgc.accumulate_select(g.view(-1), s.view(-1), r, v, plan, 1.0, zeta, scratch)

        def fused():
            vgc.sqgrad_accumulate_select(X, D, 1.0 / B, r, v, plan, 0, 1.0, zeta, scratch, ws)
        t2 = _timed(two_calls, 60.0, 60.0)
        tf = _timed(fused, 60.0, 60.0)
        vgc.pack(plan, scratch, words, hdrs, status)
        torch.cuda.synchronize()
        rho = vgc.read_status(status)[0] / n
        res[name] = {"two_calls_ms": round(t2, 4), "two_calls_GBs_32B_per_param": round(32.0 * n / t2 / 1e6, 1),
                     "fused_ms": round(tf, 4), "fused_GBs_16B_per_param": round(16.0 * n / tf / 1e6, 1),
                     "fused_frac_of_peak": round(16.0 * n / tf / 1e6 / HBM_PEAK_GBS, 4), "speedup": round(t2 / tf, 3),
                     "sent_fraction_steady_state": round(rho, 4)}
        del X, D, r, v, g, s, scratch, words, ws
    return res


def alpha_sweep(vgc, plan, g, s, r, v, zeta, scratch, words, hdrs, status, alphas, dense=None):
    """select + pack on state (r, v) = 0 for each alpha (three repetitions, state cleared before each).  With a
    dense buffer, the message of each alpha is also decoded into it (vgc_unpack_add).  A sparse message touches
    one element per memory transaction, so next to the algorithmic 12 bytes per word (word read, target read and
    written) the decode rate is also given with whole 64-byte transactions for the target: 4 + 2 x 64 bytes per
    word; the fraction of peak uses the algorithmic figure."""
    import torch
    n, res = plan.n, {}
    for alpha in alphas:
        ms = []
        for _ in range(3):
            r.zero_(); v.zero_()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            vgc.accumulate_select(g, s, r, v, plan, alpha, zeta, scratch)
            vgc.pack(plan, scratch, words, hdrs, status)
            e1.record(); torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1))
        n_words = vgc.read_status(status)[0]
        t, rho = min(ms[1:]), n_words / n
        res[str(alpha)] = {"ms": round(t, 4), "sent_fraction": float(f"{rho:.3g}"),
                           "frac_of_peak": round((24 + 4 * rho) * n / (t * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        if dense is not None:
            td = _timed(lambda: vgc.unpack_add(words, n_words, hdrs, plan, 1.0, dense), warm_ms=20.0, timed_ms=40.0)
            res[str(alpha)]["decode"] = {
                "ms": round(td, 4), "words": n_words,
                "algorithmic_GBs_12B_per_word": round(12.0 * n_words / (td * 1e-3) / 1e9, 1),
                "frac_of_peak": round(12.0 * n_words / (td * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "transaction_GBs_132B_per_word": round(132.0 * n_words / (td * 1e-3) / 1e9, 1),
                "transaction_bytes": 64}
    return res


def bench_sqgrad(dev):
    """Part (a) on layer shapes of the VGG-16 (bf16, batch 64) and ResNet-50 (float32, batch 32)
    configurations.  FC layers are bound by writing [J, C] floats (HBM roofline); conv layers by the
    matrix cores (bf16 peak 2500 TFLOP/s, float32 peak 157.3 TFLOP/s).  s alone and g + s are timed."""
    import torch
    from paper_1802_06058_amd import vgc
    res = {}
    shapes = [("vgg_fc6_25088x4096_B64_bf16", vgc.FC, torch.bfloat16, 64, 1, 25088, 4096),
              ("vgg_conv4_2_P784_4608x512_B64_bf16", vgc.CONV, torch.bfloat16, 64, 784, 4608, 512),
              ("vgg_conv3_2_P3136_2304x256_B64_bf16", vgc.CONV, torch.bfloat16, 64, 3136, 2304, 256),
              ("resnet_s3_conv2_P196_2304x256_B32_f32", vgc.CONV, torch.float32, 32, 196, 2304, 256),
              ("resnet_fc_2048x1000_B32_f32", vgc.FC, torch.float32, 32, 1, 2048, 1000)]
    for name, kind, dt, B, P, J, C in shapes:
        gen = torch.Generator(device=dev); gen.manual_seed(1)
        shp_x = (B, J) if kind == vgc.FC else (B, P, J)
        shp_d = (B, C) if kind == vgc.FC else (B, P, C)
        X = torch.randn(shp_x, generator=gen, device=dev, dtype=torch.float32).to(dt)
        D = (torch.randn(shp_d, generator=gen, device=dev, dtype=torch.float32) * 1e-3).to(dt)
        g = torch.empty(J, C, dtype=torch.float32, device=dev)
        s = torch.empty(J, C, dtype=torch.float32, device=dev)
        nb = vgc.sqgrad_workspace_bytes(kind, vgc.BF16 if dt == torch.bfloat16 else vgc.F32, B, P, J, C)
        ws = torch.empty(nb, dtype=torch.uint8, device=dev) if nb else None
        peak = 2500.0 if dt == torch.bfloat16 else 157.3
        entry = {}
        for tag, gg in (("s_only", None), ("g_and_s", g)):
            ms = _timed(lambda: vgc.sqgrad(kind, X, D, 1.0 / B, s, gg, workspace=ws))
            chains = 2.0 if (kind == vgc.FC and gg is not None) else 1.0      # FC: one contraction per output array
            flops = chains * 2.0 * B * P * J * C
            out_bytes = (8.0 if gg is not None else 4.0) * J * C
            in_bytes = X.element_size() * B * P * (J + C)
            tf = flops / (ms * 1e-3) / 1e12
            entry[tag] = {"ms": round(ms, 4), "TFLOPs": round(tf, 1), "mfma_frac": round(tf / peak, 4),
                          "algorithmic_GBs": round((out_bytes + in_bytes) / (ms * 1e-3) / 1e9, 1),
                          "hbm_frac": round((out_bytes + in_bytes) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        entry["bound"] = "hbm" if kind == vgc.FC else "mfma"
        res[name] = entry
        del X, D, g, s, ws

    # the same two VGG convolutions from their NHWC inputs (no patch matrix): 1/9 of the input bytes
    for name, B, H, Cin, C in (("vgg_conv4_2_nhwc_28x28x512_to_512_B64_bf16", 64, 28, 512, 512),
                               ("vgg_conv3_2_nhwc_56x56x256_to_256_B64_bf16", 64, 56, 256, 256)):
        gen = torch.Generator(device=dev); gen.manual_seed(1)
        A = torch.randn((B, H, H, Cin), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        D = (torch.randn((B, H, H, C), generator=gen, device=dev, dtype=torch.float32) * 1e-3).to(torch.bfloat16)
        J = 9 * Cin
        g = torch.empty(J, C, dtype=torch.float32, device=dev)
        s = torch.empty(J, C, dtype=torch.float32, device=dev)
        nb = vgc.sqgrad_conv2d_workspace_bytes(vgc.BF16, B, H, H, Cin, C, 3, 3, (1, 1), (1, 1))
        ws = torch.empty(nb, dtype=torch.uint8, device=dev) if nb else None
        entry = {}
        for tag, gg in (("s_only", None), ("g_and_s", g)):
            ms = _timed(lambda: vgc.sqgrad_conv2d(A, D, 3, 3, (1, 1), (1, 1), 1.0 / B, s, gg, workspace=ws))
            tf = 2.0 * B * H * H * J * C / (ms * 1e-3) / 1e12
            io = 2.0 * B * H * H * (Cin + C) + (8.0 if gg is not None else 4.0) * J * C
            entry[tag] = {"ms": round(ms, 4), "TFLOPs": round(tf, 1), "mfma_frac": round(tf / 2500.0, 4),
                          "algorithmic_GBs": round(io / (ms * 1e-3) / 1e9, 1)}
        entry["bound"] = "mfma"
        res[name] = entry
        del A, D, g, s, ws
    return res


def _timed(fn, warm_ms=150.0, timed_ms=100.0):
    """Average duration of fn() in steady state: the matrix-core clock takes on the order of 100 ms of load to
    settle after idle (the same call measures up to 20 % slower in the first milliseconds), so fn is repeated for
    about warm_ms untimed and then for about timed_ms between two events."""
    import torch
    fn(); torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(); fn(); e1.record(); torch.cuda.synchronize()
    once = max(e0.elapsed_time(e1), 1e-3)
    for _ in range(min(2000, max(1, int(warm_ms / once)))):
        fn()
    reps = min(2000, max(3, int(timed_ms / once)))
    e0.record()
    for _ in range(reps):
        fn()
    e1.record(); torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def _statistic_of_layers(dev, dt, B, convs, fcs, counts=None):
    """s of every layer of a network: convolutions (cin, cout, input extent, kernel, stride, pad) from their NHWC
    inputs (a layer whose channel count is not a multiple of 16 bytes and whose kh kw Cin exceeds 160 would go through a
    patch matrix with columns padded to a multiple of 16 bytes; the two networks here have none), FC layers in the FC form.  counts[i] says how often layer i occurs in the network (its
    inputs are shared, every occurrence has outputs and a workspace of its own).  Each distinct layer is timed
    alone; then the calls of the whole network are timed in one sweep, on one stream, spread over four by the caller
    (the layers are independent, so kernels of different layers can fill each other's tails), and with the NHWC
    convolutions as one batch call on one stream (the library spreads them over streams of its own).
    Returns (per-layer list, sum of the layers' times x counts, conv flops, sweep ms on 1 stream, on 4 streams, with
    the batch call)."""
    import torch
    from paper_1802_06058_amd import vgc
    code = vgc.BF16 if dt == torch.bfloat16 else vgc.F32
    piece = 8 if dt == torch.bfloat16 else 4
    gen = torch.Generator(device=dev); gen.manual_seed(5)
    rnd = lambda *shape: torch.randn(shape, generator=gen, device=dev, dtype=torch.float32).to(dt)
    counts = list(counts) if counts is not None else [1] * (len(convs) + len(fcs))
    layers, calls, batch, others, t_stat, flops = [], [], [], [], 0.0, 0.0
    for (cin, cout, sp, k, st, pd), cnt in zip(convs, counts):
        so = (sp + 2 * pd - k) // st + 1
        D = rnd(B, so, so, cout) * 1e-3
        J = k * k * cin
        mine = []
        if cin % piece == 0 or J <= 160:                                # (a first layer on few channels has a kernel of its own)
            A = rnd(B, sp, sp, cin)
            nb = vgc.sqgrad_conv2d_workspace_bytes(code, B, sp, sp, cin, cout, k, k, (st, st), (pd, pd))
            for _ in range(cnt):
                s = torch.empty(J, cout, dtype=torch.float32, device=dev)
                ws = torch.empty(nb, dtype=torch.uint8, device=dev) if nb else None
                mine.append(lambda A=A, D=D, s=s, ws=ws, k=k, st=st, pd=pd:
                            vgc.sqgrad_conv2d(A, D, k, k, (st, st), (pd, pd), 1.0 / B, s, None, workspace=ws))
                batch.append(dict(act=A, D=D, kh=k, kw=k, stride=(st, st), pad=(pd, pd), c=1.0 / B, s_out=s, workspace=ws))
            form = "nhwc"
        else:
            Jp = (J + piece - 1) // piece * piece
            A = rnd(B, so * so, Jp)
            A[:, :, J:] = 0
            Dm = D.view(B, so * so, cout)
            nb = vgc.sqgrad_workspace_bytes(vgc.CONV, code, B, so * so, Jp, cout)
            for _ in range(cnt):
                s = torch.empty(Jp, cout, dtype=torch.float32, device=dev)
                ws = torch.empty(nb, dtype=torch.uint8, device=dev) if nb else None
                mine.append(lambda A=A, Dm=Dm, s=s, ws=ws: vgc.sqgrad(vgc.CONV, A, Dm, 1.0 / B, s, None, workspace=ws))
            others += mine
            form = "patches"
        ms = _timed(mine[0])
        fl = 2.0 * B * so * so * J * cout
        layers.append({"layer": f"conv{k}x{k}/{st} {cin}->{cout} @{sp}", "form": form, "count": cnt, "ms": round(ms, 4),
                       "TFLOPs": round(fl / ms / 1e9, 1)})
        t_stat += cnt * ms; flops += cnt * fl
        calls += mine
    for (fin, fout), cnt in zip(fcs, counts[len(convs):]):
        X, D = rnd(B, fin), rnd(B, fout) * 1e-3
        mine = []
        for _ in range(cnt):
            s = torch.empty(fin, fout, dtype=torch.float32, device=dev)
            mine.append(lambda X=X, D=D, s=s: vgc.sqgrad(vgc.FC, X, D, 1.0 / B, s, None))
        ms = _timed(mine[0])
        layers.append({"layer": f"fc {fin}x{fout}", "form": "fc", "count": cnt, "ms": round(ms, 4),
                       "GBs": round(4.0 * fin * fout / ms / 1e6, 1)})
        t_stat += cnt * ms
        calls += mine
        others += mine

    main = torch.cuda.current_stream()
    side = [torch.cuda.Stream() for _ in range(4)]
    def sweep_1():
        for c in calls:
            c()
    def sweep_4():
        start = torch.cuda.Event(); start.record(main)
        for st_ in side:
            st_.wait_event(start)
        for i, c in enumerate(calls):
            with torch.cuda.stream(side[i % 4]):
                c()
        for st_ in side:
            e = torch.cuda.Event(); e.record(st_); main.wait_event(e)
    def sweep_batch():                                     # the NHWC convolutions as one vgc_sqgrad_conv2d_batch call
        vgc.sqgrad_conv2d_batch(batch)
        for c in others:
            c()
    t1, t4, tb = _timed(sweep_1), _timed(sweep_4), _timed(sweep_batch)
    return layers, t_stat, flops, t1, t4, tb


def _select_pack_update(dev, cfg_name, B, zeta):
    """select + pack over a model's parameter set, then the decode of 8 such messages fused with a Momentum SGD step."""
    import torch
    from paper_1802_06058_amd import vgc, workloads as W
    cfg = W.CONFIGS[cfg_name]
    sizes = [L["size"] for L in cfg["layers"]]
    plan = vgc.Plan(W.groups_from_sizes(sizes), dev)
    n = plan.n
    gen = torch.Generator(device=dev); gen.manual_seed(6)
    sig = torch.from_numpy(np.repeat(W.layer_sigmas(cfg["seed"], len(sizes)), sizes).astype(np.float32)).to(dev)
    z = torch.randn(n, generator=gen, device=dev)
    chi = torch.zeros(n, device=dev)
    for _ in range(B - 1):
        w = torch.randn(n, generator=gen, device=dev); chi += w * w
    g = sig * z / B ** 0.5
    s = sig * sig * (chi + z * z) / (B * B)
    del z, chi, sig
    r = torch.zeros(n, dtype=torch.float32, device=dev); v = torch.zeros(n, dtype=torch.float32, device=dev)
    scratch, hdrs, status = plan.new_scratch(), plan.new_headers(), plan.new_status()
    words = torch.empty(n, dtype=torch.int32, device=dev)

    def select_pack():
        r.zero_(); v.zero_()
        vgc.accumulate_select(g, s, r, v, plan, 1.0, zeta, scratch)
        vgc.pack(plan, scratch, words, hdrs, status)
    t_sp = _timed(select_pack) - _timed(lambda: (r.zero_(), v.zero_()))
    total = vgc.read_status(status)[0]
    param, mom = torch.zeros(n, device=dev), torch.zeros(n, device=dev)
    t_up = _timed(lambda: vgc.unpack_apply([words] * 8, [total] * 8, [hdrs] * 8, plan, 0.125, param, mom,
                                           kind=vgc.MOMENTUM_SGD, lr=1e-3, momentum=0.9))
    return n, t_sp, total / n, t_up


def bench_vgg_iteration(dev, zeta):
    """One worker's whole compression step on the VGG-16-shaped configuration (C4: batch 64, bfloat16 activations):
    the statistic s of every layer (g comes from the framework's own backward pass and is synthetic here), select +
    pack over the 138 M parameters, the decode of 8 such messages fused with a Momentum SGD step."""
    import torch
    B = 64
    convs = [(cin, cout, sp, 3, 1, 1) for cin, cout, sp in
             [(3, 64, 224), (64, 64, 224), (64, 128, 112), (128, 128, 112), (128, 256, 56), (256, 256, 56), (256, 256, 56),
              (256, 512, 28), (512, 512, 28), (512, 512, 28), (512, 512, 14), (512, 512, 14), (512, 512, 14)]]
    layers, t_stat, flops, t1, t4, tb = _statistic_of_layers(dev, torch.bfloat16, B, convs, [(25088, 4096), (4096, 4096), (4096, 1000)])
    n, t_sp, rho, t_up = _select_pack_update(dev, "C4", B, zeta)
    return _iteration_entry(B, n, layers, t_stat, flops, t1, t4, tb, t_sp, rho, t_up)


def _iteration_entry(B, n, layers, t_stat, flops, t1, t4, tb, t_sp, rho, t_up):
    """total_ms takes the statistic the fastest way a training loop can issue it (one batch call, or its own streams)."""
    best = min(t1, t4, tb)
    return {"batch": B, "n_params": n, "statistic_sum_of_layers_ms": round(t_stat, 3),
            "statistic_sweep_1_stream_ms": round(t1, 3), "statistic_sweep_4_streams_ms": round(t4, 3),
            "statistic_batch_call_ms": round(tb, 3),
            "statistic_conv_TFLOPs": round(flops / 1e12, 3), "statistic_TFLOPs_per_s": round(flops / best / 1e9, 1),
            "select_plus_pack_ms": round(t_sp, 3),
            "sent_fraction": round(rho, 4), "decode8_plus_momentum_sgd_ms": round(t_up, 3),
            "total_ms": round(best + t_sp + t_up, 3), "layers": layers}


def bench_resnet_iteration(dev, zeta):
    """The same for the ResNet-50-shaped configuration (C3: batch 32, float32 activations); identical layers are
    timed alone once and issued as often as they occur in the sweeps."""
    import torch
    B = 32
    convs, count = [], []
    def add(spec, times=1):
        convs.append(spec); count.append(times)
    add((3, 64, 224, 7, 2, 3))
    cin, prev_sp = 64, 56
    for width, blocks, sp in [(64, 3, 56), (128, 4, 28), (256, 6, 14), (512, 3, 7)]:
        st = prev_sp // sp
        add((cin, width, prev_sp, 1, 1, 0)); add((width, width, prev_sp, 3, st, 1)); add((width, 4 * width, sp, 1, 1, 0))
        add((cin, 4 * width, prev_sp, 1, st, 0))
        add((4 * width, width, sp, 1, 1, 0), blocks - 1); add((width, width, sp, 3, 1, 1), blocks - 1)
        add((width, 4 * width, sp, 1, 1, 0), blocks - 1)
        cin, prev_sp = 4 * width, sp
    layers, t_stat, flops, t1, t4, tb = _statistic_of_layers(dev, torch.float32, B, convs, [(2048, 1000)], count + [1])
    n, t_sp, rho, t_up = _select_pack_update(dev, "C3", B, zeta)
    return _iteration_entry(B, n, layers, t_stat, flops, t1, t4, tb, t_sp, rho, t_up)


def cpu_baseline(pair, a, cfg, sample):
    """The oracle, as it stands, on the leading groups of worker 0's first step: accumulate/select
    + pack + decode of that message (NumPy, one thread).  Runs group after group (2^24 parameters
    each) until about 10 s of CPU time are spent or `sample` parameters are done."""
    from oracle import vgc_oracle as O
    from paper_1802_06058_amd import workloads as W
    gsz = cfg["group"]
    done, dt = 0, 0.0
    while done < sample and dt < 10.0:
        m = min(gsz, sample - done)
        g = pair[0][done:done + m].cpu().numpy()
        s = pair[1][done:done + m].cpu().numpy()
        groups = W.flat_groups(m, gsz)
        z = np.zeros(m, np.float32)
        t0 = time.perf_counter()
        r_acc, r_out, v_out, send = O.accumulate_select(g, s, z, z, a.alpha, cfg["zeta"])
        words, hdrs, _ = O.pack(r_acc, send, groups)
        dense = np.zeros(m, np.float32)
        O.unpack_add(words, hdrs, groups, 1.0 / a.workers, dense)
        dt += time.perf_counter() - t0
        done += m
    return {"value": round(done / dt / 1e9, 5), "unit": "Gparams/s", "cores": 1, "kind": "oracle",
            "sample": f"first {done} parameters of one worker, one step (select + pack + decode of its message), "
                      f"{dt:.1f} s; host has {os.cpu_count()} logical cores, NumPy element-wise code uses one"}


if __name__ == "__main__":
    main()
