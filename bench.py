#!/usr/bin/env python3
"""Benchmark of the V-step re-encoding path on one MI355X.

One "step" is one pass of the whole hot path over one weight matrix:
    dequantize(codes) -> T = W - alpha*G and selection of the top-k groups (one
    fused call) -> re-encode the selected groups -> dequantize(updated codes)
on the 1x16 configuration (Llama-2-7B q_proj shape, 4096 x 4096, group 8, one
codebook of 2^16 codewords, tau = 0.01 -> 20 971 groups re-encoded).

All inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

PEAK_MFMA_F16 = 2500.0   # TFLOP/s dense fp16/bf16 matrix-core peak of MI355X
PEAK_HBM = 8000.0        # GB/s
PEAK_F64 = 78.6          # TFLOP/s fp64 vector (256 CU x 4 SIMD x 16 lanes x 2 (fma) x 2.4 GHz)
PEAK_F32 = 157.3         # TFLOP/s fp32 vector


def measured_traffic(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` on `workload`, from the rocprofv3 FETCH_SIZE / WRITE_SIZE
    summary under profiles/ (a line 'traffic_bytes_per_launch <kernel> <bytes> commit <hash>'),
    or None when no summary of that workload has been taken."""
    f = ROOT / "profiles" / f"{workload}_hbm_traffic.txt"
    for line in f.read_text().splitlines() if f.exists() else ():
        w = line.split()
        if len(w) >= 3 and w[0] == "traffic_bytes_per_launch" and w[1] == kernel:
            return float(w[2]), (w[4] if len(w) >= 5 else None)
    return None, None


def run_stack(args, with_oracle: bool):
    """The whole-model sweep: 32 decoder blocks x 7 linear layers of the Llama-2-7B shapes
    (6.476e9 parameters, 809.5 M groups, 1x16 codebook per matrix, tau = 0.01 per matrix).
    Inputs are drawn ON THE DEVICE with torch's generator (same distributions as workloads.py,
    whose host-side tensors for this configuration would need 78 GB of host memory).
    One step = dequantize -> targets + selection -> re-encode -> dequantize for all 224 matrices,
    dealt to several contexts on streams of their own.  With `with_oracle` one device-drawn
    matrix is copied to the host before the sweep and its result afterwards: the oracle repeats
    its step there (ids in full, the search on a bounded sample of the selected groups), which
    both checks what the sweep computed and gives the oracle's rate on this configuration.
    Returns the result line as a dict."""
    import numpy as np
    import torch

    import workloads
    from paper_2405_14852_amd import Layout, PVContext

    dev = torch.device("cuda:0")
    # The matrices are independent calls.  With --streams S they are dealt round-robin to S
    # contexts, each on a stream of its own (default priority) with its own T / W scratch, so
    # that the short latency-bound kernels of one matrix overlap the streaming kernels of another.
    nstreams = max(1, args.streams)
    streams = [torch.cuda.current_stream(dev)] + [torch.cuda.Stream(device=dev) for _ in range(nstreams - 1)]
    ctxs = [PVContext(0, stream=st) for st in streams]
    ctx = ctxs[0]
    gen = torch.Generator(device=dev)
    layers = 32
    mats = []
    shapes = list(workloads.LLAMA2_7B_BLOCK.values())
    max_n = max(o * i for o, i in shapes)
    Ts = [torch.empty(max_n, dtype=torch.float32, device=dev) for _ in range(nstreams)]
    Wqs = [torch.empty(max_n, dtype=torch.float32, device=dev) for _ in range(nstreams)]
    total_params = total_groups = total_k = 0
    for layer in range(layers):
        for pid, (name, (o, i)) in enumerate(workloads.LLAMA2_7B_BLOCK.items()):
            gen.manual_seed(layer * 16 + pid + 1)
            lay = Layout(o, i, 8, 1, 16)
            N = o * i // 8
            k = workloads.num_selected(N, 0.01)
            m = {
                "name": f"layer{layer}.{name}",
                "lay": lay, "k": k, "n": o * i,
                "W": torch.randn(o, i, generator=gen, device=dev) * 0.02,
                "G": torch.randn(o, i, generator=gen, device=dev) * 1e-4,
                "cb": torch.randn(1, 65536, 8, generator=gen, device=dev) * 0.02,
                "sc": torch.rand(o, generator=gen, device=dev) + 0.5,
                "codes": torch.randint(0, 65536, (o, i // 8, 1), generator=gen, device=dev,
                                       dtype=torch.int32).to(torch.uint16),
                "idx": torch.empty(k, dtype=torch.int32, device=dev),
            }
            mats.append(m)
            total_params += o * i
            total_groups += N
            total_k += k
    nchs = [torch.zeros(1, dtype=torch.int64, device=dev) for _ in range(nstreams)]
    torch.cuda.synchronize()

    # the matrix the oracle repeats: one of the wide ones in the middle of the stack, which the
    # sweep reaches on a stream other than the first
    probe = next(j for j, m in enumerate(mats) if m["name"] == "layer17.down_proj")
    host = None
    if with_oracle:
        m = mats[probe]
        host = {key: m[key].cpu().numpy() for key in ("W", "G", "cb", "sc")}
        host["codes0"] = m["codes"].view(torch.int16).cpu().numpy().view(np.uint16)
        codes0_dev = [mm["codes"].view(torch.int16).clone() for mm in mats]   # restored after the check

    def step(lanes=nstreams):
        for j, m in enumerate(mats):
            c = j % lanes
            cx, nch = ctxs[c], nchs[c]
            lay = m["lay"]
            t, wq = Ts[c][: m["n"]].view(lay.out_features, lay.in_features), Wqs[c][: m["n"]].view(
                lay.out_features, lay.in_features)
            cx.pv_dequantize(lay, m["codes"], m["cb"], m["sc"], wq)
            cx.pv_encode_targets_select(lay, m["W"], m["G"], 1.0, t, m["k"], m["idx"])
            cx.pv_reencode_groups(lay, t, m["cb"], m["sc"], m["idx"], m["k"], 1, m["codes"], nch)
            cx.pv_dequantize(lay, m["codes"], m["cb"], m["sc"], wq)

    steps = max(1, min(args.steps, 5))
    warmup = max(1, min(args.warmup, 1))
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    check = None
    if with_oracle:
        # the first (warm-up) sweep started from the drawn codes: that is the one the oracle repeats
        import oracle
        m = mats[probe]
        got = m["codes"].view(torch.int16).cpu().numpy().view(np.uint16)
        idx_gpu = m["idx"].cpu().numpy()
        t1 = time.perf_counter()
        T_ref = oracle.encode_targets(host["W"], host["G"], 1.0)
        idx_ref = oracle.select_topk_groups(T_ref, host["W"], 8, m["k"])
        t2 = time.perf_counter()
        sample = idx_ref[:: max(1, len(idx_ref) // 8192)]
        new_ref, info = oracle.reencode_groups(T_ref, host["cb"], host["sc"], sample, host["codes0"])
        t3 = time.perf_counter()
        differ = np.nonzero(got.reshape(-1)[sample] != new_ref.reshape(-1)[sample])[0]
        ok = bool(np.array_equal(idx_gpu, idx_ref)) and bool(info["near_tie"][differ].all())
        untouched = np.ones(got.size, bool)
        untouched[idx_ref] = False
        ok = ok and bool(np.array_equal(got.reshape(-1)[untouched], host["codes0"].reshape(-1)[untouched]))
        # per-group cost of the search does not depend on the data: scale the sample to the matrix
        secs = (t2 - t1) + (t3 - t2) * (m["k"] / len(sample))
        check = {"value": m["k"] / secs, "unit": "groups/s", "cores": oracle.num_threads(), "kind": "oracle",
                 "sample": f"{m['name']} of the device-drawn stack copied to the host: targets and selection "
                           f"in full ({t2 - t1:.2f} s), search on {len(sample)} of {m['k']} selected groups "
                           f"({t3 - t2:.2f} s) and scaled; the rate is per matrix, the stack has 224",
                 "ids_equal_oracle": bool(np.array_equal(idx_gpu, idx_ref)),
                 "codes_equal_oracle_on_sample": ok, "sample_groups_differing_on_near_ties": int(len(differ))}
        for mm, c0 in zip(mats, codes0_dev):
            mm["codes"].view(torch.int16).copy_(c0)
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / steps
    ctx.pv_timing_enable(True)      # per-kernel breakdown: one more sweep, all on one stream
    ctx.pv_timing_reset()
    step(lanes=1)
    torch.cuda.synchronize()
    kern = {}
    for name in ("dequantize", "encode_targets", "select", "prep", "score_mfma", "rerank", "exact_scan"):
        t_ms, n = ctx.pv_timing_read(name)
        if n:
            kern[name] = {"ms_per_step": t_ms, "launches_per_step": n}
    ctx.pv_timing_enable(False)
    flops = 2.0 * total_k * 65536 * 8
    a = flops / (kern["score_mfma"]["ms_per_step"] * 1e-3) / 1e12
    out = {
        "metric": "groups_reencoded_per_s", "value": total_k / (ms * 1e-3), "unit": "groups/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic (drawn on the device)",
        "config": {"workload": "c4_llama2_7b_stack", "matrices": len(mats), "parameters": total_params,
                   "groups": total_groups, "k_selected": total_k, "tau": 0.01, "group_size": 8,
                   "num_codebooks": 1, "nbits": 16, "streams": nstreams},
        "roofline": {"kernel": "k_score_mfma", "bound": "mfma", "achieved": a, "peak": PEAK_MFMA_F16,
                     "unit": "TFLOP/s", "frac": a / PEAK_MFMA_F16, "traffic": None},
        "cpu_baseline": check,
        "streaming_GBps": (12.0 + 0.5 + 2 * 4.25) * total_params
        / ((kern["dequantize"]["ms_per_step"] + kern["encode_targets"]["ms_per_step"]) * 1e-3) / 1e9,
        "kernels": kern,
    }
    for c in ctxs:
        c.close()
    del mats, Ts, Wqs
    torch.cuda.empty_cache()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2_4096x4096_1x16")
    ap.add_argument("--search-mode", type=int, default=0,
                    help="0 = matrix-core filter + exact re-rank, 1 = exact scan only")
    ap.add_argument("--separate-calls", action="store_true",
                    help="pv_encode_targets + pv_select_topk_groups instead of the fused call")
    ap.add_argument("--path", choices=("vstep", "trust_ratio", "pstep", "stochastic"), default="vstep",
                    help="trust_ratio: the subspace size is found by pv_reencode_trust_ratio "
                         "(W = the dequantised codes, gradient x40 so that codes move, ratio 0.01, "
                         "all k groups of the workload are candidates); pstep: one call of "
                         "pv_codebook_grads (gradients of codebooks and scales) per step; "
                         "stochastic: the V step with pv_reencode_groups_stochastic (two nearest "
                         "codewords, power 5) in place of the nearest-codeword search")
    ap.add_argument("--adam", action="store_true",
                    help="targets from one Adam update and selection by its size in one sweep "
                         "(pv_encode_targets_adam_select, beta 0.9/0.95, lr 3e-3)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--structured", action="store_true",
                    help="W = the dequantised initial codes and the gradient x40 (the regime of a "
                         "real V step) instead of the configuration's dense Gaussian W")
    ap.add_argument("--sparse-a9", action="store_true",
                    help="last dequantize of the step rewrites only the re-encoded groups "
                         "(pv_dequantize_groups); same weights, not the default")
    ap.add_argument("--no-stack", dest="stack", action="store_false",
                    help="leave out the `stack` key (the 224-matrix sweep of c4_llama2_7b_stack, "
                         "which the default line carries beside the single-matrix figure)")
    ap.add_argument("--streams", type=int, default=4,
                    help="c4_llama2_7b_stack only: contexts/streams the 224 matrices are dealt to")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); the path shards by "
              "matrix or by rows with no exchange inside the V step", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import workloads
    from paper_2405_14852_amd import Layout, PVContext

    if args.workload == "c4_llama2_7b_stack":
        print(json.dumps(run_stack(args, with_oracle=not args.no_cpu_baseline)))
        return 0

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    wl = workloads.make_config(args.workload, seed=0)
    L = wl.layout
    lay = Layout(L.out_features, L.in_features, L.group_size, L.num_codebooks, L.nbits)
    k = wl.k
    ctx = PVContext(0)
    ctx.pv_set_search_mode(args.search_mode)

    W = torch.from_numpy(wl.W).to(dev)
    G = torch.from_numpy(wl.G).to(dev)
    cb = torch.from_numpy(wl.codebooks).to(dev)
    sc = torch.from_numpy(wl.scales).to(dev)
    codes0 = torch.from_numpy(wl.codes.view(np.int16)).to(dev).view(torch.uint16)
    codes = codes0.clone()
    T = torch.empty_like(W)
    Wq = torch.empty_like(W)
    idx = torch.empty(k, dtype=torch.int32, device=dev)
    nch = torch.zeros(1, dtype=torch.int64, device=dev)

    if args.structured and args.path == "vstep":
        # the regime of a real V step: W is the dequantised current codes and the update is a
        # fraction of the codeword spacing (gradient x40, as in the trust-ratio path)
        ctx.pv_dequantize(lay, codes0, cb, sc, W)
        G.mul_(40.0)
        torch.cuda.synchronize()

    if args.path == "trust_ratio":
        G.mul_(40.0)
        rank = torch.empty(k, dtype=torch.int32, device=dev)
        napp = torch.zeros(1, dtype=torch.int64, device=dev)
        tstats = torch.zeros(2, dtype=torch.float64, device=dev)

    m_adam = torch.zeros_like(W) if args.adam else None
    v_adam = torch.zeros_like(W) if args.adam else None
    adam_step = [0]

    def step_trust():
        codes.view(torch.int16).copy_(codes0.view(torch.int16))
        ctx.pv_dequantize(lay, codes, cb, sc, Wq)                 # x^k, also the W of Eq. 7
        ctx.pv_encode_targets(lay, Wq, G, wl.alpha, T)
        ctx.pv_reencode_trust_ratio(lay, T, Wq, cb, sc, k, max(1, k // 10), 0.01, wl.beam_width,
                                    codes, rank, napp, tstats)
        ctx.pv_dequantize(lay, codes, cb, sc, Wq)

    if args.path == "pstep":
        gcb = torch.empty_like(cb)
        gsc = torch.empty_like(sc)

    def step():
        if args.path == "trust_ratio":
            return step_trust()
        if args.path == "pstep":
            return ctx.pv_codebook_grads(lay, G, codes0, cb, sc, gcb, gsc)
        codes.view(torch.int16).copy_(codes0.view(torch.int16))   # same work every step
        ctx.pv_dequantize(lay, codes, cb, sc, Wq)
        if args.adam:
            adam_step[0] += 1
            ctx.pv_encode_targets_adam_select(lay, W, G, m_adam, v_adam, adam_step[0], 3e-3, 0.9,
                                              0.95, 1e-8, T, k, idx)
        elif args.separate_calls:
            ctx.pv_encode_targets(lay, W, G, wl.alpha, T)
            ctx.pv_select_topk_groups(lay, T, W, k, idx)
        else:   # same outputs, T and W are not read back for the scores
            ctx.pv_encode_targets_select(lay, W, G, wl.alpha, T, k, idx)
        if args.path == "stochastic":
            ctx.pv_reencode_groups_stochastic(lay, T, cb, sc, idx, k, 5, 2024, codes, nch)
        else:
            ctx.pv_reencode_groups(lay, T, cb, sc, idx, k, wl.beam_width, codes, nch)
        if args.sparse_a9:   # Wq holds the old codes' weights: only the re-encoded groups change
            ctx.pv_dequantize_groups(lay, codes, cb, sc, idx, k, Wq)
        else:
            ctx.pv_dequantize(lay, codes, cb, sc, Wq)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # the K timed steps run as (up to) five batches with a synchronisation after each, so that
    # the line also carries the spread; ms_per_step is the whole region over K
    nb = min(5, args.steps)
    sizes = [args.steps // nb + (1 if b < args.steps % nb else 0) for b in range(nb)]
    batch_ms = []
    t0 = time.perf_counter()
    for n in sizes:
        tb = time.perf_counter()
        for _ in range(n):
            step()
        torch.cuda.synchronize()
        batch_ms.append(1e3 * (time.perf_counter() - tb) / n)
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    changed = int(nch.item())
    stats = ctx.pv_reencode_stats()

    # second timed region with HIP events around every kernel group (per-kernel durations)
    ctx.pv_timing_enable(True)
    ctx.pv_timing_reset()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    kern = {}
    for name in ("dequantize", "encode_targets", "group_scores", "select", "prep", "score_mfma",
                 "rerank", "exact_scan", "beam", "trust_ratio", "pstep", "stochastic"):
        ms, n = ctx.pv_timing_read(name)
        if n:
            kern[name] = {"ms_per_step": ms / args.steps, "launches_per_step": n / args.steps,
                          "avg_ms": ms / n}
    ctx.pv_timing_enable(False)

    g, B, M = L.group_size, L.nbits, L.num_codebooks
    params = L.out_features * L.in_features
    reenc_ms = sum(kern[n]["ms_per_step"] for n in ("prep", "score_mfma", "rerank", "exact_scan", "beam", "stochastic")
                   if n in kern)
    dominant = max(kern, key=lambda n: kern[n]["ms_per_step"])
    flops_contraction = 2.0 * k * (1 << B) * g * M            # algorithmic: 2*g*2^B per group
    roofline = None
    if args.path == "pstep":
        # algorithmic traffic: G once for the codebook sums and once for the scale sums, codes for
        # each, the gradients written
        nbytes = 2.0 * 4.0 * params + 2.0 * 2.0 * M * (params / g) + 4.0 * (M * (1 << B) * g + L.out_features)
        a = nbytes / (kern["pstep"]["avg_ms"] * 1e-3) / 1e9
        small = g % 4 == 0 and M * (1 << B) * g * 8 <= 64 * 1024 and (params // g) // (1 << B) >= 64
        route = "fixed-point LDS tables" if small else "sort + segmented sums"
        roofline = {"kernel": f"pv_codebook_grads ({route})", "bound": "hbm", "achieved": a,
                    "peak": PEAK_HBM, "unit": "GB/s", "frac": a / PEAK_HBM, "traffic": None}
    elif dominant == "score_mfma":
        a = flops_contraction / (kern[dominant]["avg_ms"] * 1e-3) / 1e12
        traffic, at_commit = measured_traffic("k_score_mfma", args.workload)
        roofline = {"kernel": "k_score_mfma", "bound": "mfma", "achieved": a, "peak": PEAK_MFMA_F16,
                    "unit": "TFLOP/s", "frac": a / PEAK_MFMA_F16,
                    "traffic": traffic, "traffic_measured_at_commit": at_commit}
    elif dominant in ("exact_scan", "beam", "stochastic"):
        # algorithmic double-precision work: 2 g FLOP (one multiply-add per dimension) for every
        # objective the search is defined to evaluate, whatever form the kernel computes it in
        tuples = k * ((1 << B) if M == 1 else (1 << B) * (1 + (M - 1) * wl.beam_width))
        fl = tuples * g * 2.0
        # the beam launches of one step (filter + exact remainder) count as one unit of work
        a = fl / (kern[dominant]["ms_per_step"] * 1e-3) / 1e12
        filtered = dominant == "beam" and args.search_mode == 0 and M == 2 and B == 8
        # the filtered 2 x 8-bit search evaluates in fp32 / fp16 with fp32 accumulation (the
        # contraction has only g terms per objective, its cost is the comparison work on the
        # vector units); the exact kernels evaluate in fp64
        peak = PEAK_F32 if filtered else PEAK_F64
        roofline = {"kernel": "k_beam_2x8_f16 + k_beam_2x8" if filtered else "k_" + dominant,
                    "bound": "alu", "achieved": a, "peak": peak, "unit": "TFLOP/s", "frac": a / peak,
                    "traffic": None}
        if filtered:
            roofline["frac_of_mfma_f16_peak"] = a / PEAK_MFMA_F16
    else:
        per_param = {"encode_targets": 28.0 + 4.0 / g if args.adam else 12.0 + (0.0 if args.separate_calls else 4.0 / g),
                     "group_scores": 8.0 + 4.0 / g,
                     "dequantize": 4.0 + 2.0 * M / g}.get(dominant)
        if per_param is not None:     # a kernel with no traffic model here gets no roofline at all
            a = per_param * params / (kern[dominant]["avg_ms"] * 1e-3) / 1e9
            roofline = {"kernel": "k_" + dominant, "bound": "hbm", "achieved": a, "peak": PEAK_HBM,
                        "unit": "GB/s", "frac": a / PEAK_HBM, "traffic": None}

    # ceilings of this machine at this moment, measured with two kernels of the library: a plain
    # 64 MiB streaming copy and a loop of nothing but fp16 matrix instructions
    csrc = torch.empty(16 * 1024 * 1024, dtype=torch.float32, device=dev).normal_()
    cdst = torch.empty_like(csrc)
    sink = torch.empty(256 * 16 * 64, dtype=torch.float32, device=dev)
    mfma_iters = 4096
    for _ in range(3):
        ctx.pv_probe_copy(cdst, csrc)
        waves = ctx.pv_probe_mfma_f16(mfma_iters, sink)
    torch.cuda.synchronize()
    ctx.pv_timing_enable(True)
    ctx.pv_timing_reset()
    for _ in range(20):
        ctx.pv_probe_copy(cdst, csrc)
    for _ in range(5):
        ctx.pv_probe_mfma_f16(mfma_iters, sink)
    t_copy, n_copy = ctx.pv_timing_read("probe_copy")
    t_mfma, n_mfma = ctx.pv_timing_read("probe_mfma")
    ctx.pv_timing_enable(False)
    ceilings = {
        "copy_GBps": 2.0 * csrc.numel() * 4 / (t_copy / n_copy * 1e-3) / 1e9,
        "mfma_f16_TFLOPs": waves * mfma_iters * 2.0 * 32 * 32 * 16 / (t_mfma / n_mfma * 1e-3) / 1e12,
        "how": "pv_probe_copy on 64 MiB (read + write), pv_probe_mfma_f16 (4 waves per SIMD, "
               "independent v_mfma_f32_32x32x16_f16 only), HIP events",
    }
    del csrc, cdst

    hbm = {}
    for name, per_param in (("encode_targets", 28.0 + 4.0 / g if args.adam else 12.0 + (0.0 if args.separate_calls else 4.0 / g)),
                            ("group_scores", 8.0 + 4.0 / g),
                            ("dequantize", 4.0 + 2.0 * M / g)):
        if name in kern:
            hbm[name + "_GBps"] = per_param * params / (kern[name]["avg_ms"] * 1e-3) / 1e9
    if "select" in kern:   # the four radix / compaction launches each read the score array once
        hbm["select_passes_GBps"] = 4 * 4.0 * (params / g) / (kern["select"]["avg_ms"] * 1e-3) / 1e9

    cpu = None
    if not args.no_cpu_baseline and args.path == "pstep":
        import oracle
        t1 = time.perf_counter()
        gc_ref, gs_ref = oracle.codebook_grads(wl.G, wl.codes, wl.codebooks, wl.scales)
        t2 = time.perf_counter()
        cpu = {"value": (params / g) / (t2 - t1), "unit": "groups/s", "cores": 1, "kind": "oracle",
               "sample": f"the whole matrix of {args.workload} ({t2 - t1:.3f} s, sequential by definition)",
               "codebook_grads_equal_oracle": bool(np.array_equal(gcb.cpu().numpy(), gc_ref)),
               "scale_grads_max_abs_diff": float(np.abs(gsc.cpu().numpy().astype(np.float64) - gs_ref).max())}
    elif not args.no_cpu_baseline and args.path == "trust_ratio":
        import oracle
        t1 = time.perf_counter()
        Wq_ref = oracle.dequantize(wl.codes, wl.codebooks, wl.scales)
        T_ref = oracle.encode_targets(Wq_ref, wl.G * np.float32(40.0), wl.alpha)
        new_ref, tinfo = oracle.reencode_trust_ratio(T_ref, Wq_ref, wl.codebooks, wl.scales, wl.codes,
                                                     k, max(1, k // 10), 0.01, wl.beam_width)
        oracle.dequantize(new_ref, wl.codebooks, wl.scales)
        t2 = time.perf_counter()
        got = codes.view(torch.int16).cpu().numpy().view(np.uint16)
        cpu = {"value": k / (t2 - t1), "unit": "groups/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"one whole trust-ratio step of {args.workload} ({t2 - t1:.2f} s; the oracle "
                         f"stops re-encoding at the chunk that breaks the bound, {tinfo['num_applied']} kept)",
               "codes_equal_oracle": bool(np.array_equal(got, new_ref)),
               "kept_equal_oracle": int(napp.item()) == tinfo["num_applied"]}
    elif not args.no_cpu_baseline and args.path == "stochastic":
        import oracle
        T_ref = oracle.encode_targets(wl.W, wl.G, wl.alpha)
        idx_ref = oracle.select_topk_groups(T_ref, wl.W, g, k)
        sample = idx_ref[:: max(1, len(idx_ref) // 4096)]
        t1 = time.perf_counter()
        new_ref, sinfo = oracle.reencode_stochastic(T_ref, wl.codebooks, wl.scales, sample, wl.codes,
                                                    power=5, seed=2024)
        t2 = time.perf_counter()
        got = codes.view(torch.int16).cpu().numpy().view(np.uint16)
        differ = np.nonzero(got.reshape(-1)[sample] != new_ref.reshape(-1)[sample])[0]
        cpu = {"value": len(sample) / (t2 - t1), "unit": "groups/s", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": f"the rounding of {len(sample)} of {k} selected groups "
                                           f"({t2 - t1:.2f} s); search only, no streaming parts",
               "codes_equal_oracle_on_sample": bool(sinfo["near_tie"][differ].all())}
    elif not args.no_cpu_baseline and not args.adam:
        import oracle
        if args.structured:      # the oracle's own copies of the same inputs
            wl.W = oracle.dequantize(wl.codes, wl.codebooks, wl.scales)
            wl.G = wl.G * np.float32(40.0)
        t1 = time.perf_counter()
        Wq_ref = oracle.dequantize(wl.codes, wl.codebooks, wl.scales)
        T_ref = oracle.encode_targets(wl.W, wl.G, wl.alpha)
        idx_ref = oracle.select_topk_groups(T_ref, wl.W, g, k)
        # bounded sample of the search: cost per group is data-independent
        sample = idx_ref if M == 1 and k * (1 << B) * g <= 3e10 else idx_ref[:: max(1, len(idx_ref) // 4096)]
        t2 = time.perf_counter()
        new_ref, info = oracle.reencode_groups(T_ref, wl.codebooks, wl.scales, sample, wl.codes,
                                               beam_width=wl.beam_width)
        t3 = time.perf_counter()
        oracle.dequantize(new_ref, wl.codebooks, wl.scales)
        t4 = time.perf_counter()
        stream_s = (t2 - t1) + (t4 - t3)
        search_s = (t3 - t2) * (k / len(sample))
        cpu = {"value": k / (stream_s + search_s), "unit": "groups/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"one whole step of {args.workload}; search timed on {len(sample)} of {k} "
                         f"selected groups and scaled ({t3 - t2:.2f} s measured), streaming parts "
                         f"in full ({stream_s:.2f} s)"}
        if len(sample) == k:
            got = codes.view(torch.int16).cpu().numpy().view(np.uint16)
            cpu["codes_equal_oracle"] = bool(np.array_equal(got, new_ref))

    n_units = (params // g) if args.path == "pstep" else k
    out = {
        "metric": "groups_differentiated_per_s" if args.path == "pstep" else "groups_reencoded_per_s",
        "value": n_units / (ms_per_step * 1e-3), "unit": "groups/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if "score_mfma" in kern else "f64", "data": "synthetic",
        "config": {"workload": args.workload, "out_features": L.out_features,
                   "in_features": L.in_features, "group_size": g, "num_codebooks": M, "nbits": B,
                   "tau": wl.tau, "k_selected": k, "beam_width": wl.beam_width,
                   "search_mode": args.search_mode, "path": args.path, "sparse_a9": bool(args.sparse_a9), "structured": bool(args.structured),
                   "calls": "fused adam targets+select" if args.adam else
                            "separate" if args.separate_calls else "fused targets+select"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "batches": {"count": nb, "ms_per_step_median": float(np.median(batch_ms)),
                    "ms_per_step_min": min(batch_ms), "ms_per_step_max": max(batch_ms)},
        "reencode_only_groups_per_s": k / (reenc_ms * 1e-3) if reenc_ms else None,
        "scoring_algorithmic_TFLOPs": (flops_contraction / (kern["score_mfma"]["avg_ms"] * 1e-3) / 1e12
                                       if "score_mfma" in kern else None),
        "scoring_frac_of_mfma_peak": (flops_contraction / (kern["score_mfma"]["avg_ms"] * 1e-3) / 1e12
                                      / PEAK_MFMA_F16 if "score_mfma" in kern else None),
        "hbm": hbm, "measured_ceilings": ceilings, "kernels": kern, "groups_changed": changed, "reencode_stats": stats,
    }
    if args.path == "trust_ratio":
        out["trust_ratio"] = {"ratio": 0.01, "candidates": k, "kept": int(napp.item()),
                              "change_sq": float(tstats[0].item()), "norm_sq": float(tstats[1].item())}
    if args.stack:
        # the whole-model sweep beside the single-matrix figure (a few seconds of GPU time)
        ctx.close()
        del W, G, T, Wq
        torch.cuda.empty_cache()
        st = run_stack(args, with_oracle=not args.no_cpu_baseline)
        out["stack"] = {key: st[key] for key in ("value", "unit", "steps", "ms_per_step", "config",
                                                  "roofline", "cpu_baseline", "streaming_GBps")}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
