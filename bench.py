#!/usr/bin/env python3
"""Benchmark of the PAHQ / ACDC edge-ablation hot path on one MI355X.

Workload (config 3, GPT-2-small shape, seeded synthetic weights and tokens):
one step = one pass over the whole split-QKV graph, every one of its 32 491
edges evaluated once by pahq_eval_edge_list against the empty removed set under
PAHQ precision (fp32 investigated head, everything else FP8 E4M3 operands).
That is one patched forward + KL per edge: the paper's per-edge cost
(Appendix "Integration with ACDC", third inference; Eq. Delta L), with the
clean / corrupted runs cached once.  value = edges evaluated per second.

Two further regimes are measured in the same run and reported with their own
roofline blocks, because the empty removed set is the best case of this design
(all receivers of a layer share one input there):
  gather_regime   the same candidates against a seeded removed set with 90 % of
                  the edges removed: every receiver gathers its own sum of
                  sender tiles (what a sweep looks like once it has removed
                  most of the graph);
  sweep           pahq_acdc_sweep at thresholds that leave a circuit (1e-4: about
                  80 edges after 1 700 decisions; 3e-5: about 800 edges, every one
                  of the 32 491 edges decided) and at the thresholds the config names (on random-initialised
                  weights each of those exceeds every increment: 157 evaluations
                  and an empty circuit).

Prints ONE JSON line.  --gpus above 1 is refused: this build is single-GPU.
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAKS = {"gemm_fp8": ("mfma", 2500.0, "TFLOP/s"), "oproj_fused": ("mfma", 2500.0, "TFLOP/s"),
         "gemm_f32": ("mfma", 157.3, "TFLOP/s")}
FP8_PEAK = 5000.0      # dense FP8 matrix-core peak, for reading the fp16-path fraction against the task's target
HBM_PEAK = 8000.0      # GB/s

# Which kernels the library launches for a kernel class (rocprofv3 names them; the library reports classes).
KERNELS_OF_CLASS = {
    "gemm_fp8": ("pahq::gemm_p_k", "pahq::gemm_x_k"),
    "gather_norm_quant": ("pahq::build_inputs_k", "pahq::build_inputs_shared_k"),
    "hidden_quant": ("pahq::hidden_quant_vec_k",), "attention": ("pahq::attention_mfma_k",),
    "oproj_fused": ("pahq::oproj_x_k",), "gemm_f32": ("pahq::gemm_f32_k",), "edge_patch": ("pahq::patch_indep_k", "pahq::patch_build_k"),
    "kl": ("pahq::kl_reduce_k", "pahq::kl_mean_k"),
}
PROFILE_FILES = {"all_edges": "hbm_traffic_per_kernel_cfg3_all_edges_pmc.txt",
                 "gather_regime": "hbm_traffic_per_kernel_cfg3_gather_regime_pmc.txt"}


def traffic_from_profile(regime, kernel_class, workload_key):
    """HBM bytes per launch of a kernel class, read from the committed rocprofv3 PMC summary of the same
    workload (profiles/): counters cannot be read from inside this process.  The summary states the
    workload it was taken on and, per kernel, launches and calibrated read / write MB per launch.  Returns
    None when the summary is of another workload; raises when the summary does not list the kernels this
    class launches (then it predates a kernel change and must be re-measured)."""
    path = os.path.join(ROOT, "profiles", PROFILE_FILES[regime])
    if not os.path.exists(path):
        return None
    rows, workload = {}, None
    for line in open(path):
        if line.startswith("# workload:"):
            workload = line.split(":", 1)[1].strip()
        m = re.match(r"^(\S.*?)\s+(\d+)\s+([0-9.]+)\s+([0-9.]+)\s*$", line)
        if m and not line.startswith("#"):
            rows[m.group(1).strip()] = (int(m.group(2)), float(m.group(3)), float(m.group(4)))
    if workload != workload_key:
        return None
    mine = {k: v for k, v in rows.items() if any(k.startswith(p) for p in KERNELS_OF_CLASS.get(kernel_class, ()))}
    if not mine:
        raise RuntimeError(f"{path} lists no kernel of class {kernel_class}: the summary is stale, re-measure it")
    n = sum(v[0] for v in mine.values())
    return round(sum(v[0] * (v[1] + v[2]) for v in mine.values()) / n * 1e6)


def all_edges_pass(gm, P, cfg, receivers, stride=1):
    """Every in-edge of the given receivers, once, layer by layer from the top (as the sweep visits them), through
    pahq_eval_edge_list: within a layer the query, key and value inputs of a head follow each other in that
    order, so that their candidates share device batches."""
    n, t_last = 0, time.perf_counter()
    todo = [int(r) for r in receivers[::-1][::stride]]
    per_layer = 3 * cfg.n_heads + (1 if cfg.d_mlp > 0 else 0)
    chunks = {}
    for r in todo:
        chunks.setdefault(r // per_layer, []).append(r)
    for i, layer in enumerate(sorted(chunks, reverse=True)):
        rs = sorted(chunks[layer], key=lambda r: (-((r % per_layer) // 3), (r % per_layer) % 3))     # heads descending, q k v ascending
        recv = np.concatenate([np.full(P.n_upstream(cfg, r), r, np.int32) for r in rs])
        send = np.concatenate([np.arange(P.n_upstream(cfg, r), dtype=np.int32) for r in rs])
        if cfg.fp32_residency and i + 1 < len(chunks):
            # the caller knows its own order: the layer underneath comes next, its heads' fp32 weights can move now
            gm.prefetch_heads(sorted(chunks, reverse=True)[i + 1], range(cfg.n_heads))
        gm.eval_edge_list(recv, send)
        n += send.size
        if time.perf_counter() - t_last > 30.0:          # long passes (the large configs) say where they are
            print(f"bench.py: layer {layer} ({i + 1} of {len(chunks)}), {n} edges", file=sys.stderr, flush=True)
            t_last = time.perf_counter()
    return n


def kernel_table(prof):
    out = {}
    for k, s in prof.items():
        if s["launches"] == 0:
            continue
        e = {"launches": s["launches"], "ms_total": round(s["ms"], 3), "us_avg": round(1e3 * s["ms"] / s["launches"], 2)}
        if s["flops"] > 0:
            e["TFLOP/s"] = round(s["flops"] / (s["ms"] * 1e-3) / 1e12, 2)
        if s["bytes"] > 0:
            e["GB/s"] = round(s["bytes"] / (s["ms"] * 1e-3) / 1e9, 1)
        out[k] = e
    return out


def roofline_of(dom, s, share, mma, traffic, measured):
    """The roofline block of kernel class `dom` from its event-timed launches `s`."""
    if dom in PEAKS:
        bound, peak, unit = PEAKS[dom]
        if mma == 0 and dom != "gemm_f32":
            peak = FP8_PEAK
        ach = s["flops"] / (s["ms"] * 1e-3) / 1e12
    else:
        bound, peak, unit = "hbm", HBM_PEAK, "GB/s"
        ach = s["bytes"] / (s["ms"] * 1e-3) / 1e9
    r = {"kernel": dom, "bound": bound, "achieved": round(ach, 2), "peak": peak, "unit": unit, "frac": round(ach / peak, 4),
         "traffic": traffic, "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated; read from profiles/)",
         "algorithmic_bytes_per_launch": (round(s["bytes"] / s["launches"]) if s["bytes"] > 0 else None),
         "avg_launch_us": round(1e3 * s["ms"] / s["launches"], 2), "launches_measured": s["launches"],
         "measured": measured, "share_of_kernel_time": round(share, 3)}
    if dom in ("gemm_fp8", "oproj_fused") and mma == 1:
        r["frac_of_fp8_peak"] = round(ach / FP8_PEAK, 4)      # the products are E4M3 x E4M3; the fp16 matrix cores form them exactly
    return r


def gather_regime(gm, P, cfg, receivers, torch, workload_key, mma):
    """The same candidates against a seeded removed set with 90 % of all edges removed, where receivers no
    longer share their inputs and every one gathers its own sum of sender tiles.  A sample of receivers
    keeps it to about 15 s.  Events around every launch give the breakdown and the gather kernels' rate."""
    rng = np.random.default_rng(12345)
    removed = (rng.random(gm.n_edges) < 0.9).astype(np.uint8)
    first_edge = np.concatenate([[0], np.cumsum([P.n_upstream(cfg, q) for q in range(P.n_receivers(cfg))])])
    sample = receivers[:: max(1, len(receivers) // 24)][::-1]

    def run(limit_s):
        t0 = time.perf_counter()
        n = done = 0
        for r in sample:                       # descending; the large configs stop early
            # the state a sweep is in when it reaches r: edges into earlier receivers are all still there
            state = removed.copy()
            state[: first_edge[int(r)]] = 0
            gm.set_removed(state)
            senders = np.arange(P.n_upstream(cfg, int(r)), dtype=np.int32)
            gm.eval_edges(int(r), senders)
            n += senders.size
            done += 1
            if time.perf_counter() - t0 > limit_s:
                break
        torch.cuda.synchronize()
        return n, done, time.perf_counter() - t0

    torch.cuda.synchronize()
    n, done, dt = run(12.0)                    # timed without events
    gm.set_profiling_sample(None, 1)
    gm.set_profiling(True)
    run(6.0)                                   # again, events around every launch
    prof = gm.get_profile()
    gm.set_profiling(False)
    gm.set_removed(np.zeros(gm.n_edges, np.uint8))
    total = sum(v["ms"] for v in prof.values())
    dom = "gather_norm_quant"
    return {"edges_per_s": round(n / dt, 1), "edges": int(n), "receivers": int(done), "removed_fraction": 0.9, "seed": 12345,
            "roofline": roofline_of(dom, prof[dom], prof[dom]["ms"] / total, mma,
                                    traffic_from_profile("gather_regime", dom, workload_key),
                                    "HIP events on the library's stream around every launch, second run of the sample"),
            "kernels": kernel_table(prof)}


def cpu_baseline(name, shape, w, clean, corrupt):
    """The oracle's cached fast path, timed on the host cores, on a bounded sample: 16 candidates into key
    inputs of heads in four receiver layers spread over the depth (a candidate into layer l recomputes
    layers l .. L-1), all cores; and one of them again on a single thread."""
    from oracle.model import Model as OModel
    from oracle.acdc import Acdc
    t0 = time.time()
    oa = Acdc(OModel(shape, w), clean, corrupt)
    oa.base()
    t_base = time.time() - t0
    g = oa.g
    L = shape.n_layers
    layers = sorted({max(0, min(L - 1, round(f * (L - 1)))) for f in (0.1, 0.37, 0.64, 0.91)})
    n_cand, dt, per_layer = 0, 0.0, {}
    for lv in layers:
        v = g.headin(lv, 0, 1)
        oa.kl_fast(v, g.empty_removed())       # state of the receiver's fp32 head (shared by its candidates): not timed
        n_up = g.n_upstream(v)
        senders = sorted({0, n_up // 3, (2 * n_up) // 3, n_up - 1})
        t1 = time.time()
        for u in senders:
            oa.kl_edge(v, u)
        per_layer[lv] = (time.time() - t1) / len(senders)
        dt += time.time() - t1
        n_cand += len(senders)
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
        v = g.headin(layers[-1], 0, 1)
        oa.kl_fast(v, g.empty_removed())
        with threadpool_limits(limits=1):
            t1 = time.time()
            oa.kl_edge(v, 0)
            one_thread = time.time() - t1
        single = {"s_per_edge_1_thread": round(one_thread, 3), "s_per_edge_all_cores_same_candidate": round(per_layer[layers[-1]], 3),
                  "receiver_layer": layers[-1]}
    except Exception:
        cores, single = os.cpu_count(), None
    return {"value": n_cand / dt, "unit": "edges/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{name}: {n_cand} candidate edges, four senders into the key input of head (l,0) for receiver layers "
                      f"l = {layers} of {L} ({[L - l for l in layers]} layers recomputed), oracle cached fast path, fp64 numpy "
                      f"(not compiled code) on all host cores; the one-off clean/corrupt cache ({t_base:.0f} s) and each head's "
                      f"precision state are not in the timed part",
            "s_per_edge_by_receiver_layer": {str(k): round(v, 3) for k, v in per_layer.items()}, "single_thread": single}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="cfg3")
    ap.add_argument("--batch", type=int, default=128, help="candidates per device batch")
    ap.add_argument("--mma", type=int, default=1,
                    help="1 (default): e4m3 codes decoded in registers, fp16 matrix cores, exact fp32 sums; "
                         "0: the FP8 matrix-core instruction (faster, but its adder truncates: KL about 1.3%% low)")
    ap.add_argument("--precision", default="pahq", choices=("pahq", "all_fp8", "all_fp32"),
                    help="all_fp32: the unaccelerated ACDC of the paper's runtime table (no quantiser anywhere)")
    ap.add_argument("--nonattn-bf16", action="store_true",
                    help="bfloat16 operands for the MLP matrices and the unembedding (the heads stay on the e4m3 grid)")
    ap.add_argument("--low-bits", type=int, default=8, choices=(4, 8, 16), help="grid of the low-precision operands")
    ap.add_argument("--fp32-on-host", action="store_true",
                    help="the heads' fp32 masters stay in pinned host memory and are prefetched into 2 H device slots "
                         "(the paper's weight scheduler); reports the transfer counters")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--only", default=None, choices=(None, "all_edges", "gather_regime", "sweep", "policies"),
                    help="run one regime only (short runs under a profiler); 'policies' (never part of the default run) "
                         "sweeps once under each precision policy -- fp32 for the head an edge feeds (the default) and "
                         "fp32 for the edge's source head as Eq. P_t prints it -- and reports where they differ")
    ap.add_argument("--tau", type=float, default=None, help="threshold of the 'policies' comparison")
    ap.add_argument("--recv-stride", type=int, default=1,
                    help="evaluate only every k-th receiver (short runs under a profiler; the headline uses 1)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(candidates are independent: on several GPUs each would take a share of every batch)", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    import paper_2510_23264_amd as P

    if not torch.cuda.is_available():
        print("bench.py: no HIP device", file=sys.stderr)
        sys.exit(1)
    precision = {"pahq": P.PAHQ, "all_fp8": P.ALL_FP8, "all_fp32": P.ALL_FP32}[args.precision]
    shape, w, clean, corrupt, spec = synth.make_workload(args.config)
    gm = P.Model(shape, w, spec["B"], spec["S"], precision=precision, max_batch_edges=args.batch, mma=args.mma,
                 low_bits=args.low_bits, nonattn_bf16=args.nonattn_bf16, fp32_on_host=args.fp32_on_host)
    cfg = gm.cfg
    # configs that name a receiver sample (4 and 5) run the in-edges of that seeded sample
    receivers = synth.make_receiver_sample(P.n_receivers(cfg), spec["n_recv"], spec["seed"])
    gm.clean_cache(clean, corrupt)
    workload_key = f"{args.config} batch={args.batch} mma={args.mma} precision={args.precision}" + \
        (" nonattn_bf16" if args.nonattn_bf16 else "") + (f" low_bits={args.low_bits}" if args.low_bits != 8 else "") + \
        (" fp32_on_host" if args.fp32_on_host else "")
    do = lambda what: args.only in (None, what)

    out = {"metric": "patched edge evals/sec (GPT-2-small shape)", "value": None, "unit": "edges/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": None,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": ("f32" if args.precision == "all_fp32" else
                     "fp8_e4m3 (FP8 matrix cores)" if args.mma == 0 else
                     "fp8_e4m3 operands for the heads, bf16 for MLPs and unembedding, fp32 accumulate" if args.nonattn_bf16 else
                     "fp8_e4m3 operands, fp16 matrix cores, fp32 accumulate"),
           "data": "synthetic"}

    if do("all_edges"):
        for _ in range(args.warmup):
            all_edges_pass(gm, P, cfg, receivers, args.recv_stride)
        torch.cuda.synchronize()
        # Untimed: one pass with HIP events around every launch, for the per-kernel breakdown and to
        # find the class with the largest summed time.  Two event records per launch slow the pass
        # down by about 9 %, so the timed steps below record the dominant class only, in every third
        # pass of the executor.
        gm.set_profiling_sample(None, 1)
        gm.set_profiling(True)
        all_edges_pass(gm, P, cfg, receivers, args.recv_stride)
        torch.cuda.synchronize()
        prof = gm.get_profile()
        gm.set_profiling(False)
        dom = max(prof, key=lambda k: prof[k]["ms"])

        gm.set_profiling_sample([dom], 3)
        gm.set_profiling(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n_evals = 0
        for _ in range(args.steps):
            n_evals += all_edges_pass(gm, P, cfg, receivers, args.recv_stride)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        timed = gm.get_profile()[dom]
        gm.set_profiling(False)
        gm.set_profiling_sample(None, 1)
        out["value"] = round(n_evals / dt, 1)
        out["ms_per_step"] = round(1e3 * dt / args.steps, 2)
        out["config"] = {"workload": (f"{args.config}: every edge of the split-QKV graph ({gm.n_edges} edges) evaluated once "
                                      if not spec["n_recv"] else
                                      f"{args.config}: every in-edge of the {len(receivers)} seeded receivers evaluated once ")
                                     + f"at the empty removed set, {args.precision} precision",
                         "B": spec["B"], "S": spec["S"], "batch_edges": args.batch, "recv_stride": args.recv_stride,
                         "edges_per_step": n_evals // args.steps, "seed": spec["seed"]}
        out["roofline"] = roofline_of(dom, timed, prof[dom]["ms"] / sum(v["ms"] for v in prof.values()), args.mma,
                                      traffic_from_profile("all_edges", dom, workload_key) if args.recv_stride == 1 else None,
                                      "HIP events on the library's stream around every launch of this class in every third "
                                      "executor pass of the timed steps")
        out["kernels"] = kernel_table(prof)
        out["kernels_note"] = "per-class HIP-event times of one untimed pass with events around every launch"

    if do("gather_regime") and not args.no_sweep:
        out["gather_regime"] = gather_regime(gm, P, cfg, receivers, torch, workload_key, args.mma)

    if do("sweep") and not args.no_sweep:
        sweeps = {}
        taus = ((1e-4, 3e-5) if args.config == "cfg3" else ()) + tuple(spec["taus"])
        for tau in taus:
            gm.clean_cache(clean, corrupt)
            profiled = tau == taus[0]
            if profiled:
                gm.set_profiling_sample(None, 1)
                gm.set_profiling(True)
            c0 = gm.counters()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            kept, ne, _ = gm.acdc_sweep(tau, receivers=(receivers if spec["n_recv"] else None), trace_cap=0)
            ts = time.perf_counter() - t1
            c1 = gm.counters()
            e = {"s": round(ts, 4), "decisions": int(ne), "kept_edges": int(kept.sum()), "decisions_per_s": round(ne / ts, 1),
                 "device_evaluations": int(c1[0] - c0[0]), "device_batches": int(c1[1] - c0[1])}
            if profiled:
                sp = gm.get_profile()
                gm.set_profiling(False)
                tot = sum(v["ms"] for v in sp.values())
                sd = max(sp, key=lambda k: sp[k]["ms"])
                e["note"] = "timed with HIP events around every launch (about 10 % slower than without)"
                e["roofline"] = roofline_of(sd, sp[sd], sp[sd]["ms"] / tot, args.mma, None, "HIP events around every launch of the sweep")
                e["kernels"] = kernel_table(sp)
            sweeps[str(tau)] = e
        out["sweep"] = sweeps

    if args.only == "policies":
        tau = args.tau if args.tau is not None else 1e-4
        recv = receivers if spec["n_recv"] else None
        res = {}
        for label, sp in (("receiver_side", False), ("sender_side", True)):
            gm.clean_cache(clean, corrupt)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            kept, ne, tr = gm.acdc_sweep(tau, receivers=recv, sender_policy=sp)
            res[label] = (kept.copy(), int(ne), time.perf_counter() - t1, tr)
        ka, kb = res["receiver_side"][0], res["sender_side"][0]
        ta, tb = res["receiver_side"][3], res["sender_side"][3]
        same_prefix = 0
        for x, y in zip(ta, tb):
            if (x["receiver"], x["sender"], x["removed"]) != (y["receiver"], y["sender"], y["removed"]):
                break
            same_prefix += 1
        out["policies"] = {"tau": tau, "edges": int(gm.n_edges),
                           "receiver_side": {"decisions": res["receiver_side"][1], "kept": int(ka.sum()), "s": round(res["receiver_side"][2], 3)},
                           "sender_side": {"decisions": res["sender_side"][1], "kept": int(kb.sum()), "s": round(res["sender_side"][2], 3)},
                           "kept_by_both": int((ka & kb).sum()), "kept_by_one_only": int((ka ^ kb).sum()),
                           "identical_decisions_before_the_first_difference": same_prefix}

    # what this device does on a pure matrix-core issue loop and on a streaming copy, measured now, next to the
    # published peaks the roofline divides by
    if args.fp32_on_host:
        out["fp32_on_host"] = dict(gm.transfer_stats(), workspace_bytes=gm.workspace_bytes,
                                   note="counters since init, over everything this run evaluated")
    tf, gb = P.measure_ceilings()
    out["ceilings"] = {"mfma_f16_issue_loop_TFLOPs": round(tf, 1), "stream_copy_GBps": round(gb, 1),
                       "note": "micro-kernels of the library (pahq_measure_ceilings), all compute units busy"}
    if not args.no_cpu_baseline:
        gm.close()
        out["cpu_baseline"] = cpu_baseline(args.config, shape, w, clean, corrupt)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
