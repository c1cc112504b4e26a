#!/usr/bin/env python3
"""Benchmark of the StructKV scoring / selection / gather sweep on one MI355X.

A step = one pass of the whole hot path over every layer of one synthetic prefill:
for each layer  score_layer -> accumulate_centrality -> select_topk(D, k, keep window) -> gather_kv,
then one select_topk on the accumulated centrality.  Inputs (per-layer Q_win, K, V) are generated
on the GPU before the timed region and stay resident in HBM; each layer has its own buffers.

Prints ONE JSON line: scored KV tokens/s for the whole sweep (median of the timed steps), the roofline of
the dominant kernel against the three units it could be bound by (HBM, bf16 MFMA, vector-ALU issue slots),
timed live with events in a separate profiled sweep of the same sequence, and the CPU oracle timed on a
bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate
# Vector ALU: 256 CUs x 4 SIMDs, one 64-lane instruction per 4 cycles, 2.4 GHz.  v_exp_f32 issues at half that rate
# on this chip (measured: 8.2 cycles per instruction), so it counts as two slots.
VALU_PEAK_GSLOTS = 256 * 4 * 2.4 / 4.0
# The same peak in flops: a slot is one 64-lane instruction, an fma counts 2 -> 78.6 TFLOP/s.  (The data sheet's
# 157.3 TFLOP/s of fp32 vector rate assumes packed fp32, two fmas per lane and slot, which this build does not use.)
VALU_PEAK_TFLOPS = VALU_PEAK_GSLOTS * 64 * 2 / 1e3
VALU_SLOTS_PER_LOGIT = {"score_pass1": 5, "score_pass2": 4}   # scale-fma, exp (2), add, fma  /  mul, exp (2), add


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3_llama8b_128k")
    ap.add_argument("--mode", choices=["graph", "eager"], default="graph",
                    help="graph: the sweep is captured once in a HIP graph and replayed per step")
    ap.add_argument("--overlap", type=int, default=4,
                    help="N >= 2 (default 4): N chains of layers, layer l on stream l mod N (default priority), the "
                         "recurrence kept in layer order by events; 1: selection + gather of layer l on a side "
                         "stream under the scoring of layer l+1; 0: one stream.  Same results bit for bit.")
    ap.add_argument("--separate-calls", action="store_true",
                    help="chains call the four entry points one by one instead of the fused structkv_layer_step")
    ap.add_argument("--profile-steps", type=int, default=3, help="sweeps timed kernel by kernel with events")
    ap.add_argument("--window", type=int, default=0,
                    help="run the workload with another observation window (the paper's default is 8): same keys, the "
                         "queries regenerated for that window; the config line says so")
    ap.add_argument("--pivot", action="store_true",
                    help="also time structkv_score_layer_pivot (scores + the pivot detector's sparsity and variance, "
                         "Eq. 5-6) against structkv_score_layer, per layer, outside the timed region; single sequences")
    ap.add_argument("--cpu-sample-layers", type=int, default=-1,
                    help="layers the CPU oracle is timed on (0 = skip; default: as many, spread evenly over the "
                         "depth, as about 25 s of CPU work allow, at least 2)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU; --gpus %d is not supported "
                         "(sequences and KV heads are independent, so several GPUs would each take a share "
                         "of them and run this same sweep).\n" % args.gpus)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads
    from paper_2604_06746_amd import binding as B
    from paper_2604_06746_amd import sweep as sweep_mod

    wl = workloads.WORKLOADS[args.workload]
    if args.window and args.window != wl.window:
        import dataclasses
        wl = dataclasses.replace(wl, name="%s_w%d" % (wl.name, args.window), window=args.window)
    torch.cuda.set_device(0)
    L = wl.n_layers
    layers = [workloads.make_layer(wl, l, "cuda") for l in range(L)]
    torch.cuda.synchronize()
    sw = sweep_mod.LayerSweep(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.torch_dtype,
                              wl.seq_lens, wl.k_per_seq, lam=wl.lam, n_layers_out=L)

    side_streams = [torch.cuda.Stream() for _ in range(max(args.overlap - 1, 1 if args.overlap else 0))]   # default priority
    side_stream = side_streams[0] if side_streams else None

    def step():
        sw.reset()
        if args.overlap >= 2:
            sw.sweep_chains(((x.q_win, x.k, x.v) for x in layers), side_streams, fused=not args.separate_calls)
        elif side_stream is not None:
            sw.sweep_overlapped(((x.q_win, x.k, x.v) for x in layers), side_stream)
        else:
            for l in range(L):
                x = layers[l]
                sw.layer(x.q_win, x.k, x.v, slot=l)
        sw.select_struct()

    mode = args.mode
    graph = None
    if mode == "graph":
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step()                      # warm every kernel outside capture
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            run = graph.replay
        except Exception as e:  # capture unavailable: time eager launches instead
            sys.stderr.write("bench.py: graph capture failed (%s); timing eager launches\n" % e)
            mode, graph, run = "eager", None, step
    else:
        run = step

    for _ in range(args.warmup):
        run()
    # exactly `steps` steps between two synchronisations; an event between steps gives each step's own time
    stream = torch.cuda.current_stream()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record(stream)
    for i in range(args.steps):
        run()
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_mean = (t1 - t0) * 1e3 / args.steps
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    ms_per_step = step_ms[len(step_ms) // 2] if len(step_ms) % 2 else 0.5 * (step_ms[len(step_ms) // 2 - 1] + step_ms[len(step_ms) // 2])
    tokens_per_step = wl.total_tokens * L
    value = tokens_per_step / (ms_per_step * 1e-3)

    # ---- per-kernel durations: the same sequence, eager, with an event between every kernel ----
    names = ["score_pass1", "score_combine", "score_pass2", "score_reduce", "accumulate", "select_topk", "gather_kv"]
    acc_ms = {k: 0.0 for k in names}
    n_meas = 0
    for rep in range(max(args.profile_steps, 0)):
        sw.reset()
        if rep == 0:
            # Two plain eager sweeps go first, without a synchronisation after them: the chip stays in the state
            # of the timed region (its clock settles over the first sweeps) and the host runs ahead of the GPU,
            # so that no launch gap lands inside a bracket.
            torch.cuda.synchronize()
            for _ in range(2):
                for l in range(L):
                    sw.layer(layers[l].q_win, layers[l].k, layers[l].v, slot=l)
            sw.reset()
        evs = []
        for l in range(L):
            x = layers[l]
            e = [torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)]
            e[0].record(stream)
            for i, mask in enumerate((1, 2, 4, 8)):
                B.structkv_debug_score_steps(sw.shape, x.q_win, x.k, sw.cu, sw.indeg, sw.entropy,
                                             sw.entropy_per_head, sw.workspace, mask)
                e[i + 1].record(stream)
            sw.accumulate(); e[5].record(stream)
            sw.select_kv(); e[6].record(stream)
            sw.gather(x.k, x.v, l); e[7].record(stream)
            evs.append(e)
        all_evs = (all_evs if rep else []) + evs
    if args.profile_steps > 0:
        torch.cuda.synchronize()
        for e in all_evs:
            for i, k in enumerate(names):
                acc_ms[k] += e[i].elapsed_time(e[i + 1])
        n_meas = len(all_evs)
    kern_us = {k: (1e3 * v / n_meas if n_meas else None) for k, v in acc_ms.items()}

    # ---- a plain device-to-device copy, as the practical HBM ceiling beside the data-sheet peak ----
    copy_gbs = None
    if n_meas:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        ce = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ce[0].record(stream)
        for _ in range(5):
            dst.copy_(src)
        ce[1].record(stream)
        torch.cuda.synchronize()
        copy_gbs = 5 * 2.0 * src.numel() / (ce[0].elapsed_time(ce[1]) * 1e-3) / 1e9     # bytes read + written
        del src, dst

    k_bytes = wl.n_kv_heads * wl.head_dim * wl.elem_bytes * wl.total_tokens       # K read once, per launch
    rows = sum(k + wl.window for k in wl.k_per_seq)
    gather_bytes = 2 * 2 * rows * wl.n_kv_heads * wl.head_dim * wl.elem_bytes + 4 * rows
    roofline = None
    extra = {}
    if n_meas:
        dom = "score_pass1" if kern_us["score_pass1"] >= kern_us["score_pass2"] else "score_pass2"
        t_dom = kern_us[dom] * 1e-6
        hbm_gbs = k_bytes / t_dom / 1e9
        qk_flops = 2.0 * wl.n_q_heads * wl.window * wl.total_tokens * wl.head_dim      # Q_win K^T of one pass
        mfma_tf = qk_flops / t_dom / 1e12
        # wave-wide vector instruction slots the softmax of one pass needs at least (one lane per logit)
        valu_slots = VALU_SLOTS_PER_LOGIT[dom] * wl.n_q_heads * wl.window * wl.total_tokens / 64.0
        valu_gs = valu_slots / t_dom / 1e9
        units = {
            "hbm": {"achieved": round(hbm_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(hbm_gbs / HBM_PEAK_GBS, 4), "algorithmic_bytes_per_launch": k_bytes},
            "mfma": {"achieved": round(mfma_tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(mfma_tf / MFMA_BF16_PEAK_TFLOPS, 4), "flops_per_launch": qk_flops},
            "alu": {"achieved": round(valu_gs * 128 / 1e3, 2), "peak": round(VALU_PEAK_TFLOPS, 2), "unit": "TFLOP/s",
                    "frac": round(valu_gs / VALU_PEAK_GSLOTS, 4), "slots_per_logit": VALU_SLOTS_PER_LOGIT[dom],
                    "slots_per_launch": valu_slots, "achieved_Gslots": round(valu_gs, 1),
                    "peak_Gslots": VALU_PEAK_GSLOTS,
                    "note": "issue slots of the softmax's own instructions, one slot = one 64-lane instruction = "
                            "128 flop at fma counting; un-packed fp32 peak (the data sheet's 157.3 assumes packed fp32)"},
        }
        # the unit that binds: the one the kernel uses the largest fraction of
        binds = max(units, key=lambda u: units[u]["frac"])
        traffic, traffic_source = None, None
        tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
        if os.path.exists(tpath):
            try:
                prof = json.load(open(tpath))
                # counters of an earlier rocprofv3 --pmc run of pmc_workload.py, not of this run: only quoted
                # while the library is the one that was profiled
                if prof.get("_library_version") == B.structkv_version():
                    traffic = prof.get(wl.name, {}).get(dom)
                    if traffic is not None:
                        traffic_source = ("profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of "
                                          "pmc_workload.py; not measured in this run)")
            except Exception:
                traffic = None
        score_us = sum(kern_us[k] for k in names[:4])
        roofline = {"bound": binds, "binds": binds, "kernel": dom, "achieved": units[binds]["achieved"],
                    "peak": units[binds]["peak"], "unit": units[binds]["unit"], "frac": units[binds]["frac"],
                    "traffic": traffic, "traffic_source": traffic_source, "avg_launch_us": round(kern_us[dom], 2),
                    "hbm": units["hbm"], "mfma": units["mfma"], "alu": units["alu"],
                    # the K stream with K counted ONCE per token per layer, over all four scoring kernels
                    "k_once_all_scoring_kernels": {"achieved": round(k_bytes / (score_us * 1e-6) / 1e9, 1),
                                                   "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                                   "frac": round(k_bytes / (score_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)},
                    "measured_copy_GBs": round(copy_gbs, 1), "hbm_frac_of_measured_copy": round(hbm_gbs / copy_gbs, 4)}
        extra = {
            "kernel_us": {k: round(v, 2) for k, v in kern_us.items()},
            "kernel_us_note": "each kernel alone on one stream, eager, an event on either side; the timed steps "
                              "run the layers as chains on several streams, where kernels share the chip",
            "gather": {"achieved_GBs": round(gather_bytes / (kern_us["gather_kv"] * 1e-6) / 1e9, 1),
                       "frac": round(gather_bytes / (kern_us["gather_kv"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                       "algorithmic_bytes_per_launch": gather_bytes},
        }

    # ---- the pivot detector's metrics from the same scoring pass (optional; not part of the timed sweep) ----
    if args.pivot:
        x = layers[min(3, L - 1)]

        def per_call_us(f, reps=30):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                f()
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps * 1e3

        sw.score_pivot(x.q_win, x.k)                      # allocates the scratch
        for _ in range(3):                                # the clock settles over the first few hundred calls
            per_call_us(lambda: sw.score(x.q_win, x.k), 60)
        t_score = min(per_call_us(lambda: sw.score(x.q_win, x.k)) for _ in range(3))
        t_pivot = min(per_call_us(lambda: sw.score_pivot(x.q_win, x.k)) for _ in range(3))
        t_score = min(t_score, min(per_call_us(lambda: sw.score(x.q_win, x.k)) for _ in range(3)))
        extra["pivot"] = {"score_layer_us": round(t_score, 1), "score_layer_pivot_us": round(t_pivot, 1),
                          "ratio": round(t_pivot / t_score, 3),
                          "note": "calls launched back to back on one stream, 30 per bracket, best of 3 brackets"}

    # ---- CPU oracle on a bounded sample of the same workload ----
    cpu = None
    if args.cpu_sample_layers != 0:
        import oracle
        to_oracle_array = workloads.to_oracle_array
        if args.cpu_sample_layers > 0:
            ns = min(args.cpu_sample_layers, L)
        else:   # ~25 s of oracle time: it scores about 3.6e5 tokens/s at a window of 64 on 16 threads
            est_layer_s = wl.total_tokens * (wl.window / 64.0) / 3.6e5
            ns = min(L, max(2, int(25.0 / max(est_layer_s, 1e-3))))
        sample = sorted(set(int(round(i * (L - 1) / max(ns - 1, 1))) for i in range(ns)))
        C = np.zeros(wl.total_tokens)
        cpu_s = 0.0
        for l in sample:
            x = layers[l]
            qh, kh, vh = to_oracle_array(x.q_win), to_oracle_array(x.k), to_oracle_array(x.v)
            c0 = time.perf_counter()
            D, ent, _, _ = oracle.score_layer(qh, kh, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window,
                                              wl.seq_lens)
            oracle.accumulate(C, D, wl.lam, 1.0 / wl.window)
            idx = oracle.select_topk(D, wl.seq_lens, wl.k_per_seq, wl.window)
            oracle.gather_kv(kh, idx, wl.seq_lens)
            oracle.gather_kv(vh, idx, wl.seq_lens)
            cpu_s += time.perf_counter() - c0
        cpu = {"value": round(wl.total_tokens * len(sample) / cpu_s, 1), "unit": "scored KV tokens/s",
               "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "%d of %d layers (%s) of %s, all tokens; %.1f s%s" % (
                   len(sample), L, sample, wl.name, cpu_s,
                   "" if len(sample) == L else "; whole sweep extrapolated: %.0f s" % (cpu_s * L / len(sample)))}

    out = {
        "metric": "scored KV tokens/s per layer sweep (score+top-k+gather)",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_stat": "median of the timed steps (an event between steps)",
        "ms_per_step_mean": round(ms_mean, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "layers": L, "n_q_heads": wl.n_q_heads, "n_kv_heads": wl.n_kv_heads,
                   "head_dim": wl.head_dim, "seq_lens": list(wl.seq_lens) if wl.batch > 1 else wl.seq_lens[0],
                   "window": wl.window, "k": list(wl.k_per_seq) if wl.batch > 1 else wl.k_per_seq[0],
                   "launch": mode, "streams": max(args.overlap, 2) if args.overlap else 1,
                   "stream_plan": {0: "one stream", 1: "selection and gather on a side stream"}.get(
                       args.overlap, "%d chains of layers, one stream each" % args.overlap)},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    out.update(extra)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
