"""Benchmark of the hot path: build taskgraph -> compile memgraph under the GPU-memory cap ->
event-driven execution on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2]

One "step" is one execution of the whole memgraph of the workload (all vertex kinds, all
transfers the memgraph contains) on one batch of seeded synthetic input; inputs that the
workload declares device-resident are placed in HBM before the timed region.  Prints ONE JSON
line: tokens/s under the cap, plus the roofline of the dominant kernel (bf16 MFMA tile GEMM),
measured with HIP events on the streams the kernels run on, and the CPU oracle timed on a
bounded sample as a baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6  # MI355X dense bf16 MFMA (256 CUs x 4096 flop/clk x 2.4 GHz)
PEAK_FP32_TFLOPS = 157.3
HOST_LINK_GBS = 64.0  # PCIe Gen5 x16, per direction


def cpu_baseline(cfg, full, budget_tokens):
    """The untiled float64 oracle on the first `budget_tokens` tokens (a causal prefill's first
    rows equal the model run on the prefix), timed on this machine's host cores."""
    import numpy as np
    from oracle import llama_ref as R
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    seen, w = {}, {}
    for k, a in full.items():  # layers that share their weights share the widened copy
        if id(a) not in seen:
            seen[id(a)] = R.widen_array(a)
        w[k] = seen[id(a)]
    t0 = time.perf_counter()
    y = R.forward(cfg, w, n_tokens_prefix=budget_tokens)
    dt = time.perf_counter() - t0
    assert np.isfinite(y).all()
    return {"value": budget_tokens * cfg.batch / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"untiled float64 oracle on the first {budget_tokens} tokens (causal prefix) of {cfg.name}, "
                      f"all {cfg.layers} layer(s), {dt:.1f} s"}, y


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--streams", type=int, default=0, help="compute streams; default: harness.BENCH_COMPUTE_STREAMS")
    ap.add_argument("--max-batch", type=int, default=1920)
    ap.add_argument("--max-transfers", type=int, default=0)
    ap.add_argument("--max-gemm-inflight", type=int, default=2)
    ap.add_argument("--queue-depth", type=int, default=3)
    ap.add_argument("--policy", default="by_order", choices=["fifo", "lifo", "random", "by_order", "in_order"])
    ap.add_argument("--max-delay-us", type=int, default=0, help="inject a pseudo-random delay of up to this many microseconds into every transfer group")
    ap.add_argument("--cpu-tokens", type=int, default=4096, help="tokens of the CPU-oracle sample; 0 = skip")
    ap.add_argument("--capped", action="store_true",
                    help="add a run with everything streamed from the host under 40 %% of the uncapped peak (offload path)")
    ap.add_argument("--no-capped", action="store_true", help=argparse.SUPPRESS)  # the default now
    ap.add_argument("--order", default="tiler", choices=["tiler", "level"],
                    help="serial order given to the compiler: the tiler's (stripe by stripe) or level by level")
    ap.add_argument("--evict-ahead-mb", type=int, default=-1,
                    help="compile option evict_ahead_bytes in MiB; default 0, for the fine-tuning step 1/32 of the cap")
    ap.add_argument("--checkpoint", action="store_true",
                    help="fine-tuning step with activation checkpointing: the reverse pass of a layer forms that "
                         "layer's forward tensors again instead of reading saved ones")
    ap.add_argument("--materialize-scores", action="store_true",
                    help="attention with scores and probabilities as taskgraph tensors and the softmax in two portions; "
                         "sets the tile to the head dimension (one head per column tile)")
    ap.add_argument("--host-outputs", type=int, default=-1,
                    help="1: marked outputs are stored to pinned host memory inside the timed step; 0: they are copied to a "
                         "buffer in GPU memory outside the capped device buffer.  Default: 0 when the inputs are device-resident "
                         "(the step begins and ends in HBM), 1 when weights are streamed from the host")
    ap.add_argument("--host-inputs", action="store_true",
                    help="weights and x start in pinned host memory and are loaded under the cap (c2 keeps them on the GPU)")
    ap.add_argument("--k-split", type=int, default=0,
                    help="cut every projection along K into this many partial products joined by a sum vertex (increments "
                         "into a write-locked output); 0 = the whole K range inside one GEMM vertex")
    ap.add_argument("--lookahead-mb", type=int, default=-1,
                    help="compile option max_lookahead_bytes in MiB; default unbounded, for the fine-tuning step a quarter of the cap")
    ap.add_argument("--next-fit", type=int, default=-1, help="compile option next_fit; default 0, for the fine-tuning step 1")
    ap.add_argument("--cap-gb", type=float, default=0.0, help="GPU-memory cap in GB instead of the workload's own")
    ap.add_argument("--copy-engine", default="auto", choices=["auto", "memcpy", "kernel"])
    ap.add_argument("--copy-workgroups", type=int, default=0)
    ap.add_argument("--transfer-depth", type=int, default=0)
    ap.add_argument("--train", type=int, default=-1,
                    help="1: fine-tuning step (adapters of rank 16 on q and v, probe loss, reverse pass); default: only for c5")
    ap.add_argument("--layers", type=int, default=0, help="run the workload's shape with this many layers instead of its own")
    ap.add_argument("--distinct-layers", type=int, default=-1,
                    help="layers with weights of their own (the others reuse them); default: all up to 8 layers, else 4")
    ap.add_argument("--kv-outputs", type=int, default=-1, help="K/V of every layer are outputs; default: only when weights are streamed")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2405_16283_amd import binding as B
    from paper_2405_16283_amd import harness as H
    from workloads import bf16_bits_to_f32, config, make_llama_inputs, make_lora_inputs
    if args.streams <= 0:
        args.streams = H.BENCH_COMPUTE_STREAMS

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    t_begin = time.perf_counter()
    cfg = config(args.workload)
    if args.layers > 0:
        cfg = cfg.with_(layers=args.layers)
    if args.cap_gb > 0:
        cfg = cfg.with_(cap_bytes=int(args.cap_gb * 1e9), cap_frac=0.0)
    if args.materialize_scores:
        cfg = cfg.with_(tile=cfg.head_dim)
    if args.host_inputs:
        cfg = cfg.with_(weights_resident=False, x_resident=False)
    train = bool(args.train) if args.train >= 0 else cfg.name == "c5"
    t0 = time.perf_counter()
    distinct = args.distinct_layers if args.distinct_layers >= 0 else (0 if cfg.layers <= 8 else 4)
    kv_outputs = bool(args.kv_outputs) if args.kv_outputs >= 0 else (cfg.layers > 1 and not cfg.weights_resident)
    full = make_llama_inputs(cfg, 0, distinct_layers=distinct, workers=16)
    if train:
        kv_outputs = False
        full.update(make_lora_inputs(cfg, 0, rank=16, b_std=0.0))
    t_gen = time.perf_counter() - t0

    def note(msg):
        print(f"[bench {time.perf_counter() - t_begin:7.1f}s] {msg}", file=sys.stderr, flush=True)

    def timed(session, steps, warmup, opts):
        reps = []
        for i in range(warmup + steps):
            session.place_inputs()  # device-resident inputs go to HBM outside the timed region
            torch.cuda.synchronize()
            t = time.perf_counter()
            rep = session.execute(opts)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t
            note(f"step {i + 1} of {warmup + steps}: {dt * 1e3:.1f} ms")
            if i >= warmup:
                reps.append((dt, rep))
        return reps

    t0 = time.perf_counter()
    # where the marked outputs go: GPU memory when the step also starts there, else pinned host memory
    device_outputs = (cfg.weights_resident and cfg.x_resident) if args.host_outputs < 0 else not args.host_outputs

    def session(c, pressed=False, device_outputs=False, level=False):
        order = None
        if pressed:  # the cap is a fraction of the uncapped peak: the compile options need it in bytes
            tg = B.tn_build_llama(H.llama_config_struct(c, kv_outputs, lora_rank=16 if train else 0, train=train,
                                                        k_split=args.k_split, materialize_scores=args.materialize_scores,
                                                        checkpoint=args.checkpoint))
            c = c.with_(cap_bytes=H.cap_for(c, tg), cap_frac=0.0)
            B.tn_taskgraph_destroy(tg)
        if args.order == "level" or level:
            tg = B.tn_build_llama(H.llama_config_struct(c, kv_outputs, lora_rank=16 if train else 0, train=train,
                                                        k_split=args.k_split, materialize_scores=args.materialize_scores,
                                                        checkpoint=args.checkpoint))
            order = H.level_major_order(tg)
            B.tn_taskgraph_destroy(tg)
        cap = c.cap_bytes or 0  # only the fine-tuning workload uses it, and that one states its cap in bytes
        copts = H.bench_compile_opts(cap, train,
                                     lookahead=args.lookahead_mb << 20 if args.lookahead_mb >= 0 else None,
                                     evict_ahead=args.evict_ahead_mb << 20 if args.evict_ahead_mb >= 0 else None,
                                     next_fit=args.next_fit if args.next_fit >= 0 else None, pressed=pressed)
        return H.GpuSession(c, full, n_compute=args.streams, kv_outputs=kv_outputs, order=order, compile_opts=copts,
                            lora_rank=16 if train else 0, train=train, progress=note, k_split=args.k_split,
                            materialize_scores=args.materialize_scores, checkpoint=args.checkpoint,
                            device_outputs=device_outputs)

    note("inputs generated")
    s = session(cfg, device_outputs=device_outputs)
    t_compile = time.perf_counter() - t0
    note(f"compiled and executor created: {int(s.stats.n_vertices)} memgraph vertices, {int(s.stats.n_offload)} offloads, "
         f"{int(s.stats.n_load)} loads")
    policy = {"fifo": B.TN_POLICY_FIFO, "lifo": B.TN_POLICY_LIFO, "random": B.TN_POLICY_RANDOM,
              "by_order": B.TN_POLICY_BY_ORDER, "in_order": B.TN_POLICY_IN_ORDER}[args.policy]
    engine = {"auto": B.TN_COPY_AUTO, "memcpy": B.TN_COPY_MEMCPY, "kernel": B.TN_COPY_KERNEL}[args.copy_engine]
    opts = B.tn_exec_opts(policy=policy, max_batch=args.max_batch, profile=1, max_transfers=args.max_transfers,
                          max_gemm_inflight=args.max_gemm_inflight, queue_depth=args.queue_depth, copy_engine=engine,
                          copy_workgroups=args.copy_workgroups, max_delay_us=args.max_delay_us, delay_seed=7,
                          transfer_depth=args.transfer_depth)
    reps = timed(s, args.steps, args.warmup, opts)
    ms = 1e3 * sum(dt for dt, _ in reps) / len(reps)
    # unprofiled steps, to show what the event pairs around every launch cost
    plain_opts = B.tn_exec_opts(policy=policy, max_batch=args.max_batch, max_transfers=args.max_transfers,
                                max_gemm_inflight=args.max_gemm_inflight, queue_depth=args.queue_depth, copy_engine=engine,
                                copy_workgroups=args.copy_workgroups, max_delay_us=args.max_delay_us, delay_seed=7,
                                transfer_depth=args.transfer_depth)
    plain = timed(s, max(1, min(3, args.steps), args.steps // 4), 1 if args.steps > 1 else 0, plain_opts)
    ms_plain = 1e3 * sum(dt for dt, _ in plain) / len(plain)
    y = s.outputs(only=["y"])["y"]
    # the same step with the outputs stored to pinned host memory (the rate that includes the host link)
    ms_host_out = None
    if device_outputs:
        sh = session(cfg, device_outputs=False)
        rh = timed(sh, max(3, args.steps // 4), 1, opts)
        ms_host_out = 1e3 * sum(dt for dt, _ in rh) / len(rh)
        assert np.array_equal(sh.outputs(only=["y"])["y"], y)
        sh.close()
    st = s.stats
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_FP32_TFLOPS
    gemm_ms = sum(r.gemm_ms for _, r in reps)
    gemm_launches = sum(r.gemm_launches for _, r in reps)
    gemm_flops = sum(r.gemm_flops for _, r in reps)
    attn_ms = sum(r.attn_ms for _, r in reps)
    attn_flops = sum(r.attn_flops for _, r in reps)
    ew_ms = sum(r.ewise_ms for _, r in reps)
    ew_bytes = sum(r.ewise_bytes for _, r in reps)
    rep0 = reps[-1][1]
    achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    total_flops = rep0.gemm_flops + rep0.attn_flops
    # HBM bytes per GEMM launch from the rocprofv3 --pmc runs recorded under profiles/ (FETCH_SIZE
    # and WRITE_SIZE in KiB per dispatch, scaled by the copy-kernel calibration)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"{cfg.name}_gemm_traffic.txt")
    if os.path.exists(tpath):
        kv = dict(l.split() for l in open(tpath) if l.strip() and not l.startswith("#"))
        traffic = 1024.0 * (float(kv["fetch_kib_per_launch"]) / float(kv["fetch_scale"])
                            + float(kv["write_kib_per_launch"]) / float(kv["write_scale"]))
    line = {
        "metric": "tokens/s under GPU-RAM cap", "value": cfg.tokens / (ms * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.layers}-layer LLaMA-shaped "
                               + ("fine-tuning step (rank-16 adapters on q and v, forward + backward)" if train else "prefill")
                               + f", d {cfg.d_model}, "
                               f"{cfg.n_heads}x{cfg.head_dim} heads, ffn {cfg.ffn}, seq {cfg.seq}, batch {cfg.batch}, "
                               f"tile {cfg.tile}, attention block {cfg.attn_block}",
                   "distinct_layers": distinct or cfg.layers, "kv_outputs": kv_outputs,
                   "gpu_cap_bytes": s.cap, "weights": "device-resident" if cfg.weights_resident else "streamed from pinned host",
                   "outputs": "GPU memory outside the capped buffer" if device_outputs else "pinned host memory",
                   "compute_streams": args.streams, "ready_policy": args.policy, "max_batch": args.max_batch,
                   "max_gemm_inflight": args.max_gemm_inflight, "queue_depth": args.queue_depth, "copy_engine": args.copy_engine, "max_delay_us": args.max_delay_us, "serial_order": args.order, "k_split": args.k_split, "materialize_scores": bool(args.materialize_scores), "checkpoint": bool(args.checkpoint), "memgraph_vertices": int(st.n_vertices),
                   "offloads": int(st.n_offload), "reloads": int(st.n_reload), "loads": int(st.n_load),
                   "offload_GB": st.offload_bytes / 1e9, "load_GB": st.load_bytes / 1e9, "mem_edges": int(st.n_mem_edges)},
        "roofline": {"bound": "mfma", "kernel": "gemm_bf16_nt256_kernel" if cfg.dtype == "bf16" else "gemm_generic_kernel",
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": traffic,
                     "avg_launch_ms": gemm_ms / max(1, gemm_launches),
                     "flops_per_launch": gemm_flops / max(1, gemm_launches)},
        "extra": {
            "ms_per_step_without_event_pairs": ms_plain,
            "ms_per_step_with_outputs_stored_to_host": ms_host_out,
            "tokens_per_s_with_outputs_stored_to_host": cfg.tokens / (ms_host_out * 1e-3) if ms_host_out else None,
            "tokens_per_s_without_event_pairs": cfg.tokens / (ms_plain * 1e-3),
            "whole_run_tflops": total_flops / (ms * 1e-3) / 1e12,
            "whole_run_frac_of_mfma_peak": total_flops / (ms * 1e-3) / 1e12 / peak,
            "attention_tflops": attn_flops / (attn_ms * 1e-3) / 1e12 if attn_ms > 0 else None,
            "elementwise_GBs": ew_bytes / (ew_ms * 1e-3) / 1e9 if ew_ms > 0 else None,
            "kernel_launches_per_step": int(rep0.n_kernel_launches),
            "gpu_idle_frac": rep0.idle_frac,
            "kernel_busy_ms": rep0.kernel_busy_ms, "gemm_ms": rep0.gemm_ms, "attn_ms": rep0.attn_ms,
            "ewise_ms": rep0.ewise_ms, "h2d_ms": rep0.h2d_ms, "d2h_ms": rep0.d2h_ms,
            "h2d_GBs_while_copying": rep0.h2d_bytes / (rep0.h2d_ms * 1e-3) / 1e9 if rep0.h2d_ms > 0 else None,
            "d2h_GBs_while_copying": rep0.d2h_bytes / (rep0.d2h_ms * 1e-3) / 1e9 if rep0.d2h_ms > 0 else None,
            "launches_per_step": int(rep0.n_launches),
            "d2h_GBs_over_wall": rep0.d2h_bytes / (ms * 1e-3) / 1e9,
            "h2d_GBs_over_wall": rep0.h2d_bytes / (ms * 1e-3) / 1e9,
            "input_generation_s": t_gen, "build_and_compile_s": t_compile,
        },
    }
    s.close()

    # the same shape with everything streamed from the host and the cap at 40 % of the uncapped
    # peak, so that the offload/reload path carries real traffic
    if args.capped and cfg.cap_bytes:
        cfg2 = cfg.with_(cap_bytes=0, cap_frac=0.40, weights_resident=False, x_resident=False)
        # level-by-level serial order: every weight tile is loaded once per step, where the tiler's
        # stripe-by-stripe order loads the feed-forward weights once per row tile
        s2 = session(cfg2, pressed=True, level=True)
        r2 = timed(s2, max(3, args.steps // 4), 1, opts)
        ms2 = 1e3 * sum(dt for dt, _ in r2) / len(r2)
        rr = r2[-1][1]
        y2 = s2.outputs(only=["y"])["y"]
        line["capped40"] = {
            "gpu_cap_bytes": s2.cap, "serial_order": "level", "ms_per_step": ms2, "tokens_per_s": cfg.tokens / (ms2 * 1e-3),
            "offloads": int(s2.stats.n_offload), "reloads": int(s2.stats.n_reload), "loads": int(s2.stats.n_load),
            "h2d_GBs_over_wall": rr.h2d_bytes / (ms2 * 1e-3) / 1e9, "d2h_GBs_over_wall": rr.d2h_bytes / (ms2 * 1e-3) / 1e9,
            "h2d_frac_of_link": rr.h2d_bytes / (ms2 * 1e-3) / 1e9 / HOST_LINK_GBS,
            "gpu_idle_frac": rr.idle_frac, "identical_to_uncapped_run": bool(np.array_equal(y, y2)),
        }
        s2.close()

    if args.cpu_tokens > 0:
        from oracle import llama_ref as R
        n = min(args.cpu_tokens, cfg.seq)
        base, y_cpu = cpu_baseline(cfg, full, n)
        line["cpu_baseline"] = base
        yy = (bf16_bits_to_f32(y) if cfg.dtype == "bf16" else y).astype(np.float64)
        rows = np.concatenate([np.arange(b * cfg.seq, b * cfg.seq + n) for b in range(cfg.batch)])
        line["extra"]["rel_err_vs_untiled_oracle_on_cpu_sample"] = R.rel_err(yy[rows], y_cpu)
    else:
        line["cpu_baseline"] = None
    print(json.dumps(line))


if __name__ == "__main__":
    main()
