#!/usr/bin/env python3
"""Benchmark of the stage hot path on one MI355X.

Headline workload (N = 1): `l70_full`, the largest configuration that fits one GPU -- the full-width
Llama-2-70B stage (TP degree 1, all 80 layers, 136.9 GB of bf16 weights), 32 ragged prompts of 128..4096 tokens
prefilled, then decoded one token per sequence and step against the ragged KV cache.
  * One timed "step" = one decode call of the whole stage for the batch of 32 (all 80 layers: RMSNorm, QKV, RoPE +
    cache append, GQA attention, W_O, RMSNorm, W1/W3 + SwiGLU, W2).  `value` = decode tokens/s of the stage.
  * The prefill of the 32 prompts that precedes the decode steps is timed on its own (it is one call of about nine
    seconds) and reported next to it: `prefill_tokens_per_s`, and the `prefill` object (GEMMs against the bf16 MFMA peak).
  * `configs` carries the same figures -- tokens/s, microseconds per layer, roofline fraction -- for every 70B-shaped
    configuration of the task: TP2 batch-1 decode, TP4 prefill + decode, TP8 batch-16 decode, and the full stage.
Inputs and weights are synthetic (seeded normal draws) and resident in HBM before any timed region.

Prints ONE JSON line.  Besides the contract fields it carries
  roofline     -- the dominant kernel of the timed region (the W1/W3 weight-streaming decode projection) against the
                  8 TB/s HBM peak, timed with HIP events on the launch stream in an instrumented pass of its own;
  roofline_prefill -- the dominant kernel of the prefill (the W1/W3 GEMM) against the bf16 MFMA peak, same method;
  cpu_baseline -- the float64 CPU oracle timed on a bounded sample of the same workload, scaled to the same unit.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_PEAK_TFLOPS = 2516.6      # MI355X published dense bf16 rate
PROF_QKV, PROF_WO, PROF_W13, PROF_W2, PROF_ATTN, PROF_CALL, PROF_W13_MAIN = range(7)
SLOT_NAMES = (("qkv", PROF_QKV), ("wo", PROF_WO), ("w13", PROF_W13), ("w2", PROF_W2), ("attn", PROF_ATTN))


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def measured_traffic(workload):
    """HBM bytes per launch of the dominant decode kernel as measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE
    scaled by a copy of known size) in an EARLIER run, read from the committed summary of that run; (None, None)
    when no summary for this workload exists.  The figure is not measured by this run: the source file is named
    beside it in the JSON."""
    path = os.path.join(ROOT, "profiles", f"{workload}_pmc_traffic.txt")
    try:
        m = re.search(r"^traffic_bytes_per_launch\s+(\S+)\s+(\d+)", open(path).read(), flags=re.M)
    except OSError:
        return None, None
    return (int(m.group(2)), f"profiles/{os.path.basename(path)} ({m.group(1)})") if m else (None, None)


# ------------------------------------------------------------------------------------------------------------------
class Bench:
    """One stage resident on the GPU with its cache; the legs below time it."""

    def __init__(self, torch, hx, generate, cfg, max_decode_steps, keep_layers=()):
        self.torch, self.hx, self.generate, self.cfg = torch, hx, generate, cfg
        self.rank = cfg.tp_ranks[0]
        self.td = {"bf16": torch.bfloat16, "f16": torch.float16}[cfg.dtype]
        t0 = time.time()
        self.st = hx.Stage(cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, cfg.n_layers, cfg.tp_degree, self.rank,
                           cfg.dtype, cfg.rms_eps, cfg.rope_theta)
        self.host_layers = {}
        for l in range(cfg.n_layers):
            w = generate.layer_weights(cfg, l, device="cuda")
            self.st.load_layer(l, *[w[k] for k in generate.LAYER_TENSOR_ORDER])
            if l in keep_layers:
                self.host_layers[l] = {k: v.cpu() for k, v in w.items()}
            del w
        self.b = cfg.batch
        if cfg.kv_context is not None:
            self.lens = [cfg.kv_context] * self.b
        else:
            self.lens = generate.prompt_lengths(cfg)
        self.kv = self.st.kv_cache_create(self.b, max(self.lens) + max_decode_steps + 1)
        if cfg.kv_context is not None:
            for l in range(cfg.n_layers):
                for s in range(self.b):
                    k, v = generate.synthetic_kv(cfg, l, s, cfg.kv_context, device="cuda")
                    self.kv.fill(l, s, k.cpu(), v.cpu())
        n_x = max_decode_steps
        self.X = torch.stack([generate.hidden_rows(cfg, self.b, stream_id=1 + i, device="cuda") for i in range(n_x)])
        self.X = self.X.to(self.td).contiguous()
        self.outp = torch.empty(self.b, cfg.hidden, dtype=self.td, device="cuda")
        self.outr = torch.empty_like(self.outp)
        torch.cuda.synchronize()
        log(f"{cfg.name}: setup {time.time() - t0:.1f}s, weights {self.st.weight_bytes() / 1e9:.3f} GB")

    # ---- prefill ---------------------------------------------------------------------------------------------
    def prefill(self, reps, warm=1):
        torch, cfg, st = self.torch, self.cfg, self.st
        T = sum(self.lens)
        Xp = self.generate.hidden_rows(cfg, T, device="cuda").to(self.td).contiguous()
        outp, outr = torch.empty_like(Xp), torch.empty_like(Xp)
        for _ in range(warm):
            st.prefill(self.kv, Xp, self.lens, outp, outr)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            st.prefill(self.kv, Xp, self.lens, outp, outr)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / reps
        assert torch.isfinite(outp.float()).all() and torch.isfinite(outr.float()).all()
        # the instrumented pass follows at least 0.2 s of the same work: after a pause the part takes some tens of
        # milliseconds to reach the clocks it then sustains, and a short call measured right away reads 10 % slow
        for _ in range(min(32, int(0.2 / dt)) if dt * (reps + warm) < 0.2 else 0):
            st.prefill(self.kv, Xp, self.lens, outp, outr)
        st.profile_enable(0b11111)
        st.prefill(self.kv, Xp, self.lens, outp, outr)
        H, d = cfg.hidden, cfg.head_dim
        flops = {"qkv": 2 * T * H * (cfg.hq_l + 2 * cfg.hkv_l) * d, "wo": 2 * T * cfg.hq_l * d * H,
                 "w13": 2 * T * H * 2 * cfg.ffn_l, "w2": 2 * T * cfg.ffn_l * H}
        gemm, tot_f, tot_t = {}, 0.0, 0.0
        for name, slot in SLOT_NAMES:
            ms, n = st.profile_read(slot)
            us = ms / max(n, 1) * 1e3
            if name == "attn":
                gemm["attn"] = {"avg_us": round(us, 1)}
                continue
            gemm[name] = {"avg_us": round(us, 1), "TFLOPs": round(flops[name] / us / 1e6, 1),
                          "frac": round(flops[name] / us / 1e6 / MFMA_PEAK_TFLOPS, 4), "launches": n}
            tot_f += flops[name]
            tot_t += us
        st.profile_enable(0)
        del Xp, outp, outr
        layer_flops = sum(flops.values()) + sum(2 * n * n * d * cfg.hq_l for n in self.lens)
        self.prefill_w13 = (flops["w13"], gemm["w13"]["avg_us"], gemm["w13"]["launches"])
        return {"rows": T, "sequences": self.b, "tokens_per_s": round(T / dt, 1), "ms_per_call": round(dt * 1e3, 3),
                "us_per_layer": round(dt * 1e6 / cfg.n_layers, 1), "reps": reps,
                "stage_mfma_frac": round(layer_flops * cfg.n_layers / dt / 1e12 / MFMA_PEAK_TFLOPS, 4),
                "gemm_mfma_frac": round(tot_f / tot_t / 1e6 / MFMA_PEAK_TFLOPS, 4), "gemm": gemm}

    # ---- decode ----------------------------------------------------------------------------------------------
    def run_decode(self, n):
        """n decode steps from the context the workload starts its decode phase with; returns seconds.
        Bracketed by a device synchronisation on both sides (one process, one GPU: no rank barrier exists)."""
        self.kv.set_lengths(self.lens)
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            self.st.decode(self.kv, i, self.X[i], self.outp, self.outr)
        self.torch.cuda.synchronize()
        return time.perf_counter() - t0

    def decode(self, steps, warmup):
        cfg = self.cfg
        self.run_decode(warmup)
        dt = self.run_decode(steps)
        assert self.torch.isfinite(self.outp.float()).all() and self.torch.isfinite(self.outr.float()).all()
        # algorithmic bytes of a step: every weight once + the K / V rows of every sequence's context (which grows
        # by one position per step)
        kv_pos = sum(n + (steps + 1) / 2.0 for n in self.lens)
        step_bytes = cfg.n_layers * (cfg.weight_elems_per_layer_rank * 2 + cfg.kv_bytes_per_pos_layer() * kv_pos)
        return dt, {"batch": self.b, "steps": steps, "tokens_per_s": round(self.b * steps / dt, 2),
                    "ms_per_step": round(dt / steps * 1e3, 4),
                    "us_per_layer": round(dt / steps * 1e6 / cfg.n_layers, 2),
                    "hbm_frac": round(step_bytes / (dt / steps) / 1e9 / HBM_PEAK_GBS, 4),
                    "GB_per_step": round(step_bytes / 1e9, 3)}

    def decode_kernels(self, steps):
        """Instrumented passes (HIP events recorded by the library on the launch stream): first the main kernel of
        the W1/W3 projection alone, so that its figure carries no other event's overhead, then every projection."""
        cfg, st = self.cfg, self.st
        st.profile_enable(1 << PROF_W13_MAIN)
        self.run_decode(steps)
        w13_ms, w13_n = st.profile_read(PROF_W13_MAIN)
        st.profile_enable(0b11111)
        self.run_decode(steps)
        H, Fl, eb = cfg.hidden, cfg.ffn_l, 2
        nbytes = {"qkv": H * (cfg.hq_l + 2 * cfg.hkv_l) * cfg.head_dim * eb, "wo": cfg.hq_l * cfg.head_dim * H * eb,
                  "w13": H * 2 * Fl * eb, "w2": Fl * H * eb}
        per = {}
        for name, slot in SLOT_NAMES:
            ms, n = st.profile_read(slot)
            us = ms / max(n, 1) * 1e3
            per[name] = {"avg_us": round(us, 2)}
            if name in nbytes:
                per[name]["GBps"] = round(nbytes[name] / us / 1e3, 1)
        # the four projections together (weight bytes over the time of their launches, finishing kernels included)
        tot_b = sum(nbytes.values())
        tot_us = sum(per[k]["avg_us"] for k in nbytes)
        per["projections"] = {"avg_us": round(tot_us, 2), "GBps": round(tot_b / tot_us / 1e3, 1),
                              "hbm_frac": round(tot_b / tot_us / 1e3 / HBM_PEAK_GBS, 4)}
        st.profile_enable(0)
        b2b_ms, b2b_n = st.time_w13_decode(max(1, 256 // cfg.n_layers))
        # W1/W3 main kernel, algorithmic bytes: the weights + the rows' activation operand (hi and lo halves); the
        # outputs (and, on the batched path, the fp32 partial sums handed to the finishing kernel) are not counted
        w13_bytes = nbytes["w13"] + self.b * H * eb * 2
        w13_us = w13_ms / max(w13_n, 1) * 1e3
        return per, {"bytes_per_launch": w13_bytes, "avg_launch_us": round(w13_us, 2), "launches_timed": w13_n,
                     "projection_back_to_back_us": round(b2b_ms / b2b_n * 1e3, 2)}


def hbm_roofline(cfg, b, k):
    achieved = k["bytes_per_launch"] / (k["avg_launch_us"] * 1e-6) / 1e9
    name = ("decode_splitk_kernel<2> (W1/W3 projection, 17..32 rows; its finishing kernel with the SwiGLU epilogue "
            "follows)" if b > 16 else
            "decode_splitk_kernel<1> (W1/W3 projection, 3..16 rows; finishing kernel follows)" if b > 2 else
            "decode_proj_kernel<1,2,8,4,SWIGLU> (W1/W3 projection + SwiGLU epilogue)")
    traffic, src = measured_traffic(cfg.name)
    return {"bound": "hbm", "kernel": name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": src, **k}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="l70_full", help="headline workload (a bf16 configuration)")
    ap.add_argument("--dtype", default="bf16", choices=("bf16", "f16"),
                    help="16-bit storage type of the headline workload (the configurations name bf16; f16 runs the "
                         "same shapes through the fp16 build of the kernels)")
    ap.add_argument("--prefill-reps", type=int, default=2)
    ap.add_argument("--layers", type=int, default=0,
                    help="measurement aid for profiler passes: run the headline stage with this many layers instead of the "
                         "workload's (per-layer and per-kernel figures are unchanged; the JSON line says so)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the other configurations' legs")
    ap.add_argument("--no-head", action="store_true", help="skip the LM-head leg (model end next to the last stage)")
    ap.add_argument("--no-sched", action="store_true", help="skip the host-only scheduler-search leg")
    ap.add_argument("--short-prompts", action="store_true",
                    help="also time one prompt of 128 and of 512 rows on the headline stage (the split-contraction and skinny-kernel "
                         "regime; the configurations leg does this for l70_tp4_prefill)")
    ap.add_argument("--calibrate", action="store_true",
                    help="measure what a plain streaming kernel and a register-resident MFMA loop sustain, then exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one rank's share of a stage at its real shape); "
              "--gpus > 1 is not supported and no multi-GPU figure is produced.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2311_11514_amd as hx
    from workloads import CONFIGS, CONFIG_ORDER, generate

    if args.calibrate:
        calibrate(torch, hx)
        calibrate_gemm(torch, hx)
        return
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg = CONFIGS[args.workload]
    assert cfg.dtype == "bf16", "the headline workload must be one of the bf16 configurations"
    if args.dtype != cfg.dtype:
        cfg = cfg.scaled(dtype=args.dtype)         # same shapes and draws, stored in the other 16-bit format
    if args.layers > 0:
        cfg = cfg.scaled(n_layers=args.layers)
    K, W = args.steps, args.warmup
    nproc = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    log(f"host: nproc {nproc} (os.cpu_count {os.cpu_count()})")

    # three plain copies of known size: the yardstick the profiler's byte counters are scaled by
    cal_src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
    cal_dst = torch.empty_like(cal_src)
    for _ in range(3):
        hx.stream_copy(cal_dst, cal_src, blocks=512)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    be = Bench(torch, hx, generate, cfg, max(K, W), keep_layers=() if args.no_cpu_baseline else (0,))
    pre = None
    if cfg.kv_context is None:
        pre = be.prefill(args.prefill_reps)          # leaves the prompts' K / V in the cache for the decode steps
        log(f"prefill {pre['ms_per_call']:.1f} ms per call, {pre['tokens_per_s']:.0f} tokens/s, GEMMs "
            f"{pre['gemm_mfma_frac']:.3f} of the MFMA peak")
    dt, dec = be.decode(K, W)
    per_kernel, w13 = be.decode_kernels(min(K, 32))
    log(f"decode {dec['ms_per_step']:.3f} ms per step, {dec['tokens_per_s']:.1f} tokens/s, {dec['hbm_frac']:.3f} of HBM peak")

    lens = be.lens
    result = {
        "metric": "decode_tokens_per_s_per_stage", "value": dec["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": dec["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: Llama-2-70B-shaped stage, TP{cfg.tp_degree} rank {be.rank}, "
                               f"{cfg.n_layers} layers, batch {be.b}, "
                               + (f"decode from a synthetic KV context of {cfg.kv_context}" if cfg.kv_context is not None
                                  else f"prompts of {min(lens)}..{max(lens)} tokens ({sum(lens)} rows) prefilled, then "
                                       f"one decode step per timed step against the ragged cache"),
                   "hidden": cfg.hidden, "local_q_heads": cfg.hq_l, "local_kv_heads": cfg.hkv_l,
                   "head_dim": cfg.head_dim, "local_ffn": cfg.ffn_l, "layers": cfg.n_layers,
                   "layers_of_the_workload": CONFIGS[args.workload].n_layers, "batch": be.b,
                   "weights_GB": round(be.st.weight_bytes() / 1e9, 1)},
        "us_per_layer": dec["us_per_layer"], "stage_hbm_frac": dec["hbm_frac"],
        "prefill_tokens_per_s": pre["tokens_per_s"] if pre else None,
        "per_kernel": per_kernel,
        "roofline": hbm_roofline(cfg, be.b, w13),
        "host": {"nproc": nproc, "os_cpu_count": os.cpu_count()},
    }
    if pre:
        result["prefill"] = pre
        f, us, n = be.prefill_w13
        result["roofline_prefill"] = {"bound": "mfma", "kernel": "gemm_mfma_kernel (W1/W3 GEMM + SwiGLU epilogue)",
                                      "achieved": round(f / us / 1e6, 1), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                                      "frac": round(f / us / 1e6 / MFMA_PEAK_TFLOPS, 4), "traffic": None,
                                      "flops_per_launch": f, "avg_launch_us": us, "launches_timed": n}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(torch, be, nproc)
    if args.short_prompts:
        result["one_short_prompt"] = short_prompts(torch, be)
    summary = {cfg.name: {"decode": dec, **({"prefill": {k: v for k, v in pre.items() if k != "gemm"}} if pre else {})}}
    # The headline's stage stays allocated while the other configurations run (they need a few GB each): on this driver a
    # process that has just freed a large allocation runs the same kernels on the same buffers a few percent slower (the
    # TP2 batch-1 leg 165-166 us per layer behind the freed 137 GB stage, 160-162 with it still resident or in a process
    # of its own).

    if not args.no_configs:
        for name in CONFIG_ORDER:
            c = CONFIGS[name]
            if c.dtype != "bf16" or name == cfg.name:
                continue
            steps = c.decode_steps
            ob = Bench(torch, hx, generate, c, steps)
            entry = {}
            if c.kv_context is None:
                p = ob.prefill(5, warm=2)
                entry["prefill"] = p
                if name == "l70_tp4_prefill":
                    entry["one_short_prompt"] = short_prompts(torch, ob)
            _, d = ob.decode(steps, min(8, steps))
            pk, k13 = ob.decode_kernels(min(steps, 64))
            d["per_kernel"] = pk
            d["w13_main_kernel"] = {**k13, "GBps": round(k13["bytes_per_launch"] / k13["avg_launch_us"] / 1e3, 1)}
            entry["decode"] = d
            summary[name] = entry
            log(f"{name}: decode {d['us_per_layer']} us/layer, {d['hbm_frac']} of HBM peak"
                + (f"; prefill GEMMs {entry['prefill']['gemm_mfma_frac']} of MFMA peak" if "prefill" in entry else ""))
            del ob
            torch.cuda.empty_cache()
    result["configs"] = summary
    if not args.no_head:
        result["lm_head"] = head_leg(torch, hx, generate)
    if not args.no_configs and "l70_tp4_prefill" in summary and "l70_tp2_decode" in summary:
        result["cost_model"] = cost_model_alignment(torch, hx, CONFIGS, summary)
    if not args.no_sched:
        result["scheduler"] = scheduler_leg(hx)
    print(json.dumps(result), flush=True)


def short_prompts(torch, ob, reps=5):
    """One short prompt on the TP4 stage: the regime of the split contraction and the skinny kernel (weight-streaming
    bound: the floor is the stage's weight bytes at the HBM peak)."""
    cfg, st = ob.cfg, ob.st
    X = ob.generate.hidden_rows(cfg, 512, device="cuda").to(torch.bfloat16).contiguous()
    outp, outr = torch.empty_like(X), torch.empty_like(X)
    short = {}
    for rows in (128, 512):
        kv1 = st.kv_cache_create(1, rows + 8)
        for _ in range(2):
            st.prefill(kv1, X[:rows], [rows], outp[:rows], outr[:rows])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            st.prefill(kv1, X[:rows], [rows], outp[:rows], outr[:rows])
        torch.cuda.synchronize()
        dt1 = (time.perf_counter() - t0) / reps
        short[str(rows)] = {"us_per_layer": round(dt1 * 1e6 / cfg.n_layers, 1), "tokens_per_s": round(rows / dt1, 1),
                            "weights_at_hbm_peak_us_per_layer": round(st.weight_bytes() / cfg.n_layers / HBM_PEAK_GBS / 1e3, 1)}
        del kv1
    return short


def scheduler_leg(hx):
    """Host-only leg: the search over deployments (Section 4.3) on a synthetic pool in the shape of the paper's
    full-price rental (58 GPUs, 6 types), Llama-2-70B-sized task, 400 Poisson arrivals at 2 requests/s, deadline
    5 x the fastest start group; wall time of the library call on one host core."""
    from workloads import serving
    pool = serving.hetero_pool("full_price")
    task, n_layers = (8192, 12.0, 2, 1, 128, 32), 80
    model_bytes = n_layers * 12 * 8192 ** 2 * 2
    start = hx.sched_initial_groups(pool)
    lat0 = [hx.sched_plan_group(pool, task, g, n_layers, 8, True)[0] for g in start]
    arrival = serving.poisson_arrivals(2.0, 400, 7)
    deadline = 5 * min(lat0)
    t0 = time.perf_counter()
    res = hx.sched_search(pool, task, n_layers, model_bytes, 8, arrival, deadline, 11, 400, 8, True)
    dt = time.perf_counter() - t0
    return {"pool": "synthetic full-price shape, 58 GPUs of 6 types", "steps": 400, "population": 8,
            "search_s": round(dt, 2), "start_groups": len(start),
            "start_attainment": round(hx.slo_attainment(arrival, [[x] for x in lat0], [deadline]), 4),
            "groups": len(res["groups"]), "attainment": round(res["attainment"], 4)}


def head_leg(torch, hx, generate, reps=50):
    """The model's end next to the last stage: final RMSNorm + LM head (8192 x 32000 bf16, one rank) + greedy arg-max
    for one decode row; HBM-bound on the head's weights."""
    from workloads import StageConfig
    cfg = StageConfig("head70b", "bf16", 8192, 64, 8, 28672, 1, 1, (0,), batch=1, seed=41, vocab=32000)
    hw = generate.head_weights(cfg, device="cuda")
    hd = hx.Head(cfg.hidden, cfg.vocab, 1, 0, "bf16", cfg.rms_eps)
    hd.load(hw["g_final"], hw["w_lm"])
    del hw
    x = generate.hidden_rows(cfg, 1, device="cuda").to(torch.bfloat16).contiguous()
    for _ in range(5):
        hd.greedy(x)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        tok, _ = hd.greedy(x)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) / reps * 1e3
    nbytes = cfg.hidden * cfg.vocab * 2
    return {"workload": "final RMSNorm + LM head 8192 x 32000 bf16 + arg-max, 1 row, vocabulary on one rank",
            "us_per_token": round(us, 2), "GBps": round(nbytes / us / 1e3, 1), "hbm_frac": round(nbytes / us / 1e3 / 8000.0, 4),
            "token": int(tok.item())}


def cost_model_alignment(torch, hx, CONFIGS, summary):
    """The paper's computation-cost formula (Eq. 3, with Llama-2-70B's 12.75 H^2 parameters per layer) fed with this
    machine's MEASURED rates -- m_d: a cold 470 MB streaming read, c_d: the rate of the largest prefill GEMM -- against
    the measured times of the TP2 decode and TP4 prefill workloads (the paper's own alignment table compares the same
    two columns)."""
    big = torch.empty(1880 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
    sink = torch.zeros(1 << 16, dtype=torch.float32, device="cuda")
    n = 470 << 20
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    hx.stream_read(big[:n], sink, 512)
    torch.cuda.synchronize()
    e0.record()
    for i in range(4):
        hx.stream_read(big[i * n:(i + 1) * n], sink, 512)
    e1.record()
    torch.cuda.synchronize()
    m_d = 4 * n / (e0.elapsed_time(e1) * 1e-3)
    pre = summary["l70_tp4_prefill"]["prefill"]
    c_d = pre["gemm"]["w13"]["TFLOPs"] * 1e12
    dc, pc = CONFIGS["l70_tp2_decode"], CONFIGS["l70_tp4_prefill"]
    dec = hx.cost_comp(dc.hidden, 2, dc.batch, 0, 1, dc.n_layers, [m_d] * dc.tp_degree, [c_d] * dc.tp_degree, 12.75, "decode")
    est = hx.cost_comp(pc.hidden, 2, pc.batch, pc.prompt_len, 0, pc.n_layers, [m_d] * pc.tp_degree, [c_d] * pc.tp_degree,
                       12.75, "prefill")
    # the same two columns for every workload of the run: where the two-parameter model holds (weight-streaming decode of
    # large shards, long prefills) and where it does not (small shards: launch-bound; ragged long prompts: attention)
    table = []
    for name, entry in summary.items():
        c = CONFIGS[name]
        m, cc = [m_d] * c.tp_degree, [c_d] * c.tp_degree
        if "decode" in entry:
            e = hx.cost_comp(c.hidden, 2, entry["decode"]["batch"], 0, 1, c.n_layers, m, cc, 12.75, "decode")
            table.append({"workload": name, "phase": "decode step", "estimated_ms": round(e * 1e3, 4),
                          "measured_ms": entry["decode"]["ms_per_step"],
                          "measured_over_estimated": round(entry["decode"]["ms_per_step"] / (e * 1e3), 3)})
        if "prefill" in entry:
            pr = entry["prefill"]
            e = hx.cost_comp(c.hidden, 2, pr["sequences"], int(round(pr["rows"] / pr["sequences"])), 0, c.n_layers, m, cc,
                             12.75, "prefill")
            table.append({"workload": name, "phase": "prefill call", "estimated_ms": round(e * 1e3, 3),
                          "measured_ms": pr["ms_per_call"], "measured_over_estimated": round(pr["ms_per_call"] / (e * 1e3), 3)})
    return {"m_d_GBps": round(m_d / 1e9, 1), "c_d_TFLOPs": round(c_d / 1e12, 1),
            "decode_ms_per_token": {"estimated": round(dec * 1e3, 4),
                                    "measured": summary["l70_tp2_decode"]["decode"]["ms_per_step"]},
            "prefill_ms_per_call": {"estimated": round(est * 1e3, 3), "measured": pre["ms_per_call"]},
            "table": table}


def calibrate(torch, hx):
    """Practical ceilings of this machine, printed as a table: HBM streaming (cold: a 2.4 GB buffer is walked
    through in slices so nothing is re-read from cache) and dense bf16 MFMA from registers."""
    dev = "cuda"
    def timed(fn, reps):
        fn(0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            fn(i + 1)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3          # microseconds
    big = torch.empty(2400 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
    sink = torch.zeros(1 << 16, dtype=torch.float32, device=dev)
    print("HBM streaming, cold (MB, blocks of 256 threads, kernel, us, TB/s moved)")
    for mb in (32, 84, 235, 470):
        n = mb << 20
        slices = big.numel() // n
        for blocks in (512, 4096):
            us = timed(lambda i: hx.stream_read(big[(i % slices) * n:(i % slices + 1) * n], sink, blocks), 20)
            print(f"  {mb:4d} {blocks:5d} read  {us:8.1f} {n / us / 1e6:6.2f}")
            us = timed(lambda i: hx.stream_copy(dst[:n], big[(i % slices) * n:(i % slices + 1) * n], blocks), 20)
            print(f"  {mb:4d} {blocks:5d} copy  {us:8.1f} {2 * n / us / 1e6:6.2f}")
    print("dense bf16 MFMA, 4 waves per CU, operands in registers, ~50 ms per run (variant, TFLOP/s, fraction of 2516.6)")
    names = ["16x16x32, registers only", "32x32x16, registers only", "16x16x32 + GEMM-rate LDS reads",
             "32x32x16 + GEMM-rate LDS reads"]
    blocks = 256
    for v in range(8):
        name = names[v % 4] + (", random operand bits" if v >= 4 else ", operands all 1.0")
        iters = 100000
        us = timed(lambda i: hx.mfma_probe(v, sink, iters, blocks), 1)
        tf = blocks * 4 * iters * (1 << 20) / us / 1e6
        print(f"  {name:58s} {tf:8.1f} {tf / 2516.6:6.3f}")
    names2 = {8: "results in accumulation registers, row by row", 9: "results in vector registers, row by row",
              10: "results in accumulation registers, serpentine", 11: "results in vector registers, serpentine"}
    for v in (8, 9, 10, 11, 8, 9):
        iters = 100000
        us = timed(lambda i: hx.mfma_probe(v, sink, iters, blocks), 1)
        tf = blocks * 4 * iters * (1 << 20) / us / 1e6
        print(f"  16x16x32, random bits, 128 result registers: {names2[v]:46s} {tf:8.1f} {tf / 2516.6:6.3f}")


class _PowerMeter:
    """Socket power from the amdgpu hwmon file, sampled every 50 ms by a thread (None when the file is absent)."""

    def __init__(self):
        import glob
        files = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") +
                       glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average"))
        self.path = files[0] if files else None

    def run(self, torch, fn, secs):
        """Calls fn() back to back for `secs` seconds; returns (calls per second, mean watts of the second half)."""
        import threading
        samples, stop = [], []

        def sample():
            while not stop:
                try:
                    samples.append(int(open(self.path).read()) / 1e6)
                except Exception:
                    pass
                time.sleep(0.05)
        th = threading.Thread(target=sample, daemon=True)
        fn()
        torch.cuda.synchronize()
        if self.path:
            th.start()
        t0, n = time.perf_counter(), 0
        while time.perf_counter() - t0 < secs:
            for _ in range(4):
                fn()
            torch.cuda.synchronize()
            n += 4
        dt = time.perf_counter() - t0
        stop.append(1)
        if self.path:
            th.join()
        half = samples[len(samples) // 2:]
        return n / dt, (sum(half) / len(half) if half else None)


def calibrate_gemm(torch, hx):
    """What bounds the prefill GEMM on this machine, as a table: sustained rate and socket power of
      * the vendor library's bf16 GEMM (torch.nn.functional.linear -> hipBLASLt) on the W1/W3 shapes of the workloads --
        a yardstick only, never part of the product path;
      * this library's FFN sub-layer (W1/W3 + SwiGLU and W2 + residual GEMMs) on the same rows, with the default
        tile and with the k-loop ablations of include/hexgen_bench.h (loads removed / cache-hit loads / no LDS reads)."""
    from workloads import CONFIGS, generate
    pm = _PowerMeter()
    print(f"power file: {pm.path}")
    print("vendor bf16 GEMM (hipBLASLt through torch), x ~ N(0,1), w ~ N(0, 0.02^2): rows x 8192 x features, TFLOP/s, fraction of 2516.6, W")
    for T, N in ((2048, 14336), (16384, 14336), (65536, 14336), (71102, 57344)):
        x = torch.randn(T, 8192, device="cuda", dtype=torch.bfloat16)
        w = (torch.randn(N, 8192, device="cuda") * 0.02).to(torch.bfloat16)
        rate, watts = pm.run(torch, lambda: torch.nn.functional.linear(x, w), 2.0)
        tf = 2.0 * T * 8192 * N * rate / 1e12
        print(f"  {T:6d} x 8192 x {N:6d}   {tf:8.1f}  {tf / MFMA_PEAK_TFLOPS:6.3f}  {watts if watts is None else round(watts):>6}")
        del x, w
    cfg = CONFIGS["l70_tp4_prefill"].scaled(n_layers=1)
    st = hx.Stage(cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, 1, cfg.tp_degree, cfg.tp_ranks[0], "bf16")
    w = generate.layer_weights(cfg, 0, device="cuda")
    st.load_layer(0, *[w[k] for k in generate.LAYER_TENSOR_ORDER])
    del w
    print("this library, FFN sub-layer of the TP4 shard (W1/W3 2 x 7168 features + W2), rows, tile code, TFLOP/s of the two GEMMs, fraction, W")
    names = {0: "default", 1198: "ablation: no loads in the k-loop", 2198: "ablation: loads hit in cache",
             3198: "ablation: no LDS operand reads"}
    for T in (2048, 16384, 65536):
        kv = st.kv_cache_create(1, T)             # the FFN sub-layer leaves the cache alone; the call validates rows against it
        h = torch.randn(T, cfg.hidden, device="cuda", dtype=torch.float32)
        out = torch.empty_like(h)
        flop = 2.0 * T * cfg.hidden * 3 * cfg.ffn_l
        for code in (0, 1198, 2198, 3198):
            hx.set_gemm_tile(code)
            rate, watts = pm.run(torch, lambda: st.run_sublayer(kv, 0, 1, h, [T], 1, out), 2.0)
            hx.set_gemm_tile(0)
            tf = flop * rate / 1e12
            print(f"  {T:6d}  {names[code]:36s} {tf:8.1f}  {tf / MFMA_PEAK_TFLOPS:6.3f}  {watts if watts is None else round(watts):>6}")
        del kv, h, out
    st.close()
    # The same comparison on the headline workload's own shape and over its own duration: the headline prefill keeps the
    # matrix cores busy for many seconds, and what the part sustains at its power limit falls as it warms up.
    print("sustained, 12 s each, 71102 rows (the headline workload's prompt batch), full-width FFN 8192 <-> 28672: TFLOP/s, fraction, W")
    T = 71102
    x = torch.randn(T, 8192, device="cuda", dtype=torch.bfloat16)
    w = (torch.randn(57344, 8192, device="cuda") * 0.02).to(torch.bfloat16)
    rate, watts = pm.run(torch, lambda: torch.nn.functional.linear(x, w), 12.0)
    tf = 2.0 * T * 8192 * 57344 * rate / 1e12
    print(f"  vendor bf16 GEMM, rows x 8192 x 57344 (W1/W3's shape, no epilogue)   {tf:8.1f}  {tf / MFMA_PEAK_TFLOPS:6.3f}  {watts if watts is None else round(watts):>6}")
    del x, w
    cfg = CONFIGS["l70_full"].scaled(n_layers=1)
    st = hx.Stage(cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, 1, 1, 0, "bf16")
    w = generate.layer_weights(cfg, 0, device="cuda")
    st.load_layer(0, *[w[k] for k in generate.LAYER_TENSOR_ORDER])
    del w
    kv = st.kv_cache_create(1, T)
    h = torch.randn(T, cfg.hidden, device="cuda", dtype=torch.float32)
    out = torch.empty_like(h)
    rate, watts = pm.run(torch, lambda: st.run_sublayer(kv, 0, 1, h, [T], 1, out), 12.0)
    tf = 2.0 * T * cfg.hidden * 3 * cfg.ffn_l * rate / 1e12
    print(f"  this library, FFN sub-layer (W1/W3 + SwiGLU, W2 + residual)           {tf:8.1f}  {tf / MFMA_PEAK_TFLOPS:6.3f}  {watts if watts is None else round(watts):>6}")


def cpu_baseline(torch, be, nproc):
    """The oracle as it stands, on the host cores, on a bounded sample of the headline workload: ONE layer (layer 0) of
    the same stage -- a few decode steps of the whole batch from the GPU-prefilled context of that layer, and (when
    the workload has prompts) the prefill of one of the batch's prompts -- scaled to the stage by the layer count."""
    from oracle import stage_oracle as so
    from workloads import generate
    cfg = be.cfg
    try:
        from threadpoolctl import threadpool_info
        blas = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        blas = nproc
    ora = so.OracleStage(cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, 1, cfg.tp_degree, be.rank, cfg.rms_eps,
                         cfg.rope_theta)
    ora.load_layer(0, *[be.host_layers[0][k] for k in generate.LAYER_TENSOR_ORDER])
    oc = ora.new_cache(be.b)
    for s in range(be.b):                                  # layer 0's context as the GPU holds it
        k, v = be.kv.read(0, s, 0, be.lens[s])
        oc.fill(0, s, k, v)
    xs = be.X.float().cpu()
    ora.decode(oc, xs[0])                       # untimed first touch
    n, t0 = 0, time.perf_counter()
    while n < 32 and time.perf_counter() - t0 < 12.0:
        ora.decode(oc, xs[(1 + n) % xs.shape[0]])
        n += 1
    per_layer_step = (time.perf_counter() - t0) / n
    value = be.b / (per_layer_step * cfg.n_layers)
    out = {"value": round(value, 4), "unit": "tokens/s", "cores": blas, "kind": "oracle",
           "sample": f"1 of {cfg.n_layers} layers, {n} decode steps of the batch of {be.b} at its "
                     f"{'ragged ' if cfg.kv_context is None else ''}context, float64 numpy; "
                     f"stage rate = batch / (layer-step time x {cfg.n_layers}); projections on {blas} BLAS threads, "
                     f"the attention loop on 1 (nproc {nproc})"}
    log(f"cpu oracle: decode {per_layer_step * 1e3:.1f} ms per layer-step on {blas} BLAS threads (nproc {nproc})")
    if cfg.kv_context is None:
        # prefill of ONE prompt of the batch (the one closest to 1024 rows) through the same layer
        s = min(range(be.b), key=lambda i: abs(be.lens[i] - 1024))
        rows = be.lens[s]
        x = generate.hidden_rows(cfg, sum(be.lens), device="cuda")[sum(be.lens[:s]): sum(be.lens[:s]) + rows].cpu()
        t0 = time.perf_counter()
        ora.prefill(ora.new_cache(1), x, [rows])
        dtp = time.perf_counter() - t0
        out["prefill"] = {"value": round(rows / (dtp * cfg.n_layers), 4), "unit": "tokens/s",
                          "sample": f"1 of {cfg.n_layers} layers, one prompt of {rows} rows ({dtp:.1f} s); "
                                    f"stage rate = rows / (layer time x {cfg.n_layers})"}
        log(f"cpu oracle: prefill of {rows} rows through one layer {dtp:.1f} s")
    return out


if __name__ == "__main__":
    main()
