#!/usr/bin/env python3
"""Benchmark of the stage hot path on one MI355X.

Workload (N = 1): the Llama-2-70B-shaped shard at tensor-parallel degree 2, rank 0, 8-layer stage,
batch-1 decode from a synthetic KV context of 1024 positions -- the configuration the headline metric
(decode tokens/s per stage, fraction of HBM peak) is quoted on.  One "step" = one decode step of the whole
stage (all layers: RMSNorm, QKV, RoPE + cache append, attention, W_O, RMSNorm, W1/W3 + SwiGLU, W2).
Inputs and weights are synthetic (seeded normal draws) and resident in HBM before the timed region.

Prints ONE JSON line.  Besides the contract fields it carries
  roofline     -- the dominant kernel (W1/W3 weight-streaming projection) against the 8 TB/s HBM peak,
                  timed with HIP events on the launch stream in a second, instrumented pass;
  cpu_baseline -- the float64 CPU oracle timed on a bounded sample (one layer, a few decode steps),
                  scaled to the same unit.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
PROF_QKV, PROF_WO, PROF_W13, PROF_W2, PROF_ATTN, PROF_CALL = range(6)

# HBM bytes per launch of the dominant kernel measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE scaled
# by a copy kernel of known size); see profiles/.  None until measured for the current kernel.
MEASURED_TRAFFIC_BYTES = 470_662_000     # profiles/decode_l70_tp2_pmc_traffic.txt


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="l70_tp2_decode")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefill", action="store_true", help="skip the prefill leg (second workload)")
    ap.add_argument("--no-head", action="store_true", help="skip the LM-head leg (model end next to the last stage)")
    ap.add_argument("--no-sched", action="store_true", help="skip the host-only scheduler-search leg")
    ap.add_argument("--calibrate", action="store_true",
                    help="measure what a plain streaming kernel and a register-resident MFMA loop sustain, then exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one rank's share of a stage at its real shape); "
              "--gpus > 1 is not supported and no multi-GPU figure is produced.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2311_11514_amd as hx
    from workloads import CONFIGS, generate

    if args.calibrate:
        calibrate(torch, hx)
        return

    cfg = CONFIGS[args.workload]
    assert cfg.kv_context is not None and cfg.dtype == "bf16", "bench workload must be a bf16 decode config"
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda"
    rank = cfg.tp_ranks[0]
    K, W = args.steps, args.warmup
    b, ctx = cfg.batch, cfg.kv_context

    t_setup = time.time()
    st = hx.Stage(cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, cfg.n_layers, cfg.tp_degree, rank, cfg.dtype,
                  cfg.rms_eps, cfg.rope_theta)
    layer0_host = None
    for l in range(cfg.n_layers):
        w = generate.layer_weights(cfg, l, device=dev)
        st.load_layer(l, *[w[k] for k in generate.LAYER_TENSOR_ORDER])
        if l == 0 and not args.no_cpu_baseline:
            layer0_host = {k: v.cpu() for k, v in w.items()}
        del w
    kv = st.kv_cache_create(b, ctx + max(K, W) + 1)
    kv_host = {}
    for l in range(cfg.n_layers):
        for s in range(b):
            k, v = generate.synthetic_kv(cfg, l, s, ctx, device=dev)
            k, v = k.cpu(), v.cpu()
            kv.fill(l, s, k, v)
            if l == 0:
                kv_host[s] = (k, v)
    X = torch.stack([generate.hidden_rows(cfg, b, stream_id=1 + i, device=dev) for i in range(max(K, W))])
    X = X.to(torch.bfloat16).contiguous()
    outp = torch.empty(b, cfg.hidden, dtype=torch.bfloat16, device=dev)
    outr = torch.empty_like(outp)
    torch.cuda.synchronize()
    log(f"setup {time.time() - t_setup:.1f}s, weights {st.weight_bytes() / 1e9:.3f} GB")

    def run(n):
        kv.set_lengths([ctx] * b)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            st.decode(kv, i, X[i], outp, outr)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    # three plain copies of known size: the yardstick the profiler's byte counters are scaled by
    cal_src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
    cal_dst = torch.empty_like(cal_src)
    for _ in range(3):
        hx.stream_copy(cal_dst, cal_src, blocks=512)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    run(W)
    dt = run(K)
    ms_per_step = dt / K * 1e3
    tok_s = b * K / dt
    assert torch.isfinite(outp.float()).all() and torch.isfinite(outr.float()).all()

    # instrumented passes: HIP events on the launch stream; first around the dominant kernel alone (so its
    # figure carries no other events' overhead), then around every projection for the per-kernel table
    st.profile_enable(1 << PROF_W13)
    run(K)
    w13_ms, w13_n = st.profile_read(PROF_W13)
    st.profile_enable(True)
    run(K)
    slots = {}
    for name, slot in (("qkv", PROF_QKV), ("wo", PROF_WO), ("w13", PROF_W13), ("w2", PROF_W2),
                       ("attn", PROF_ATTN), ("call", PROF_CALL)):
        ms, n = st.profile_read(slot)
        slots[name] = {"avg_us": ms / max(n, 1) * 1e3, "launches": n}
    st.profile_enable(False)
    # the same kernel once more, all layers back to back between two events only (no per-launch events): its duration
    # without the dispatch gap that an event pair around a single launch includes
    b2b_ms, b2b_n = st.time_w13_decode(32)

    eb = 2
    H, Fl = cfg.hidden, cfg.ffn_l
    w13_bytes = H * 2 * Fl * eb + b * H * eb * 2        # weights + hi/lo activation operand (outputs are negligible)
    w13_us = w13_ms / max(w13_n, 1) * 1e3
    achieved = w13_bytes / (w13_us * 1e-6) / 1e9
    bytes_by_proj = {"qkv": H * (cfg.hq_l + 2 * cfg.hkv_l) * cfg.head_dim * eb, "wo": cfg.hq_l * cfg.head_dim * H * eb,
                     "w13": H * 2 * Fl * eb, "w2": Fl * H * eb}
    per_kernel = {k: {"avg_us": round(slots[k]["avg_us"], 2),
                      "GBps": round(bytes_by_proj[k] / (slots[k]["avg_us"] * 1e-6) / 1e9, 1)} for k in bytes_by_proj}
    per_kernel["attn_block"] = {"avg_us": round(slots["attn"]["avg_us"], 2)}
    # whole-step algorithmic bytes: weights + KV read (context grows by one per step)
    kv_bytes_avg = cfg.kv_bytes_per_pos_layer() * b * (ctx + (K + 1) / 2.0)
    step_bytes = cfg.n_layers * (cfg.weight_elems_per_layer_rank * eb + kv_bytes_avg)
    stage_frac = step_bytes / (dt / K) / 1e9 / HBM_PEAK_GBS

    result = {
        "metric": "decode_tokens_per_s_per_stage", "value": round(tok_s, 2), "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: Llama-2-70B-shaped shard, TP{cfg.tp_degree} rank {rank}, "
                               f"{cfg.n_layers}-layer stage, batch {b} decode from KV context {ctx}",
                   "hidden": H, "local_q_heads": cfg.hq_l, "local_kv_heads": cfg.hkv_l, "head_dim": cfg.head_dim,
                   "local_ffn": Fl, "layers": cfg.n_layers, "batch": b, "kv_context": ctx},
        "us_per_layer": round(ms_per_step * 1e3 / cfg.n_layers, 2),
        "stage_hbm_frac": round(stage_frac, 4),
        "per_kernel": per_kernel,
        "roofline": {"bound": "hbm", "kernel": "decode_proj_kernel<1,2,8,4,SWIGLU> (W1/W3 projection + SwiGLU epilogue)",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES, "bytes_per_launch": w13_bytes,
                     "avg_launch_us": round(w13_us, 2), "launches_timed": w13_n,
                     "back_to_back": {"avg_launch_us": round(b2b_ms / b2b_n * 1e3, 2), "launches": b2b_n,
                                      "frac": round(w13_bytes / (b2b_ms / b2b_n * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}},
    }

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, rank, layer0_host, kv_host, X, ctx)
    if not args.no_prefill:
        del st, kv, X
        torch.cuda.empty_cache()
        result["prefill"] = prefill_leg(torch, hx, CONFIGS["l70_tp4_prefill"], generate)
    if not args.no_head:
        torch.cuda.empty_cache()
        result["lm_head"] = head_leg(torch, hx, generate)
    if "prefill" in result:
        result["cost_model"] = cost_model_alignment(torch, hx, cfg, result)
    if not args.no_sched:
        result["scheduler"] = scheduler_leg(hx)
    print(json.dumps(result), flush=True)


def scheduler_leg(hx):
    """Host-only leg: the search over deployments (Section 4.3) on a synthetic pool in the shape of the paper's
    full-price rental (58 GPUs, 6 types), Llama-2-70B-sized task, 400 Poisson arrivals at 2 requests/s, deadline
    5 x the fastest start group; wall time of the library call on one host core."""
    import time

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


MFMA_PEAK_TFLOPS = 2516.6      # MI355X published dense bf16 rate


def prefill_leg(torch, hx, cfg, generate, reps=5):
    """Second half of the headline metric: prefill tokens/s of the asymmetric TP4 shard (20 layers, 4 x 512 rows)
    and the projection GEMMs against the bf16 MFMA peak.  Reported beside the decode figure, not as `value`."""
    dev, rank = "cuda", cfg.tp_ranks[0]
    st = hx.Stage(cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, cfg.n_layers, cfg.tp_degree, rank, cfg.dtype,
                  cfg.rms_eps, cfg.rope_theta)
    for l in range(cfg.n_layers):
        w = generate.layer_weights(cfg, l, device=dev)
        st.load_layer(l, *[w[k] for k in generate.LAYER_TENSOR_ORDER])
        del w
    lens = generate.prompt_lengths(cfg)
    T = sum(lens)
    kv = st.kv_cache_create(cfg.batch, max(lens) + 8)
    X = generate.hidden_rows(cfg, T, device=dev).to(torch.bfloat16).contiguous()
    outp, outr = torch.empty_like(X), torch.empty_like(X)
    for _ in range(2):
        st.prefill(kv, X, lens, outp, outr)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        st.prefill(kv, X, lens, outp, outr)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    assert torch.isfinite(outp.float()).all()
    st.profile_enable(0b1111)
    st.prefill(kv, X, lens, outp, outr)
    H, d = cfg.hidden, cfg.head_dim
    flops = {"qkv": 2 * T * H * (cfg.hq_l + 2 * cfg.hkv_l) * d, "wo": 2 * T * cfg.hq_l * d * H,
             "w13": 2 * T * H * 2 * cfg.ffn_l, "w2": 2 * T * cfg.ffn_l * H}
    gemm = {}
    tot_f, tot_t = 0.0, 0.0
    for slot, name in enumerate(("qkv", "wo", "w13", "w2")):
        ms, n = st.profile_read(slot)
        us = ms / max(n, 1) * 1e3
        gemm[name] = {"avg_us": round(us, 1), "TFLOPs": round(flops[name] / us / 1e6, 1)}
        tot_f += flops[name]
        tot_t += us
    st.profile_enable(0)
    # one short prompt on the same stage: the regime of the split contraction and the skinny kernel (weight-streaming
    # bound: the floor is the stage's weight bytes at the HBM peak)
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
    layer_flops = sum(flops.values()) + sum(2 * n * n * d * cfg.hq_l for n in lens)
    return {"workload": f"{cfg.name}: TP{cfg.tp_degree} rank {rank}, {cfg.n_layers} layers, {cfg.batch} x {lens[0]} rows",
            "tokens_per_s": round(T / dt, 1), "ms_per_call": round(dt * 1e3, 3),
            "us_per_layer": round(dt * 1e6 / cfg.n_layers, 1),
            "stage_mfma_frac": round(layer_flops * cfg.n_layers / dt / 1e12 / MFMA_PEAK_TFLOPS, 4),
            "gemm_mfma_frac": round(tot_f / tot_t / 1e6 / MFMA_PEAK_TFLOPS, 4), "gemm": gemm,
            "peak_TFLOPs": MFMA_PEAK_TFLOPS, "one_short_prompt": short}


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


def cost_model_alignment(torch, hx, cfg, result):
    """The paper's computation-cost formula (Eq. 3, with Llama-2-70B's 12.75 H^2 parameters per layer) fed with this
    machine's MEASURED rates -- m_d: a cold 470 MB streaming read, c_d: the rate of the largest prefill GEMM -- against
    the measured times of the two workloads above (the paper's own alignment table compares the same two columns)."""
    from workloads import CONFIGS
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
    c_d = result["prefill"]["gemm"]["w13"]["TFLOPs"] * 1e12
    pc = CONFIGS["l70_tp4_prefill"]
    dec = hx.cost_comp(cfg.hidden, 2, cfg.batch, 0, 1, cfg.n_layers, [m_d] * cfg.tp_degree, [c_d] * cfg.tp_degree, 12.75, "decode")
    pre = hx.cost_comp(pc.hidden, 2, pc.batch, pc.prompt_len, 0, pc.n_layers, [m_d] * pc.tp_degree, [c_d] * pc.tp_degree,
                       12.75, "prefill")
    return {"m_d_GBps": round(m_d / 1e9, 1), "c_d_TFLOPs": round(c_d / 1e12, 1),
            "decode_ms_per_token": {"estimated": round(dec * 1e3, 4), "measured": result["ms_per_step"]},
            "prefill_ms_per_call": {"estimated": round(pre * 1e3, 3), "measured": result["prefill"]["ms_per_call"]}}


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


def cpu_baseline(cfg, rank, layer0, kv_host, X, ctx):
    """The oracle as it stands, on the host cores: ONE layer of the same shard, a few decode steps from
    the same synthetic context; tokens/s of the stage = batch / (per-layer step time * layers)."""
    from oracle import stage_oracle as so
    from workloads import generate
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    ora = so.OracleStage(cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, 1, cfg.tp_degree, rank, cfg.rms_eps,
                         cfg.rope_theta)
    ora.load_layer(0, *[layer0[k] for k in generate.LAYER_TENSOR_ORDER])
    oc = ora.new_cache(cfg.batch)
    for s, (k, v) in kv_host.items():
        oc.fill(0, s, k, v)
    xs = X.float().cpu()
    ora.decode(oc, xs[0])                       # untimed first touch
    n, t0 = 0, time.perf_counter()
    while n < 64 and time.perf_counter() - t0 < 15.0:
        ora.decode(oc, xs[1 + n % (xs.shape[0] - 1)])
        n += 1
    per_layer_step = (time.perf_counter() - t0) / n
    value = cfg.batch / (per_layer_step * cfg.n_layers)
    log(f"cpu oracle: {per_layer_step * 1e3:.1f} ms per layer-step on {cores} threads")
    return {"value": round(value, 4), "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"1 of {cfg.n_layers} layers, {n} decode steps at context {ctx}+, float64 numpy; "
                      f"stage rate = batch / (layer-step time x {cfg.n_layers})"}


if __name__ == "__main__":
    main()
