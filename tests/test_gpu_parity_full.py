"""GPU parity at the full sizes of the 70B-shaped workloads, in the launch configuration bench.py times.

The oracle cannot run these workloads whole in test time, so each case compares what it can compute:
  * decode-only workloads: every layer of the stage, a few decode steps from the synthetic context;
  * the prefill workload: one whole sequence of the batch through every layer (sequences of a batch are
    independent -- the oracle's own pins check that), then decode steps for that sequence.
Weights are drawn on the GPU (seeded torch generator) and the oracle receives copies of the same values.
"""
import numpy as np
import pytest
import torch

from workloads import CONFIGS, generate
from tests.helpers import ORDER, TOL, gpu_decode, gpu_prefill, max_abs_over_l2, row_rel_err, to_dev

pytestmark = pytest.mark.gpu


def build_both(cfg, rank):
    """GPU stage and oracle from the same device-generated weights, one layer at a time."""
    import paper_2311_11514_amd as hx
    from oracle import stage_oracle as so
    st = hx.Stage(cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, cfg.n_layers, cfg.tp_degree, rank, cfg.dtype,
                  cfg.rms_eps, cfg.rope_theta)
    ora = so.OracleStage(cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, cfg.n_layers, cfg.tp_degree, rank,
                         cfg.rms_eps, cfg.rope_theta)
    for l in range(cfg.n_layers):
        w = generate.layer_weights(cfg, l, device="cuda")
        args = [w[k] for k in ORDER]
        st.load_layer(l, *args)
        ora.load_layer(l, *args)        # slices the shard on the device, copies only that to the host
        del w, args
    return st, ora


def install_context(cfg, st_kv, ora_cache, seqs, ctx):
    for l in range(cfg.n_layers):
        for s in seqs:
            k, v = generate.synthetic_kv(cfg, l, s, ctx, device="cuda")
            k, v = k.cpu(), v.cpu()
            st_kv.fill(l, s, k, v)
            ora_cache.fill(l, s, k, v)


@pytest.mark.parametrize("name,steps", [("l70_tp2_decode", 3), ("l70_tp8_decode", 2)])
def test_decode_workloads_full_depth(name, steps):
    cfg = CONFIGS[name]
    rank = cfg.tp_ranks[0]
    st, ora = build_both(cfg, rank)
    b, ctx = cfg.batch, cfg.kv_context
    kv = st.kv_cache_create(b, ctx + cfg.decode_steps)
    oc = ora.new_cache(b)
    install_context(cfg, kv, oc, range(b), ctx)
    kv.set_lengths([ctx] * b)
    for step in range(steps):
        x = generate.hidden_rows(cfg, b, stream_id=1 + step, device="cuda").cpu()
        p_ref, h_ref = ora.decode(oc, x)
        p, h = gpu_decode(st, kv, cfg, step, x)
        eh, ep = row_rel_err(h, h_ref), row_rel_err(p, p_ref)
        print(f"{name} step {step}: resid err {eh:.3e} partial err {ep:.3e}", flush=True)
        assert eh < TOL["bf16"] and ep < TOL["bf16"]
    # the rows appended by the GPU are the oracle's rows
    kk, vv = kv.read(cfg.n_layers - 1, b - 1, ctx, steps)
    d = cfg.head_dim
    assert row_rel_err(kk.numpy().reshape(-1, d), oc.k[-1][b - 1][ctx:].reshape(-1, d)) < TOL["bf16"]
    assert row_rel_err(vv.numpy().reshape(-1, d), oc.v[-1][b - 1][ctx:].reshape(-1, d)) < TOL["bf16"]


def test_prefill_workload_one_sequence_full_depth():
    """20-layer prefill of 4 x 512 rows, then decode.  Two gates:
      * every layer on its own, teacher-forced FROM THE ORACLE (the GPU sub-layer receives the oracle's
        residual stream entering that sub-layer): per-row relative L2 error <= 2e-2;
      * end to end through all 20 layers: max elementwise error relative to the row's L2 norm <= 2e-2.
    The per-row relative L2 error of the end-to-end result is printed and loosely bounded, not gated at
    2e-2: rounding K and V alone to bf16 (which the bf16 cache must do) already exceeds 1e-2 after four
    layers of this randomly weighted stage, whatever the kernels do (emulated on the CPU in float64)."""
    import paper_2311_11514_amd as hx
    cfg = CONFIGS["l70_tp4_prefill"]
    rank = cfg.tp_ranks[0]
    st, ora = build_both(cfg, rank)
    lens = generate.prompt_lengths(cfg)
    T = sum(lens)
    X = generate.hidden_rows(cfg, T, device="cuda").cpu()
    kv = st.kv_cache_create(cfg.batch, cfg.prompt_len + cfg.decode_steps)
    p, h = gpu_prefill(st, kv, cfg, X, lens)
    assert np.isfinite(p).all() and np.isfinite(h).all()
    s = 2                                   # the sequence the oracle recomputes
    r0, n = sum(lens[:s]), lens[s]
    oc = ora.new_cache(1)
    taps = {}
    p_ref, h_ref = ora.prefill(oc, X[r0: r0 + n], [n], taps=taps)
    eh, ep = row_rel_err(h[r0: r0 + n], h_ref), row_rel_err(p[r0: r0 + n], p_ref)
    mh, mp = max_abs_over_l2(h[r0: r0 + n], h_ref), max_abs_over_l2(p[r0: r0 + n], p_ref)
    print(f"prefill seq {s}, 20 layers end to end: per-row L2 err resid {eh:.3e} partial {ep:.3e}; "
          f"max-abs / L2 resid {mh:.3e} partial {mp:.3e}", flush=True)
    assert mh < TOL["bf16"] and mp < TOL["bf16"]
    assert eh < 0.15 and ep < 0.15          # regression guard only, see the docstring
    for step in range(2):
        x = generate.hidden_rows(cfg, cfg.batch, stream_id=1 + step, device="cuda").cpu()
        pg, hg = gpu_decode(st, kv, cfg, step, x)
        p_ref, h_ref = ora.decode(oc, x[s: s + 1])
        mh, mp = max_abs_over_l2(hg[s: s + 1], h_ref), max_abs_over_l2(pg[s: s + 1], p_ref)
        print(f"decode after prefill, step {step}: max-abs / L2 resid {mh:.3e} partial {mp:.3e}; per-row L2 "
              f"{row_rel_err(hg[s: s + 1], h_ref):.3e} {row_rel_err(pg[s: s + 1], p_ref):.3e}", flush=True)
        assert mh < TOL["bf16"] and mp < TOL["bf16"]
    # layer by layer, inputs taken from the oracle
    kv1 = st.kv_cache_create(1, n)
    worst = 0.0
    part = torch.empty(n, cfg.hidden, dtype=torch.float32, device="cuda")
    for l in range(cfg.n_layers):
        h_l = taps[l]
        c1 = ora.new_cache(1)
        pa_ref = ora.attn_partial(l, c1, h_l, [0] * n)
        h_mid = h_l + pa_ref
        pf_ref = ora.ffn_partial(l, h_mid)
        st.run_sublayer(kv1, l, 0, torch.from_numpy(h_l).to("cuda", torch.float32).contiguous(), [n], 1, part)
        torch.cuda.synchronize()
        ea = row_rel_err(part.cpu().numpy(), pa_ref)
        st.run_sublayer(kv1, l, 1, torch.from_numpy(h_mid).to("cuda", torch.float32).contiguous(), [n], 1, part)
        torch.cuda.synchronize()
        ef = row_rel_err(part.cpu().numpy(), pf_ref)
        worst = max(worst, ea, ef)
        assert ea < TOL["bf16"] and ef < TOL["bf16"], f"layer {l}: attn {ea:.3e} ffn {ef:.3e}"
    print(f"teacher-forced per-layer worst per-row L2 err {worst:.3e}", flush=True)


def test_full_width_80_layer_stage_sampled():
    """The full-width 80-layer stage (136.9 GB of weights), 32 ragged prompts of 128..4096 tokens, then decode.
    The oracle cannot run it whole; it recomputes layer 0 for the shortest and the longest sequence at
    sampled rows (prefill) and for the same sequences' decode rows, against the GPU's residual stream
    entering layer 1 (a tap, i.e. a GPU output).  At full depth the GPU run is checked for finiteness and
    for bit-identical repetition."""
    import paper_2311_11514_amd as hx
    from oracle import stage_oracle as so
    cfg = CONFIGS["l70_full"]
    lens = generate.prompt_lengths(cfg)
    T = sum(lens)
    st = hx.Stage(cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, cfg.n_layers, 1, 0, cfg.dtype, cfg.rms_eps,
                  cfg.rope_theta)
    ora = so.OracleStage(cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, 1, 1, 0, cfg.rms_eps, cfg.rope_theta)
    for l in range(cfg.n_layers):
        w = generate.layer_weights(cfg, l, device="cuda")
        args = [w[k] for k in ORDER]
        st.load_layer(l, *args)
        if l == 0:
            ora.load_layer(0, *args)
        del w, args
    print(f"loaded {st.weight_bytes() / 1e9:.1f} GB of weights; {T} prompt rows", flush=True)
    X = generate.hidden_rows(cfg, T, device="cuda")
    kv = st.kv_cache_create(cfg.batch, max(lens) + 8)
    tap = torch.empty(T, cfg.hidden, dtype=torch.float32, device="cuda")
    st.set_tap(1, tap)
    xin = to_dev(X, cfg)
    outp, outr = torch.empty_like(xin), torch.empty_like(xin)
    st.prefill(kv, xin, lens, outp, outr)
    torch.cuda.synchronize()
    assert torch.isfinite(outp.float()).all() and torch.isfinite(outr.float()).all()
    first = (outp.clone(), outr.clone())
    h1 = tap.cpu().numpy()
    cu = np.concatenate([[0], np.cumsum(lens)])
    rng = np.random.default_rng(5)
    caches = {}
    for s in (int(np.argmin(lens)), int(np.argmax(lens))):
        n = lens[s]
        rows = sorted(set([0, n - 1] + [int(v) for v in rng.integers(0, n, 16)]))
        ref, K, V = ora.layer_rows(0, X[cu[s]: cu[s] + n].cpu(), rows)
        err = row_rel_err(h1[cu[s]: cu[s] + n][rows], ref)
        print(f"prefill layer 0, sequence {s} (len {n}), {len(rows)} sampled rows: per-row L2 err {err:.3e}", flush=True)
        assert err < TOL["bf16"]
        kk, vv = kv.read(0, s, 0, n)
        d = cfg.head_dim
        assert row_rel_err(kk.numpy().reshape(-1, d), K.reshape(-1, d)) < TOL["bf16"]
        assert row_rel_err(vv.numpy().reshape(-1, d), V.reshape(-1, d)) < TOL["bf16"]
        caches[s] = (K, V)
    # bit-identical repetition of the whole 80-layer prefill
    st.prefill(kv, xin, lens, outp, outr)
    torch.cuda.synchronize()
    assert torch.equal(outp, first[0]) and torch.equal(outr, first[1])
    # decode: layer 0 of the two sequences against the oracle, full depth for finiteness
    tapd = torch.empty(cfg.batch, cfg.hidden, dtype=torch.float32, device="cuda")
    st.set_tap(1, tapd)
    for step in range(2):
        x = generate.hidden_rows(cfg, cfg.batch, stream_id=1 + step, device="cuda")
        pg, hg = gpu_decode(st, kv, cfg, step, x.cpu())
        assert np.isfinite(pg).all() and np.isfinite(hg).all()
        hd = tapd.cpu().numpy()
        for s, (K, V) in caches.items():
            oc = ora.new_cache(1)
            oc.fill(0, 0, K, V)
            xs = so._f64(x[s: s + 1])
            h_mid = xs + ora.attn_partial(0, oc, xs, [0])
            ref = h_mid + ora.ffn_partial(0, h_mid)
            caches[s] = (oc.k[0][0], oc.v[0][0])
            err = row_rel_err(hd[s: s + 1], ref)
            print(f"decode step {step}, layer 0, sequence {s}: per-row L2 err {err:.3e}", flush=True)
            assert err < TOL["bf16"]
    assert kv.get_lengths(cfg.batch) == [n + 2 for n in lens]
