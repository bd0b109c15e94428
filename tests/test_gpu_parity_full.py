"""GPU parity at the full sizes of the 70B-shaped workloads, in the launch configuration bench.py times.

The oracle cannot run every workload whole in test time, so each case compares what it can compute:
  * TP2 8-layer decode: every layer, every one of the 256 decode steps, the oracle keeping its own cache;
  * TP8 40-layer decode: every layer, the first steps with the oracle's own cache and the last step with the
    oracle's cache brought up to date from the rows the GPU appended (read back through the C ABI);
  * TP4 20-layer prefill: all four sequences through every layer, then decode steps (first ones, and the last);
  * full-width 80-layer stage: single layers (first, middle, last) fed the GPU's own residual stream at their
    entry (taps), at sampled rows of three sequences in prefill and at every row of the first and the last decode step.
Every comparison goes through tests.helpers.check, which prints both error metrics and applies the one gate rule.
Weights are drawn on the GPU (seeded torch generator) and the oracle receives copies of the same values.
"""
import time

import numpy as np
import pytest
import torch

from workloads import CONFIGS, generate
from tests.helpers import ORDER, TOL, check, gpu_decode, gpu_prefill, row_rel_err, to_dev

pytestmark = pytest.mark.gpu
BF = TOL["bf16"]


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


def sync_oracle_cache(cfg, kv, oc, batch):
    """Bring the oracle's cache up to the GPU's committed lengths with the rows the GPU appended (a GPU output that
    earlier assertions of the same test compared with the oracle's own rows)."""
    lens = kv.get_lengths(batch)
    for l in range(cfg.n_layers):
        for s in range(batch):
            have = oc.length(l, s)
            if lens[s] > have:
                kk, vv = kv.read(l, s, have, lens[s] - have)
                oc.append(l, s, kk.numpy().astype(np.float64), vv.numpy().astype(np.float64))


def compare_appended_rows(cfg, kv, oc, layer, seq, pos0, n, label):
    kk, vv = kv.read(layer, seq, pos0, n)
    d = cfg.head_dim
    check(f"{label}: appended K rows", kk.numpy().reshape(-1, d), oc.k[layer][seq][pos0: pos0 + n].reshape(-1, d), BF)
    check(f"{label}: appended V rows", vv.numpy().reshape(-1, d), oc.v[layer][seq][pos0: pos0 + n].reshape(-1, d), BF)


def test_tp2_decode_all_256_steps_full_depth():
    """Batch-1 decode of the TP2 8-layer stage from the synthetic context of 1024: every decode step of the workload,
    the oracle appending to its own cache (nothing is fed back from the GPU)."""
    cfg = CONFIGS["l70_tp2_decode"]
    st, ora = build_both(cfg, cfg.tp_ranks[0])
    b, ctx, steps = cfg.batch, cfg.kv_context, cfg.decode_steps
    kv = st.kv_cache_create(b, ctx + steps)
    oc = ora.new_cache(b)
    install_context(cfg, kv, oc, range(b), ctx)
    kv.set_lengths([ctx] * b)
    t0 = time.time()
    worst = [0.0, 0.0]
    for step in range(steps):
        x = generate.hidden_rows(cfg, b, stream_id=1 + step, device="cuda").cpu()
        p_ref, h_ref = ora.decode(oc, x)
        p, h = gpu_decode(st, kv, cfg, step, x)
        quiet = step not in (0, 1, 64, 128, steps - 1)
        for name, g, r in (("resid", h, h_ref), ("partial", p, p_ref)):
            if quiet:
                e2 = row_rel_err(g, r)
                assert e2 < BF, f"step {step} {name}: per-row L2 err {e2:.3e}"
            else:
                e2, _ = check(f"{cfg.name} step {step} {name}", g, r, BF)
            worst[name == "partial"] = max(worst[name == "partial"], e2)
    print(f"{cfg.name}: {steps} steps, worst per-row L2 err resid {worst[0]:.3e} partial {worst[1]:.3e} "
          f"({time.time() - t0:.0f} s)", flush=True)
    assert kv.get_lengths(b) == [ctx + steps] * b
    compare_appended_rows(cfg, kv, oc, cfg.n_layers - 1, 0, ctx, steps, f"{cfg.name} layer {cfg.n_layers - 1}")
    compare_appended_rows(cfg, kv, oc, 0, 0, ctx, steps, f"{cfg.name} layer 0")


def test_tp8_decode_first_steps_and_last_step_full_depth():
    """Batch-16 decode of the TP8 40-layer stage from the synthetic context of 2048: steps 0..3 with the oracle's own
    cache, then the GPU alone up to the last step of the workload, which is compared again after the oracle's cache
    has been brought up to date from the GPU's appended rows."""
    cfg = CONFIGS["l70_tp8_decode"]
    st, ora = build_both(cfg, cfg.tp_ranks[0])
    b, ctx, steps = cfg.batch, cfg.kv_context, cfg.decode_steps
    kv = st.kv_cache_create(b, ctx + steps)
    oc = ora.new_cache(b)
    install_context(cfg, kv, oc, range(b), ctx)
    kv.set_lengths([ctx] * b)
    first = 4
    for step in range(steps):
        x = generate.hidden_rows(cfg, b, stream_id=1 + step, device="cuda").cpu()
        if step == steps - 1:
            sync_oracle_cache(cfg, kv, oc, b)
        p, h = gpu_decode(st, kv, cfg, step, x)
        if step < first or step == steps - 1:
            p_ref, h_ref = ora.decode(oc, x)
            check(f"{cfg.name} step {step} resid", h, h_ref, BF)
            check(f"{cfg.name} step {step} partial", p, p_ref, BF)
        else:
            assert np.isfinite(p).all() and np.isfinite(h).all()
        if step == first - 1:
            compare_appended_rows(cfg, kv, oc, cfg.n_layers - 1, b - 1, ctx, first, f"{cfg.name} layer {cfg.n_layers - 1}")
    assert kv.get_lengths(b) == [ctx + steps] * b
    compare_appended_rows(cfg, kv, oc, cfg.n_layers - 1, 3, ctx + steps - 1, 1, f"{cfg.name} last step, last layer")


def test_tp4_prefill_all_sequences_full_depth_then_decode():
    """20-layer prefill of 4 x 512 rows, then the 64 decode steps of the workload (compared: steps 0..3 and the last).
      * End to end through all 20 layers, all four sequences: the gate is max-abs over the row's L2 norm only
        (per_row_l2=False, the one exemption of tests.helpers.check; tests/test_bf16_kv_floor.py shows that rounding the
        cached K / V to bf16 alone exceeds 2e-2 per-row L2 error at this depth).  The per-row L2 error is printed and
        bounded as a regression guard.
      * Every layer on its own, teacher-forced FROM THE ORACLE (the GPU sub-layer receives the oracle's residual stream
        entering that sub-layer): full gate, per-row L2 error included."""
    cfg = CONFIGS["l70_tp4_prefill"]
    rank = cfg.tp_ranks[0]
    st, ora = build_both(cfg, rank)
    lens = generate.prompt_lengths(cfg)
    T, b = sum(lens), cfg.batch
    X = generate.hidden_rows(cfg, T, device="cuda").cpu()
    kv = st.kv_cache_create(b, cfg.prompt_len + cfg.decode_steps)
    p, h = gpu_prefill(st, kv, cfg, X, lens)
    assert np.isfinite(p).all() and np.isfinite(h).all()
    oc = ora.new_cache(b)
    taps = {}
    p_ref, h_ref = ora.prefill(oc, X, lens, taps=taps)
    cu = np.concatenate([[0], np.cumsum(lens)])
    for s in range(b):
        r = slice(cu[s], cu[s + 1])
        eh, _ = check(f"prefill seq {s}, 20 layers end to end, resid", h[r], h_ref[r], BF, per_row_l2=False)
        ep, _ = check(f"prefill seq {s}, 20 layers end to end, partial", p[r], p_ref[r], BF, per_row_l2=False)
        assert eh < 0.15 and ep < 0.15          # regression guard only, see the docstring
    steps = cfg.decode_steps
    for step in range(steps):
        x = generate.hidden_rows(cfg, b, stream_id=1 + step, device="cuda").cpu()
        if step == steps - 1:
            sync_oracle_cache(cfg, kv, oc, b)
        pg, hg = gpu_decode(st, kv, cfg, step, x)
        if step < 4 or step == steps - 1:
            p_ref, h_ref = ora.decode(oc, x)
            check(f"decode after prefill, step {step}, resid", hg, h_ref, BF, per_row_l2=False)
            check(f"decode after prefill, step {step}, partial", pg, p_ref, BF, per_row_l2=False)
        else:
            assert np.isfinite(pg).all() and np.isfinite(hg).all()
    assert kv.get_lengths(b) == [n + steps for n in lens]
    # layer by layer, inputs taken from the oracle; one sequence (the layers see every row of it)
    s = 2
    r0, n = int(cu[s]), lens[s]
    kv1 = st.kv_cache_create(1, n)
    worst = 0.0
    part = torch.empty(n, cfg.hidden, dtype=torch.float32, device="cuda")
    for l in range(cfg.n_layers):
        h_l = taps[l][r0: r0 + n]
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
        assert ea < BF and ef < BF, f"layer {l}: attn {ea:.3e} ffn {ef:.3e}"
    print(f"teacher-forced per-layer worst per-row L2 err {worst:.3e}", flush=True)


def test_full_width_80_layer_stage_sampled_layers():
    """The full-width 80-layer stage (136.9 GB of weights), 32 ragged prompts of 128..4096 tokens, then the 128 decode
    steps of the workload.  The oracle cannot run it whole: it evaluates the layers 0, 39 and 79 one at a time, each
    fed the residual stream the GPU had at that layer's entry (taps; layer 0: the stage input), and is compared with
    what the GPU had at the next layer's entry (layer 79: the stage outputs):
      * prefill: the shortest, the longest and one random sequence, at the first, the last and 16 random rows, plus
        the K / V rows the GPU cached for those sequences in that layer;
      * decode steps 0 and 127: all 32 rows, the oracle's cache of that layer holding the GPU's cached rows.
    Full depth is also checked for finiteness, the cache lengths, and bit-identical repetition of the prefill."""
    import paper_2311_11514_amd as hx
    from oracle import stage_oracle as so
    cfg = CONFIGS["l70_full"]
    lens = generate.prompt_lengths(cfg)
    T, b, L, H = sum(lens), cfg.batch, cfg.n_layers, cfg.hidden
    layers = (0, L // 2 - 1, L - 1)
    st = hx.Stage(H, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, L, 1, 0, cfg.dtype, cfg.rms_eps, cfg.rope_theta)
    oras = {}
    for l in range(L):
        w = generate.layer_weights(cfg, l, device="cuda")
        args = [w[k] for k in ORDER]
        st.load_layer(l, *args)
        if l in layers:
            oras[l] = so.OracleStage(H, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, 1, 1, 0, cfg.rms_eps, cfg.rope_theta)
            oras[l].load_layer(0, *args)
        del w, args
    print(f"loaded {st.weight_bytes() / 1e9:.1f} GB of weights; {T} prompt rows", flush=True)
    X = generate.hidden_rows(cfg, T, device="cuda")
    kv = st.kv_cache_create(b, max(lens) + cfg.decode_steps)
    tap_layers = sorted({l for l in layers if l > 0} | {l + 1 for l in layers if l + 1 < L})
    taps = {l: torch.empty(T, H, dtype=torch.float32, device="cuda") for l in tap_layers}
    for l, t in taps.items():
        st.set_tap(l, t)
    xin = to_dev(X, cfg)
    outp, outr = torch.empty_like(xin), torch.empty_like(xin)
    st.prefill(kv, xin, lens, outp, outr)
    torch.cuda.synchronize()
    assert torch.isfinite(outp.float()).all() and torch.isfinite(outr.float()).all()
    first = (outp.clone(), outr.clone())
    cu = np.concatenate([[0], np.cumsum(lens)])
    rng = np.random.default_rng(5)
    shortest, longest = int(np.argmin(lens)), int(np.argmax(lens))
    other = [s for s in range(b) if s not in (shortest, longest)]
    seqs = (shortest, longest, other[int(rng.integers(0, len(other)))])
    d = cfg.head_dim
    for l in layers:
        h_in = xin.float() if l == 0 else taps[l]
        for s in seqs:
            n = lens[s]
            rows = sorted(set([0, n - 1] + [int(v) for v in rng.integers(0, n, 16)]))
            sl = slice(int(cu[s]), int(cu[s]) + n)
            ref, K, V = oras[l].layer_rows(0, h_in[sl].cpu(), rows, split_ffn=(l == L - 1))
            tag = f"prefill layer {l}, sequence {s} (len {n}), {len(rows)} rows"
            if l == L - 1:
                check(f"{tag}, resid", outr[sl].float().cpu().numpy()[rows], ref[0], BF)
                check(f"{tag}, partial", outp[sl].float().cpu().numpy()[rows], ref[1], BF)
            else:
                out = taps[l + 1][sl].cpu().numpy()[rows]
                check(tag, out, ref, BF)
                # what the layer ADDED to the residual stream (deep in the stage the stream itself is large, and an error
                # of the layer would hide in it)
                h_rows = h_in[sl].cpu().numpy().astype(np.float64)[rows]
                check(f"{tag}: the layer's contribution", out - h_rows, ref - h_rows, BF)
            kk, vv = kv.read(l, s, 0, n)
            check(f"{tag}: cached K", kk.numpy().reshape(-1, d), K.reshape(-1, d), BF)
            check(f"{tag}: cached V", vv.numpy().reshape(-1, d), V.reshape(-1, d), BF)
    # bit-identical repetition of the whole 80-layer prefill
    for l in tap_layers:
        st.set_tap(l, None)
    st.prefill(kv, xin, lens, outp, outr)
    torch.cuda.synchronize()
    assert torch.equal(outp, first[0]) and torch.equal(outr, first[1])
    del taps, first
    # decode: all steps of the workload; layers 0 / 39 / 79 against the oracle at the first and the last step
    dtaps = {l: torch.empty(b, H, dtype=torch.float32, device="cuda") for l in tap_layers}
    steps = cfg.decode_steps
    for step in range(steps):
        compared = step in (0, steps - 1)
        for l in tap_layers:
            st.set_tap(l, dtaps[l] if compared else None)
        x = generate.hidden_rows(cfg, b, stream_id=1 + step, device="cuda")
        pg, hg = gpu_decode(st, kv, cfg, step, x.cpu())
        assert np.isfinite(pg).all() and np.isfinite(hg).all()
        if not compared:
            continue
        for l in layers:
            ora = oras[l]
            oc = ora.new_cache(b)
            for s in range(b):
                kk, vv = kv.read(l, s, 0, lens[s] + step)          # the context the new rows attend to
                oc.fill(0, s, kk, vv)
            h_in = so._f64(x) if l == 0 else dtaps[l].cpu().numpy().astype(np.float64)
            h_mid = h_in + ora.attn_partial(0, oc, h_in, list(range(b)))
            p_ffn = ora.ffn_partial(0, h_mid)
            tag = f"decode step {step}, layer {l}, all {b} rows"
            if l == L - 1:
                check(f"{tag}, resid", hg, h_mid, BF)
                check(f"{tag}, partial", pg, p_ffn, BF)
            else:
                out = dtaps[l + 1].cpu().numpy()
                check(tag, out, h_mid + p_ffn, BF)
                check(f"{tag}: the layer's contribution", out - h_in, h_mid + p_ffn - h_in, BF)
            # the row the GPU appended in this layer is the oracle's
            s = longest
            kk, vv = kv.read(l, s, lens[s] + step, 1)
            check(f"{tag}: appended K", kk.numpy().reshape(-1, d), oc.k[0][s][-1:].reshape(-1, d), BF)
            check(f"{tag}: appended V", vv.numpy().reshape(-1, d), oc.v[0][s][-1:].reshape(-1, d), BF)
    assert kv.get_lengths(b) == [n + steps for n in lens]
