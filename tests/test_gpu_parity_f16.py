"""GPU parity of the fp16 stage (the 2-byte precision the cost model's B_type example names, Section 4.1 /
Appendix B): the same kernels as the bf16 stage compiled for the other 16-bit element, so the cases below walk the
same kernel switches -- prefill (fused, split and skinny projections, every GEMM tile family), decode row counts,
long-context split attention, the LM head -- against the float64 oracle fed inputs rounded to fp16.

Tolerance: fp16 carries 11 significand bits against bf16's 8, so the gate is the bf16 gate scaled by the ratio of
the unit roundoffs, 2e-2 * 2^-11 / 2^-9 = 5e-3 (same metrics, same rule)."""
import numpy as np
import pytest
import torch

from oracle import stage_oracle as so
from tests.helpers import TOL, check, gpu_decode, gpu_prefill, make_gpu_stage, make_oracle
from workloads import StageConfig, generate

pytestmark = pytest.mark.gpu

F128 = StageConfig("f16_mini128", "f16", 1024, 8, 2, 2816, 3, 2, (1,), batch=3, seed=41)
F64 = StageConfig("f16_mini64", "f16", 512, 8, 4, 1408, 2, 1, (0,), batch=2, seed=42)
F2K = StageConfig("f16_mini2k", "f16", 2048, 16, 4, 5632, 2, 2, (1,), batch=4, seed=43)
FRAG = StageConfig("f16_minirag", "f16", 1024, 8, 2, 2880, 2, 2, (0,), batch=2, seed=44)
FG16 = StageConfig("f16_minig16", "f16", 1024, 16, 1, 2816, 2, 1, (0,), batch=2, seed=45)
TOLF = TOL["f16"]


def _weights(cfg):
    return [generate.layer_weights(cfg, l) for l in range(cfg.n_layers)]


def _install_context(cfg, ctx, oc, kv):
    for layer in range(cfg.n_layers):
        for s, n in enumerate(ctx):
            k, v = generate.synthetic_kv(cfg, layer, s, n)
            oc.fill(layer, s, k, v)
            kv.fill(layer, s, k, v)
    kv.set_lengths(ctx)


@pytest.mark.parametrize("cfg,lens", [(F128, [37, 5, 64]), (F64, [16, 33]), (F2K, [100, 29, 150]), (FRAG, [129, 3]),
                                      (FRAG, [90]), (F128, [300, 41])])
def test_f16_prefill_then_decode(cfg, lens):
    w = _weights(cfg)
    rank = cfg.tp_ranks[0]
    X = generate.hidden_rows(cfg, sum(lens))
    ora = make_oracle(cfg, rank, w)
    oc = ora.new_cache(len(lens))
    p_ref, h_ref = ora.prefill(oc, X, lens)
    st = make_gpu_stage(cfg, rank, w)
    kv = st.kv_cache_create(len(lens), max(lens) + 64)
    p, h = gpu_prefill(st, kv, cfg, X, lens)
    check(f"{cfg.name} {lens} prefill resid", h, h_ref, TOLF)
    check(f"{cfg.name} {lens} prefill partial", p, p_ref, TOLF)
    assert kv.get_lengths(len(lens)) == lens
    for k in range(4):
        x = generate.hidden_rows(cfg, len(lens), stream_id=1 + k)
        p_ref, h_ref = ora.decode(oc, x)
        p, h = gpu_decode(st, kv, cfg, k, x)
        check(f"{cfg.name} decode {k} resid", h, h_ref, TOLF)
        check(f"{cfg.name} decode {k} partial", p, p_ref, TOLF)
    for layer in range(cfg.n_layers):
        for s, n in enumerate(lens):
            kk, vv = kv.read(layer, s, 0, n + 4)
            check(f"K layer {layer} seq {s}", kk.numpy().reshape(-1, cfg.head_dim), oc.k[layer][s].reshape(-1, cfg.head_dim), TOLF)
            check(f"V layer {layer} seq {s}", vv.numpy().reshape(-1, cfg.head_dim), oc.v[layer][s].reshape(-1, cfg.head_dim), TOLF)


@pytest.mark.parametrize("tile", [88, 98, 198, 194, 184, 84, 48, 94, 49, 44, 72])
def test_f16_prefill_every_gemm_tile_configuration(tile):
    import paper_2311_11514_amd as hx
    cfg = F128
    lens = [150, 3, 140]
    w = _weights(cfg)
    rank = cfg.tp_ranks[0]
    X = generate.hidden_rows(cfg, sum(lens), stream_id=7)
    ora = make_oracle(cfg, rank, w)
    p_ref, h_ref = ora.prefill(ora.new_cache(len(lens)), X, lens)
    st = make_gpu_stage(cfg, rank, w)
    kv = st.kv_cache_create(len(lens), 160)
    hx.set_gemm_tile(tile)
    try:
        p, h = gpu_prefill(st, kv, cfg, X, lens)
    finally:
        hx.set_gemm_tile(0)
    check(f"tile {tile} resid", h, h_ref, TOLF)
    check(f"tile {tile} partial", p, p_ref, TOLF)


@pytest.mark.parametrize("cfg,b", [(F64, 1), (F64, 2), (F128, 3), (F128, 16), (F128, 17), (F64, 32), (F2K, 4), (F2K, 9),
                                   (F128, 33), (FG16, 5), (FG16, 34)])
def test_f16_decode_batch_sizes(cfg, b):
    w = _weights(cfg)
    ctx = [1 + (7 * i) % 50 for i in range(b)]
    rank = cfg.tp_ranks[0]
    ora = make_oracle(cfg, rank, w)
    oc = ora.new_cache(b)
    st = make_gpu_stage(cfg, rank, w)
    kv = st.kv_cache_create(b, 64)
    _install_context(cfg, ctx, oc, kv)
    for step in range(2):
        x = generate.hidden_rows(cfg, b, stream_id=1 + step)
        p_ref, h_ref = ora.decode(oc, x)
        p, h = gpu_decode(st, kv, cfg, step, x)
        check(f"{cfg.name} b={b} step {step} resid", h, h_ref, TOLF)
        check(f"{cfg.name} b={b} step {step} partial", p, p_ref, TOLF)


@pytest.mark.parametrize("cfg,ctx", [(F128, [1700, 40, 1537]), (F64, [5, 1600]), (FG16, [1800, 33])])
def test_f16_decode_long_context_split_over_blocks(cfg, ctx):
    w = _weights(cfg)
    rank = cfg.tp_ranks[0]
    ora = make_oracle(cfg, rank, w)
    oc = ora.new_cache(len(ctx))
    st = make_gpu_stage(cfg, rank, w)
    kv = st.kv_cache_create(len(ctx), max(ctx) + 8)
    _install_context(cfg, ctx, oc, kv)
    outs = []
    for rep in range(2):
        kv.set_lengths(ctx)
        got = []
        for step in range(3):
            x = generate.hidden_rows(cfg, len(ctx), stream_id=1 + step)
            p, h = gpu_decode(st, kv, cfg, step, x)
            got.append((p, h))
            if rep == 0:
                p_ref, h_ref = ora.decode(oc, x)
                check(f"{cfg.name} ctx {ctx} step {step} resid", h, h_ref, TOLF)
                check(f"{cfg.name} ctx {ctx} step {step} partial", p, p_ref, TOLF)
        outs.append(got)
    for (p0, h0), (p1, h1) in zip(*outs):
        assert np.array_equal(p0, p1) and np.array_equal(h0, h1)


def test_f16_static_decode_matches_the_ordinary_entry_point():
    """The allocation-free decode entry point runs the fp16 kernels on the same file-scope scratch: same bits."""
    cfg = F128
    w = _weights(cfg)
    rank = cfg.tp_ranks[0]
    ctx = [70, 1, 33, 64]
    st = make_gpu_stage(cfg, rank, w)
    outs = []
    for static in (False, True):
        kv = st.kv_cache_create(len(ctx), 96)
        for layer in range(cfg.n_layers):
            for s, n in enumerate(ctx):
                kv.fill(layer, s, *generate.synthetic_kv(cfg, layer, s, n))
        kv.set_lengths(ctx)
        got = []
        for step in range(3):
            x = generate.hidden_rows(cfg, len(ctx), stream_id=1 + step).to("cuda", torch.float16).contiguous()
            p, h = torch.empty_like(x), torch.empty_like(x)
            (st.decode_static if static else st.decode)(kv, step, x, p, h)
            torch.cuda.synchronize()
            got.append((p.cpu(), h.cpu()))
        outs.append(got)
    for (p0, h0), (p1, h1) in zip(*outs):
        assert torch.equal(p0, p1) and torch.equal(h0, h1)


@pytest.mark.parametrize("t,n_rows", [(1, 5), (2, 32), (4, 17)])
def test_f16_head_greedy_vocab_parallel(t, n_rows):
    import paper_2311_11514_amd as hx
    cfg = StageConfig("f16_head1k", "f16", 1024, 8, 2, 2816, 1, 1, (0,), batch=1, seed=46, vocab=4104 if t == 1 else 4096 + 64 * t)
    hw = generate.head_weights(cfg)
    g, w = hw["g_final"], hw["w_lm"]
    a = generate.hidden_rows(cfg, n_rows, stream_id=3).to(torch.float16)
    b = (0.5 * generate.hidden_rows(cfg, n_rows, stream_id=4)).to(torch.float16)
    x = a.double().numpy() + b.double().numpy()
    gd, wd = g.double().numpy(), w.double().numpy()
    decisive = 0
    for r in range(t):
        hd = hx.Head(cfg.hidden, cfg.vocab, t, r, "f16", cfg.rms_eps)
        hd.load(g.cuda(), w.cuda())
        tok, val = hd.greedy(a.cuda().contiguous(), b.cuda().contiguous())
        torch.cuda.synchronize()
        tok, val = tok.cpu().numpy(), val.cpu().numpy().astype(np.float64)
        ids_ref, val_ref = so.head_shard_greedy(x, gd, wd, cfg.rms_eps, t, r)
        lo = r * (cfg.vocab // t)
        logits = so.rmsnorm(x, gd, cfg.rms_eps) @ wd[:, lo:lo + cfg.vocab // t]
        srt = np.sort(logits, axis=1)
        gap, scale = srt[:, -1] - srt[:, -2], np.max(np.abs(logits), axis=1)
        assert np.max(np.abs(val - val_ref) / scale) < TOLF
        clear = gap > 2 * TOLF * scale * 0.05
        decisive += int(np.sum(clear))
        assert np.array_equal(tok[clear], ids_ref[clear])
    assert decisive >= 0.8 * t * n_rows, "too many near-ties: the token comparison would be vacuous"


def test_f16_full_width_shards_decode_and_prefill():
    """The 70B shard shapes in fp16 at reduced depth (the oracle's cost is per layer): TP8 batch-16 decode from a
    context of 2048 (split projections, 16 splits on the narrow QKV matrix, split attention) and a TP4 prompt batch of
    4 x 512 rows (the large GEMM tiles), two layers each, every row compared."""
    from tests.test_gpu_parity_full import build_both, install_context
    from workloads import CONFIGS
    cfg = CONFIGS["l70_tp8_decode"].scaled(dtype="f16", n_layers=2, name="f16_tp8")
    st, ora = build_both(cfg, cfg.tp_ranks[0])
    b, ctx = cfg.batch, cfg.kv_context
    kv = st.kv_cache_create(b, ctx + 8)
    oc = ora.new_cache(b)
    install_context(cfg, kv, oc, range(b), ctx)
    kv.set_lengths([ctx] * b)
    for step in range(3):
        x = generate.hidden_rows(cfg, b, stream_id=1 + step)
        p_ref, h_ref = ora.decode(oc, x)
        p, h = gpu_decode(st, kv, cfg, step, x)
        check(f"f16 TP8 decode step {step} resid", h, h_ref, TOLF)
        check(f"f16 TP8 decode step {step} partial", p, p_ref, TOLF)
    del st, kv
    cfg = CONFIGS["l70_tp4_prefill"].scaled(dtype="f16", n_layers=2, name="f16_tp4")
    st, ora = build_both(cfg, cfg.tp_ranks[0])
    lens = generate.prompt_lengths(cfg)
    X = generate.hidden_rows(cfg, sum(lens))
    kv = st.kv_cache_create(len(lens), max(lens) + 8)
    oc = ora.new_cache(len(lens))
    p_ref, h_ref = ora.prefill(oc, X, lens)
    p, h = gpu_prefill(st, kv, cfg, X, lens)
    check("f16 TP4 prefill resid", h, h_ref, TOLF)
    check("f16 TP4 prefill partial", p, p_ref, TOLF)
    x = generate.hidden_rows(cfg, len(lens), stream_id=1)
    p_ref, h_ref = ora.decode(oc, x)
    p, h = gpu_decode(st, kv, cfg, 0, x)
    check("f16 TP4 decode after prefill resid", h, h_ref, TOLF)
    check("f16 TP4 decode after prefill partial", p, p_ref, TOLF)
