"""GPU parity on sizes the CPU oracle finishes in seconds: the tiny fp32 stage (both ranks, group mode,
greedy tokens) and reduced-width bf16 stages that still span several MFMA tiles and ragged tails."""
import numpy as np
import pytest
import torch

from workloads import CONFIGS, StageConfig, generate
from tests.helpers import (ORDER, TOL, gpu_decode, gpu_prefill, make_gpu_stage, make_oracle, row_rel_err, to_dev)

pytestmark = pytest.mark.gpu

TINY = CONFIGS["tiny_f32"]

# reduced-width bf16 stages: same structure as the 70B shards (GQA, head_dim 128 and 64, SwiGLU)
MINI128 = StageConfig("mini128", "bf16", 1024, 8, 2, 2816, 3, 2, (1,), batch=3, seed=11)
MINI64 = StageConfig("mini64", "bf16", 512, 8, 4, 1408, 2, 1, (0,), batch=2, seed=12)
MINI2K = StageConfig("mini2k", "bf16", 2048, 16, 4, 5632, 2, 2, (1,), batch=4, seed=13)
# FFN shard of 1440: 180 feature tiles for W1/W3 (not a multiple of the 8 a block owns) and 45 k-tiles for W2 (odd)
MINIRAG = StageConfig("minirag", "bf16", 1024, 8, 2, 2880, 2, 2, (0,), batch=2, seed=14)
# 16 query heads on one kv head: every column of the decode attention's 16-column MFMA results is a live head
MINIG16 = StageConfig("minig16", "bf16", 1024, 16, 1, 2816, 2, 1, (0,), batch=2, seed=15)
# wide enough (40 to 64 feature blocks, 128 to 160 k-tiles) that a short prompt's skinny launches pair their splits inside
# 8-wave blocks, in all four epilogues
MINI5K = StageConfig("mini5k", "bf16", 5120, 40, 8, 4096, 1, 1, (0,), batch=1, seed=16)
# 140 k-tiles in 4 splits of 35: the two wave groups of an 8-wave skinny block walk 17 and 18 k-steps (QKV, 45 feature blocks)
MINIODD = StageConfig("miniodd", "bf16", 4480, 35, 5, 4480, 1, 1, (0,), batch=1, seed=17)


def _weights(cfg, n_layers=None):
    return [generate.layer_weights(cfg, l) for l in range(n_layers or cfg.n_layers)]


def test_tiny_f32_solo_prefill_and_decode():
    cfg = TINY
    w = _weights(cfg)
    X = generate.hidden_rows(cfg, cfg.prompt_len)
    for rank in cfg.tp_ranks:
        ora = make_oracle(cfg, rank, w)
        oc = ora.new_cache(1)
        p_ref, h_ref = ora.prefill(oc, X, [cfg.prompt_len])
        st = make_gpu_stage(cfg, rank, w)
        kv = st.kv_cache_create(1, 64)
        p, h = gpu_prefill(st, kv, cfg, X, [cfg.prompt_len])
        assert row_rel_err(p, p_ref) < TOL["f32"] and row_rel_err(h, h_ref) < TOL["f32"]
        for k in range(4):
            x = generate.hidden_rows(cfg, 1, stream_id=1 + k)
            p_ref, h_ref = ora.decode(oc, x)
            p, h = gpu_decode(st, kv, cfg, k, x)
            assert row_rel_err(p, p_ref) < TOL["f32"] and row_rel_err(h, h_ref) < TOL["f32"]
        # cache contents (K after rotation) match the oracle's cache
        kk, vv = kv.read(1, 0, 0, cfg.prompt_len + 4)
        assert row_rel_err(kk.numpy().reshape(-1, cfg.head_dim), oc.k[1][0].reshape(-1, cfg.head_dim)) < TOL["f32"]
        assert row_rel_err(vv.numpy().reshape(-1, cfg.head_dim), oc.v[1][0].reshape(-1, cfg.head_dim)) < TOL["f32"]


def _gpu_group_forward(stages, kvs, cfg, h_in, seq_lens, batch):
    """All ranks one after another on the same GPU, partials summed in rank order (fp32)."""
    import paper_2311_11514_amd as hx
    h = h_in.to(device="cuda", dtype=torch.float32).contiguous()
    part = torch.empty_like(h)
    parts = None
    for layer in range(cfg.n_layers):
        for which in (0, 1):
            last = layer == cfg.n_layers - 1 and which == 1
            ps = []
            for st, kv in zip(stages, kvs):
                p = torch.empty_like(h)
                st.run_sublayer(kv, layer, which, h, seq_lens, batch, p)
                ps.append(p)
            if last:
                parts = ps
            else:
                for p in ps:
                    hx.accumulate_f32(h, p)
    for kv in kvs:
        kv.commit(seq_lens, batch)
    torch.cuda.synchronize()
    return [p.cpu().numpy() for p in parts], h.cpu().numpy()


def test_tiny_f32_group_mode_greedy_tokens():
    """The tiny configuration as stated: both ranks run, partials summed, 32-row prompt, 8 greedy steps
    through a 1000-entry embedding / LM head; GPU tokens must equal the oracle's."""
    from oracle import stage_oracle as so
    cfg = TINY
    w = _weights(cfg)
    head = generate.head_weights(cfg)
    E = head["embedding"]
    X = generate.hidden_rows(cfg, cfg.prompt_len)

    oracles = [make_oracle(cfg, r, w) for r in cfg.tp_ranks]
    ocaches = [o.new_cache(1) for o in oracles]
    stages = [make_gpu_stage(cfg, r, w) for r in cfg.tp_ranks]
    kvs = [s.kv_cache_create(1, 64) for s in stages]

    def pick(x_last):
        return so.greedy_head(x_last, head["g_final"], head["w_lm"], cfg.rms_eps)

    x_o, x_g = X, X
    seq_lens, toks_o, toks_g = [cfg.prompt_len], [], []
    for step in range(cfg.decode_steps):
        seqs = [0] * x_o.shape[0]
        parts_o, resid_o = so.group_forward(oracles, ocaches, x_o, seqs)
        parts_g, resid_g = _gpu_group_forward(stages, kvs, cfg, x_g, seq_lens if step == 0 else None, 1)
        out_o = resid_o + sum(parts_o)
        out_g = resid_g + sum(np.asarray(p, dtype=np.float64) for p in parts_g)
        assert row_rel_err(out_g, out_o) < TOL["f32"]
        for pg, po in zip(parts_g, parts_o):
            assert row_rel_err(pg, po) < TOL["f32"]
        t_o, logits_o = pick(out_o[-1])
        t_g, _ = pick(out_g[-1])
        top2 = np.sort(logits_o)[-2:]
        assert top2[1] - top2[0] > 1e-6, "oracle argmax is a near-tie; token comparison would be meaningless"
        toks_o.append(t_o)
        toks_g.append(t_g)
        x_o = E[t_o][None, :]
        x_g = E[t_g][None, :]
    assert toks_g == toks_o


@pytest.mark.parametrize("cfg,lens", [(MINI128, [37, 5, 64]), (MINI64, [16, 33]), (MINI2K, [70]), (MINI2K, [100, 29, 150]),
                                      (MINIRAG, [90]), (MINIRAG, [128]), (MINIRAG, [129, 3]),
                                      (MINI64, [1, 128, 129, 256, 5, 127, 130, 64, 33, 257, 2]),
                                      (MINI2K, [300, 212]), (MINI2K, [520, 500]), (MINI5K, [128]), (MINI5K, [61, 40]), (MINIODD, [128]), (MINIODD, [77])])
def test_bf16_small_prefill_then_decode(cfg, lens):
    """Short prompts: few token tiles, so the projections with at least 32 k-tiles split their contraction over
    several blocks and finish in a second pass: up to 128 rows through the skinny kernel (weights in a register ring),
    beyond through the LDS-staged kernel; MINI64 (16 k-tiles) does neither.  MINIRAG has a ragged last feature block
    and an odd number of k-tiles; 128 and 129 + 3 rows sit on either side of the one-token-tile limit.  The batch of
    eleven prompts around the 128-row block size gives the prefill attention a work list of 16 (sequence, block) pairs
    in an order that differs from the batch order (longest walks first, dealt over the XCDs).  512 and 1020 rows on
    MINI2K: split launches of 12 to 88 tiles, whose second pass finishes a tile with four blocks (up to 64 tiles) or
    two (W1/W3 at 1020 rows), each with its share of the tile's waves.  MINI5K: the skinny kernel's 8-wave form (two
    groups of waves on two halves of a block's contraction, summed through LDS) in every epilogue, full and ragged tile;
    MINIODD: halves of unequal length."""
    w = _weights(cfg)
    rank = cfg.tp_ranks[0]
    X = generate.hidden_rows(cfg, sum(lens))
    ora = make_oracle(cfg, rank, w)
    oc = ora.new_cache(len(lens))
    p_ref, h_ref = ora.prefill(oc, X, lens)
    st = make_gpu_stage(cfg, rank, w)
    kv = st.kv_cache_create(len(lens), max(lens) + 64)
    p, h = gpu_prefill(st, kv, cfg, X, lens)
    assert row_rel_err(h, h_ref) < TOL["bf16"]
    assert row_rel_err(p, p_ref) < TOL["bf16"]
    assert kv.get_lengths(len(lens)) == lens
    for k in range(5):
        x = generate.hidden_rows(cfg, len(lens), stream_id=1 + k)
        p_ref, h_ref = ora.decode(oc, x)
        p, h = gpu_decode(st, kv, cfg, k, x)
        assert row_rel_err(h, h_ref) < TOL["bf16"], f"decode step {k}"
        assert row_rel_err(p, p_ref) < TOL["bf16"], f"decode step {k}"
    # K (after rotation) and V written by prefill and decode, for every layer and sequence
    for layer in range(cfg.n_layers):
        for s, n in enumerate(lens):
            kk, vv = kv.read(layer, s, 0, n + 5)
            assert row_rel_err(kk.numpy().reshape(-1, cfg.head_dim), oc.k[layer][s].reshape(-1, cfg.head_dim)) < TOL["bf16"]
            assert row_rel_err(vv.numpy().reshape(-1, cfg.head_dim), oc.v[layer][s].reshape(-1, cfg.head_dim)) < TOL["bf16"]


@pytest.mark.parametrize("tile", [88, 98, 198, 194, 184, 84, 48, 94, 49, 44, 72])
def test_bf16_prefill_every_gemm_tile_configuration(tile):
    """Every instantiation of the prefill projection GEMM (4- and 8-wave blocks, 256/128-wide tiles, odd and even
    load counts per stage), forced through the library's tile hook, on a ragged prompt batch that spans several
    block tiles with a ragged tail (293 rows: one full 256-token block and a partial one)."""
    import paper_2311_11514_amd as hx
    cfg = MINI128
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
    assert row_rel_err(h, h_ref) < TOL["bf16"]
    assert row_rel_err(p, p_ref) < TOL["bf16"]
    with pytest.raises(hx.HexgenError):
        hx.set_gemm_tile(17)


# a launch of a few more than a multiple of 256 large GEMM tiles: the feature blocks that fill whole rounds of the chip go
# first, the remaining one follows as a launch of its own with a split contraction.  MINIREM13: W1/W3 has 17 x 16 = 272
# tiles at 4096 rows (SwiGLU epilogue on a feature range); MINIREMO: W_O has 8 x 33 = 264 tiles at 8448 rows (residual
# epilogue, its sums of squares indexed by feature block).
MINIREM13 = StageConfig("minirem13", "bf16", 1024, 8, 2, 2176, 1, 1, (0,), batch=16, seed=16)
MINIREMO = StageConfig("miniremo", "bf16", 2048, 16, 2, 256, 1, 1, (0,), batch=33, seed=17)


@pytest.mark.parametrize("cfg,lens", [(MINIREM13, [256] * 16), (MINIREMO, [256] * 33)])
def test_bf16_prefill_launch_with_a_nearly_empty_last_round(cfg, lens):
    w = _weights(cfg)
    rank = cfg.tp_ranks[0]
    X = generate.hidden_rows(cfg, sum(lens))
    ora = make_oracle(cfg, rank, w)
    oc = ora.new_cache(len(lens))
    p_ref, h_ref = ora.prefill(oc, X, lens)
    st = make_gpu_stage(cfg, rank, w)
    kv = st.kv_cache_create(len(lens), max(lens) + 8)
    p, h = gpu_prefill(st, kv, cfg, X, lens)
    assert row_rel_err(h, h_ref) < TOL["bf16"]
    assert row_rel_err(p, p_ref) < TOL["bf16"]
    x = generate.hidden_rows(cfg, len(lens), stream_id=1)
    p_ref, h_ref = ora.decode(oc, x)
    p, h = gpu_decode(st, kv, cfg, 0, x)
    assert row_rel_err(h, h_ref) < TOL["bf16"] and row_rel_err(p, p_ref) < TOL["bf16"]


def test_bf16_decode_from_synthetic_context():
    """Decode-only workloads start from an installed synthetic KV context (ragged lengths here)."""
    cfg = MINI128
    w = _weights(cfg)
    rank = cfg.tp_ranks[0]
    ctx = [70, 1, 33, 64]
    ora = make_oracle(cfg, rank, w)
    oc = ora.new_cache(len(ctx))
    st = make_gpu_stage(cfg, rank, w)
    kv = st.kv_cache_create(len(ctx), 96)
    for layer in range(cfg.n_layers):
        for s, n in enumerate(ctx):
            k, v = generate.synthetic_kv(cfg, layer, s, n)
            oc.fill(layer, s, k, v)
            kv.fill(layer, s, k, v)
    kv.set_lengths(ctx)
    import paper_2311_11514_amd as hx
    with pytest.raises(hx.HexgenError):
        st.time_w13_decode(1)                       # no decode call yet
    for step in range(3):
        x = generate.hidden_rows(cfg, len(ctx), stream_id=1 + step)
        p_ref, h_ref = ora.decode(oc, x)
        p, h = gpu_decode(st, kv, cfg, step, x)
        assert row_rel_err(h, h_ref) < TOL["bf16"] and row_rel_err(p, p_ref) < TOL["bf16"]
        # the measurement pass of the FFN up-projection touches nothing the next step depends on
        ms, n = st.time_w13_decode(2)
        assert ms > 0 and n == 2 * cfg.n_layers


@pytest.mark.parametrize("cfg,b", [(MINI64, 32), (MINI64, 1), (MINI64, 2), (MINI128, 3), (MINI128, 16), (MINI128, 17),
                                   (MINI64, 31), (MINI2K, 3), (MINI2K, 4), (MINI2K, 8), (MINI2K, 9), (MINI128, 33),
                                   (MINI64, 40), (MINIG16, 2), (MINIG16, 5), (MINIG16, 34)])
def test_bf16_decode_batch_sizes(cfg, b):
    """Decode across the row counts that switch kernels: 1-2 rows (one kernel per projection, operand in LDS),
    3-16 rows (split contraction, one token tile), 17-32 rows (two token tiles); MINI128's FFN has 44 k-tiles, so its
    splits end in a partial chunk.  MINI2K's contractions are long enough (64 and 88 k-tiles) for its small matrices
    to take the single-kernel path with 3-8 rows (every block fetching the rows' operand pieces itself; its W_O, with 32
    k-tiles, stays on the split path), and the split path from 9 rows on.  More than 32 rows (33, 40) leave the
    weight-streaming decode kernels for the prefill kernels with one new row per sequence."""
    w = _weights(cfg)
    ctx = [1 + (7 * i) % 50 for i in range(b)]
    rank = cfg.tp_ranks[0]
    ora = make_oracle(cfg, rank, w)
    oc = ora.new_cache(b)
    st = make_gpu_stage(cfg, rank, w)
    kv = st.kv_cache_create(b, 64)
    for layer in range(cfg.n_layers):
        for s, n in enumerate(ctx):
            k, v = generate.synthetic_kv(cfg, layer, s, n)
            oc.fill(layer, s, k, v)
            kv.fill(layer, s, k, v)
    kv.set_lengths(ctx)
    for step in range(2):
        x = generate.hidden_rows(cfg, b, stream_id=1 + step)
        p_ref, h_ref = ora.decode(oc, x)
        p, h = gpu_decode(st, kv, cfg, step, x)
        assert row_rel_err(h, h_ref) < TOL["bf16"] and row_rel_err(p, p_ref) < TOL["bf16"]


@pytest.mark.parametrize("cfg,ctx", [(MINI128, [1700, 40, 1537]), (MINI64, [2100]), (MINI64, [5, 1600]), (MINIG16, [1800, 33]),
                                     (MINI64, [16500]), (MINI128, [9001, 300])])
def test_bf16_decode_long_context_split_over_blocks(cfg, ctx):
    """Few sequences with a long context: the attention of one (sequence, kv head) is split over several blocks and
    merged by the block that finishes last.  Ragged lengths leave the short sequences' later splits empty; the second
    pass over the same state must give the same bits whichever block happened to merge."""
    w = _weights(cfg)
    rank = cfg.tp_ranks[0]
    ora = make_oracle(cfg, rank, w)
    oc = ora.new_cache(len(ctx))
    st = make_gpu_stage(cfg, rank, w)
    kv = st.kv_cache_create(len(ctx), max(ctx) + 8)
    for layer in range(cfg.n_layers):
        for s, n in enumerate(ctx):
            k, v = generate.synthetic_kv(cfg, layer, s, n)
            oc.fill(layer, s, k, v)
            kv.fill(layer, s, k, v)
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
                assert row_rel_err(h, h_ref) < TOL["bf16"] and row_rel_err(p, p_ref) < TOL["bf16"]
        outs.append(got)
    for (p0, h0), (p1, h1) in zip(*outs):
        assert np.array_equal(p0, p1) and np.array_equal(h0, h1)


@pytest.mark.parametrize("nsplit", [1, 2, 3, 5, 8])
def test_bf16_decode_attention_with_a_forced_split(nsplit):
    """Any split of the decode attention gives the same result to rounding: forced through the library's hook on a ragged
    batch whose short sequences have fewer 32-position tiles than splits (their surplus blocks leave at once and must
    not be waited for), on both the ordinary and the allocation-free entry point."""
    import paper_2311_11514_amd as hx
    cfg = MINI128
    ctx = [70, 1, 33, 300, 31]
    w = _weights(cfg)
    rank = cfg.tp_ranks[0]
    ora = make_oracle(cfg, rank, w)
    st = make_gpu_stage(cfg, rank, w)
    hx.set_attn_split(nsplit)
    try:
        for static in (False, True):
            oc = ora.new_cache(len(ctx))
            kv = st.kv_cache_create(len(ctx), 320)
            for layer in range(cfg.n_layers):
                for s, n in enumerate(ctx):
                    k, v = generate.synthetic_kv(cfg, layer, s, n)
                    oc.fill(layer, s, k, v)
                    kv.fill(layer, s, k, v)
            kv.set_lengths(ctx)
            for step in range(3):
                x = generate.hidden_rows(cfg, len(ctx), stream_id=1 + step)
                p_ref, h_ref = ora.decode(oc, x)
                xin = to_dev(x, cfg)
                p, h = torch.empty_like(xin), torch.empty_like(xin)
                (st.decode_static if static else st.decode)(kv, step, xin, p, h)
                torch.cuda.synchronize()
                assert row_rel_err(h.float().cpu().numpy(), h_ref) < TOL["bf16"]
                assert row_rel_err(p.float().cpu().numpy(), p_ref) < TOL["bf16"]
    finally:
        hx.set_attn_split(0)
    with pytest.raises(hx.HexgenError):
        hx.set_attn_split(9)


def test_run_to_run_determinism_bf16():
    cfg = MINI128
    w = _weights(cfg)
    lens = [37, 5, 64]
    X = generate.hidden_rows(cfg, sum(lens))
    st = make_gpu_stage(cfg, 1, w)
    kv = st.kv_cache_create(3, 128)
    outs = []
    for _ in range(2):
        p, h = gpu_prefill(st, kv, cfg, X, lens)
        x = generate.hidden_rows(cfg, 3, stream_id=1)
        pd, hd = gpu_decode(st, kv, cfg, 0, x)
        outs.append((p, h, pd, hd))
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)


def test_error_paths_on_device():
    import paper_2311_11514_amd as hx
    cfg = MINI64
    w = _weights(cfg)
    st = make_gpu_stage(cfg, 0, w)
    kv = st.kv_cache_create(2, 40)
    x = to_dev(generate.hidden_rows(cfg, 2), cfg)
    out = torch.empty_like(x)
    with pytest.raises(hx.HexgenError) as e:
        st.decode(kv, 0, x, out)            # decode before prefill
    assert e.value.status == 3
    X = to_dev(generate.hidden_rows(cfg, 60), cfg)
    O = torch.empty_like(X)
    with pytest.raises(hx.HexgenError) as e:
        st.prefill(kv, X, [41, 19], O)      # longer than max_seq
    assert e.value.status == 4
    st.prefill(kv, X[:50], [40, 10], O[:50])
    with pytest.raises(hx.HexgenError) as e:
        st.decode(kv, 1, x, out)            # wrong step number
    assert e.value.status == 3
    with pytest.raises(hx.HexgenError) as e:
        st.decode(kv, 0, x, out)            # sequence 0 is full
    assert e.value.status == 4
    torch.cuda.synchronize()


def test_bf16_prefill_and_decode_on_a_side_stream():
    """A fresh stage used first on a non-default (non-blocking) torch stream: the workspace the first call allocates
    is zero-filled before any kernel of the call can read it, whatever stream the caller launches on; covers the
    batched decode path (split partial sums) and the split-KV attention (arrival counters) as well."""
    cfg = MINI128
    lens = [1700, 40, 1537]
    w = _weights(cfg)
    rank = cfg.tp_ranks[0]
    ora = make_oracle(cfg, rank, w)
    oc = ora.new_cache(len(lens))
    st = make_gpu_stage(cfg, rank, w)
    side = torch.cuda.Stream()
    kv = st.kv_cache_create(len(lens), max(lens) + 8)
    X = generate.hidden_rows(cfg, 77, stream_id=9)
    p_ref, h_ref = ora.prefill(ora.new_cache(2), X, [50, 27])
    xin = to_dev(X, cfg)
    outp, outr = torch.empty_like(xin), torch.empty_like(xin)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        st.prefill(kv, xin, [50, 27], outp, outr, stream=side)
    side.synchronize()
    assert row_rel_err(outr.float().cpu().numpy(), h_ref) < TOL["bf16"]
    assert row_rel_err(outp.float().cpu().numpy(), p_ref) < TOL["bf16"]
    # decode from long synthetic contexts on the same side stream
    for l in range(cfg.n_layers):
        for s, n in enumerate(lens):
            k, v = generate.synthetic_kv(cfg, l, s, n)
            kv.fill(l, s, k, v)
            oc.fill(l, s, k, v)
    kv.set_lengths(lens)
    for step in range(2):
        x = generate.hidden_rows(cfg, len(lens), stream_id=1 + step)
        p_ref, h_ref = ora.decode(oc, x)
        xd = to_dev(x, cfg)
        op, orr = torch.empty_like(xd), torch.empty_like(xd)
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            st.decode(kv, step, xd, op, orr, stream=side)
        side.synchronize()
        assert row_rel_err(orr.float().cpu().numpy(), h_ref) < TOL["bf16"]
        assert row_rel_err(op.float().cpu().numpy(), p_ref) < TOL["bf16"]


def test_rope_theta_changed_after_cache_creation_is_refused():
    import paper_2311_11514_amd as hx
    cfg = MINI64
    st = make_gpu_stage(cfg, 0, _weights(cfg))
    kv = st.kv_cache_create(1, 64)
    assert hx.lib.hexgen_stage_set_params(st.handle, 1e-5, 500000.0) == 0
    x = to_dev(generate.hidden_rows(cfg, 8), cfg)
    with pytest.raises(hx.HexgenError) as e:
        st.prefill(kv, x, [8], torch.empty_like(x), torch.empty_like(x))
    assert e.value.status == 3          # HEXGEN_ERR_STATE
    kv2 = st.kv_cache_create(1, 64)     # a cache created under the new theta is accepted
    st.prefill(kv2, x, [8], torch.empty_like(x), torch.empty_like(x))
    torch.cuda.synchronize()
