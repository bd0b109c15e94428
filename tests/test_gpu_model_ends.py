"""GPU parity of the model's ends next to the stage: embedding row gather, final RMSNorm + vocabulary-parallel LM
head + greedy arg-max, and a token-in / token-out greedy loop, all through the C ABI against the CPU oracle.

Arg-max is an integer decision taken from floating-point logits: token ids are compared only where the oracle's
decision is not a near-tie at the kernel's precision (the margin is stated per test), and every test asserts that
almost all of its rows are decisive, so that the comparison cannot pass vacuously."""
import numpy as np
import pytest
import torch

from oracle import stage_oracle as so
from tests.helpers import TOL, make_gpu_stage, make_oracle
from workloads import CONFIGS, StageConfig, generate

pytestmark = pytest.mark.gpu

HEAD1K = StageConfig("head1k", "bf16", 1024, 8, 2, 2816, 1, 1, (0,), batch=1, seed=31, vocab=4104)


def _shard_margin(x, g, w, eps, t, r):
    """Per row: gap between the best and the second-best logit of rank r's shard, and the largest |logit|."""
    V = w.shape[1]
    lo = r * (V // t)
    logits = so.rmsnorm(np.asarray(x, np.float64), np.asarray(g, np.float64), eps) @ np.asarray(w, np.float64)[:, lo:lo + V // t]
    srt = np.sort(logits, axis=1)
    return srt[:, -1] - srt[:, -2], np.max(np.abs(logits), axis=1)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_embed_rows_matches_the_gather(dtype):
    import paper_2311_11514_amd as hx
    cfg = StageConfig("emb", dtype, 512, 8, 2, 1408, 1, 1, (0,), batch=1, seed=33, vocab=300)
    table = generate.head_weights(cfg)["embedding"]
    tok = np.array([0, 299, 17, 17, 123, 5, 298, 1], dtype=np.int32)
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    out = hx.embed_rows(table.to("cuda", td).contiguous(), torch.tensor(tok, device="cuda"))
    torch.cuda.synchronize()
    ref = so.embed_rows(table.to(td).double().numpy(), tok)
    assert np.array_equal(out.double().cpu().numpy(), ref)          # a copy: bit-exact
    # ids outside the table are clamped to its ends (documented behaviour of the boundary)
    out = hx.embed_rows(table.to("cuda", td).contiguous(), torch.tensor([-3, 10 ** 6], dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    assert np.array_equal(out.double().cpu().numpy(), so.embed_rows(table.to(td).double().numpy(), [0, 299]))


@pytest.mark.parametrize("t,n_rows", [(1, 1), (1, 5), (2, 32), (1, 40), (4, 17)])
def test_head_greedy_bf16_vocab_parallel(t, n_rows):
    """Vocabulary 4104: the t = 1 shard is not a multiple of 16 (zero-padded tiles must never win), t = 2 / 4 shards
    are; 1, 5, 17, 32 and 40 rows cover the single-kernel projection, both batched forms and the 32-row chunking."""
    import paper_2311_11514_amd as hx
    cfg = HEAD1K.scaled(vocab=4104 if t == 1 else 4096 + 64 * t)
    hw = generate.head_weights(cfg)
    g, w = hw["g_final"], hw["w_lm"]
    a = generate.hidden_rows(cfg, n_rows, stream_id=3).to(torch.bfloat16)
    b = (0.5 * generate.hidden_rows(cfg, n_rows, stream_id=4)).to(torch.bfloat16)
    x = a.double().numpy() + b.double().numpy()
    cands = []
    decisive = 0
    for r in range(t):
        hd = hx.Head(cfg.hidden, cfg.vocab, t, r, "bf16", cfg.rms_eps)
        hd.load(g.cuda(), w.cuda())
        tok, val = hd.greedy(a.cuda().contiguous(), b.cuda().contiguous())
        torch.cuda.synchronize()
        tok, val = tok.cpu().numpy(), val.cpu().numpy().astype(np.float64)
        ids_ref, val_ref = so.head_shard_greedy(x, g.double().numpy(), w.double().numpy(), cfg.rms_eps, t, r)
        gap, scale = _shard_margin(x, g.double().numpy(), w.double().numpy(), cfg.rms_eps, t, r)
        assert np.all((tok >= r * cfg.vocab // t) & (tok < (r + 1) * cfg.vocab // t))
        # the winning logit itself, to the bf16 tolerance relative to the row's largest logit
        assert np.max(np.abs(val - val_ref) / scale) < TOL["bf16"]
        clear = gap > 2 * TOL["bf16"] * scale * 0.05          # 0.1 % of the row's logit scale
        decisive += int(np.sum(clear))
        assert np.array_equal(tok[clear], ids_ref[clear])
        cands.append((tok, val))
    assert decisive >= 0.8 * t * n_rows, "too many near-ties: the token comparison would be vacuous"
    # the group's choice from the ranks' candidates
    ref_cands = [so.head_shard_greedy(x, g.double().numpy(), w.double().numpy(), cfg.rms_eps, t, r) for r in range(t)]
    merged, merged_ref = so.merge_greedy(cands), so.merge_greedy(ref_cands)
    full_gap, full_scale = _shard_margin(x, g.double().numpy(), w.double().numpy(), cfg.rms_eps, 1, 0)
    clear = full_gap > 2 * TOL["bf16"] * full_scale * 0.05
    assert np.array_equal(merged[clear], merged_ref[clear]) and np.sum(clear) >= 0.8 * n_rows


def test_head_errors():
    import paper_2311_11514_amd as hx
    with pytest.raises(hx.HexgenError):
        hx.Head(1024, 4100, 3, 0, "bf16")            # vocabulary not divisible by the degree
    with pytest.raises(hx.HexgenError):
        hx.Head(1000, 4096, 1, 0, "bf16")            # hidden not a multiple of 128
    hd = hx.Head(1024, 4096, 1, 0, "bf16")
    x = torch.zeros(1, 1024, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(hx.HexgenError):
        hd.greedy(x)                                  # before load


def test_tiny_f32_token_in_token_out_greedy_loop():
    """Embedding -> stage (prefill, then decode) -> head -> next token, entirely on the GPU, against the oracle doing the
    same in float64: the 8 generated tokens are identical (the oracle's decisions are checked not to be near-ties)."""
    import paper_2311_11514_amd as hx
    cfg = CONFIGS["tiny_f32"].scaled(tp_degree=1, tp_ranks=(0,))
    w = [generate.layer_weights(cfg, l) for l in range(cfg.n_layers)]
    hw = generate.head_weights(cfg)
    E, g, wl = hw["embedding"], hw["g_final"], hw["w_lm"]
    rng = np.random.default_rng(7)
    prompt = rng.integers(0, cfg.vocab, size=cfg.prompt_len).astype(np.int32)

    ora = make_oracle(cfg, 0, w)
    oc = ora.new_cache(1)
    st = make_gpu_stage(cfg, 0, w)
    kv = st.kv_cache_create(1, cfg.prompt_len + cfg.decode_steps + 1)
    hd = hx.Head(cfg.hidden, cfg.vocab, 1, 0, "f32", cfg.rms_eps)
    hd.load(g.cuda(), wl.cuda())
    E_dev = E.to("cuda", torch.float32).contiguous()

    # oracle
    toks_o = []
    x = so.embed_rows(E.double().numpy(), prompt)
    p, h = ora.prefill(oc, x, [cfg.prompt_len])
    for step in range(cfg.decode_steps):
        tok, logits = so.greedy_head((h + p)[-1], g, wl, cfg.rms_eps)
        top2 = np.sort(logits)[-2:]
        assert top2[1] - top2[0] > 1e-6, "oracle argmax is a near-tie; token comparison would be meaningless"
        toks_o.append(tok)
        p, h = ora.decode(oc, so.embed_rows(E.double().numpy(), [tok]))

    # GPU: tokens never leave the device between the head and the embedding
    toks_g = []
    xg = hx.embed_rows(E_dev, torch.tensor(prompt, device="cuda"))
    outp, outr = torch.empty_like(xg), torch.empty_like(xg)
    st.prefill(kv, xg, [cfg.prompt_len], outp, outr)
    tok, _ = hd.greedy(outr[-1:].contiguous(), outp[-1:].contiguous())
    for step in range(cfg.decode_steps):
        toks_g.append(tok)
        x1 = hx.embed_rows(E_dev, tok)
        p1, r1 = torch.empty_like(x1), torch.empty_like(x1)
        st.decode(kv, step, x1, p1, r1)
        tok, _ = hd.greedy(r1, p1)
    torch.cuda.synchronize()
    assert [int(t.item()) for t in toks_g] == toks_o


def test_head_full_size_llama70b_shape():
    """The full Llama-2-70B head, 8192 x 32000 bf16 (524 MB), one and four rows: winning logit and token against the
    oracle's float64 matrix-vector products."""
    import paper_2311_11514_amd as hx
    cfg = StageConfig("head70b", "bf16", 8192, 64, 8, 28672, 1, 1, (0,), batch=1, seed=41, vocab=32000)
    hw = generate.head_weights(cfg, device="cuda")
    g, wl = hw["g_final"], hw["w_lm"]
    hd = hx.Head(cfg.hidden, cfg.vocab, 1, 0, "bf16", cfg.rms_eps)
    hd.load(g, wl)
    g64, w64 = g.double().cpu().numpy(), wl.double().cpu().numpy()
    for n in (1, 4):
        a = generate.hidden_rows(cfg, n, stream_id=9).to(torch.bfloat16)
        tok, val = hd.greedy(a.cuda().contiguous())
        torch.cuda.synchronize()
        ids_ref, val_ref = so.head_shard_greedy(a.double().numpy(), g64, w64, cfg.rms_eps, 1, 0)
        gap, scale = _shard_margin(a.double().numpy(), g64, w64, cfg.rms_eps, 1, 0)
        assert np.max(np.abs(val.cpu().numpy() - val_ref) / scale) < TOL["bf16"]
        clear = gap > 2 * TOL["bf16"] * scale * 0.05
        assert np.sum(clear) >= n - 1 and np.array_equal(tok.cpu().numpy()[clear], ids_ref[clear])
