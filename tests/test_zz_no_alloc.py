"""The decode entry point that allocates nothing (hexgen_stage_decode_static) against hexgen_stage_decode.

Same stage, two caches with the same synthetic context: one is advanced by the ordinary entry point, the other by the
static-scratch one; outputs and appended K / V rows must agree exactly (same kernels, same order of summation).  Two
calls in a row on the shared scratch array, the second with a smaller batch, then a second step of each."""
import pytest
import torch

from workloads import StageConfig, generate
from tests.helpers import make_gpu_stage, to_dev

pytestmark = pytest.mark.gpu

CFG = StageConfig("mini128_static", "bf16", 1024, 8, 2, 2816, 3, 2, (1,), batch=16, seed=31)


def _context(cfg, st, lens):
    kvs = [st.kv_cache_create(len(lens), max(lens) + 8) for _ in range(2)]
    for l in range(cfg.n_layers):
        for s, n in enumerate(lens):
            k, v = generate.synthetic_kv(cfg, l, s, n)
            for kv in kvs:
                kv.fill(l, s, k, v)
    for kv in kvs:
        kv.set_lengths(lens)
    return kvs


def test_static_scratch_decode_matches_decode_on_two_calls_in_a_row():
    cfg = CFG
    w = [generate.layer_weights(cfg, l) for l in range(cfg.n_layers)]
    st = make_gpu_stage(cfg, cfg.tp_ranks[0], w)
    # first call: 16 sequences, contexts long enough that the attention splits over blocks (arrival counters and
    # partials in the scratch) and the projections take the batched path (split partial sums in the scratch);
    # second call: 3 sequences (the smaller input), short and long contexts
    big = [1700, 40, 1537, 1601, 9, 1900, 333, 1650, 64, 1800, 1555, 31, 1999, 1777, 5, 1620]
    small = [1650, 7, 130]
    ref_big, sta_big = _context(cfg, st, big)
    ref_small, sta_small = _context(cfg, st, small)
    assert 0 < st.decode_static_bytes(len(big)) <= 64 << 20
    assert st.decode_static_bytes(len(small)) < st.decode_static_bytes(len(big))
    for step in range(2):
        xb = to_dev(generate.hidden_rows(cfg, len(big), stream_id=1 + step), cfg)
        xs = to_dev(generate.hidden_rows(cfg, len(small), stream_id=5 + step), cfg)
        want = []
        for kv, x in ((ref_big, xb), (ref_small, xs)):
            p, h = torch.empty_like(x), torch.empty_like(x)
            st.decode(kv, step, x, p, h)
            want.append((p, h))
        got = []
        for kv, x in ((sta_big, xb), (sta_small, xs)):           # two calls in a row, the second one smaller
            p, h = torch.full_like(x, float("nan")), torch.full_like(x, float("nan"))
            st.decode_static(kv, step, x, p, h)
            got.append((p, h))
        torch.cuda.synchronize()
        for (p, h), (pr, hr), name in zip(got, want, ("16 rows", "3 rows")):
            assert torch.isfinite(p.float()).all() and torch.isfinite(h.float()).all(), f"step {step}, {name}"
            assert torch.equal(p, pr), f"step {step}, {name}: out_partial differs"
            assert torch.equal(h, hr), f"step {step}, {name}: out_resid differs"
    # the rows each entry point appended are the same, and both caches advanced alike
    assert sta_big.get_lengths(len(big)) == ref_big.get_lengths(len(big)) == [n + 2 for n in big]
    assert sta_small.get_lengths(len(small)) == ref_small.get_lengths(len(small)) == [n + 2 for n in small]
    for ref, sta, lens in ((ref_big, sta_big, big), (ref_small, sta_small, small)):
        for l in range(cfg.n_layers):
            for s in (0, len(lens) - 1):
                k0, v0 = ref.read(l, s, lens[s], 2)
                k1, v1 = sta.read(l, s, lens[s], 2)
                assert torch.equal(k0, k1) and torch.equal(v0, v1)
    # the two entry points can be mixed step by step on one cache
    x = to_dev(generate.hidden_rows(cfg, len(small), stream_id=9), cfg)
    p0, h0, p1, h1 = (torch.empty_like(x) for _ in range(4))
    st.decode_static(ref_small, 2, x, p0, h0)
    st.decode(sta_small, 2, x, p1, h1)
    torch.cuda.synchronize()
    assert torch.equal(p0, p1) and torch.equal(h0, h1)


def test_static_scratch_decode_rejects_what_it_cannot_hold():
    import paper_2311_11514_amd as hx
    cfg = CFG
    w = [generate.layer_weights(cfg, l) for l in range(cfg.n_layers)]
    st = make_gpu_stage(cfg, cfg.tp_ranks[0], w)
    kv = st.kv_cache_create(40, 16)
    kv.set_lengths([4] * 33)                       # 33 sequences: beyond the weight-streaming decode kernels
    x = to_dev(generate.hidden_rows(cfg, 33), cfg)
    with pytest.raises(hx.HexgenError) as e:
        st.decode_static(kv, 0, x, torch.empty_like(x), torch.empty_like(x))
    assert e.value.status == 4                     # HEXGEN_ERR_CAPACITY
    assert kv.get_lengths(33) == [4] * 33          # untouched
    kv2 = st.kv_cache_create(2, 16)
    with pytest.raises(hx.HexgenError) as e:       # not prefilled
        st.decode_static(kv2, 0, x[:2], torch.empty_like(x[:2]), torch.empty_like(x[:2]))
    assert e.value.status == 3
    assert st.decode_static_bytes(0) == -1
