"""GPU parity on seeded random shapes: stage geometry (head_dim 64 / 128, GQA group 1..16, TP degree and rank, ragged FFN
widths), storage type (bf16 / fp16) and row structure (a few short prompts, prompts around the 128-row block size,
many one- to five-row sequences, batches above 32 that leave the weight-streaming decode kernels) are drawn from one
fixed seed, every draw a valid configuration by construction.  Each case runs a ragged prefill and three decode steps
against the float64 oracle and checks the rows, and the cache rows of one sequence.  The cases are generated at import
time, so a failure names its case and the parameters are printed before anything is launched."""
import numpy as np
import pytest

from tests.helpers import TOL, check, gpu_decode, gpu_prefill, make_gpu_stage, make_oracle
from workloads import StageConfig, generate

pytestmark = pytest.mark.gpu


def _cases(n=28, seed=2311):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        d = int(rng.choice([64, 128]))
        tp = int(rng.choice([1, 2, 4]))
        hkv = tp * int(rng.choice([1, 2]))
        G = int(rng.choice([1, 2, 4, 8, 16]))
        hq = hkv * G
        hidden = hq * d
        if hidden % 128 or hidden > 2048 or hidden < 256 or (hq // tp) * d % 32:
            continue
        F_l = 32 * int(rng.integers(8, 100))
        layers = int(rng.choice([1, 2]))
        rank = int(rng.integers(0, tp))
        dtype = "f16" if len(out) % 3 == 2 else "bf16"
        mode = ["short", "blocky", "many", "wide"][len(out) % 4]
        if mode == "short":
            lens = [int(rng.integers(1, 60)) for _ in range(int(rng.integers(1, 5)))]
        elif mode == "blocky":
            lens = [int(rng.choice([127, 128, 129, 255, 256, 257, 1, 2])) for _ in range(int(rng.integers(2, 6)))]
        elif mode == "many":
            lens = [int(rng.integers(1, 6)) for _ in range(int(rng.integers(20, 33)))]
        else:
            lens = [int(rng.integers(1, 4)) for _ in range(int(rng.integers(33, 44)))]
        out.append((len(out), dtype, d, tp, rank, hq, hkv, hidden, F_l * tp, layers, lens))
    return out


CASES = _cases()


@pytest.mark.parametrize("case", CASES, ids=[f"case{c[0]}-{c[1]}" for c in CASES])
def test_random_stage_prefill_then_decode(case):
    idx, dtype, d, tp, rank, hq, hkv, hidden, ffn, layers, lens = case
    print(f"case {idx}: {dtype} d={d} tp={tp} rank={rank} hq={hq} hkv={hkv} H={hidden} F={ffn} layers={layers} "
          f"batch={len(lens)} rows={sum(lens)} lens={lens[:8]}{'...' if len(lens) > 8 else ''}", flush=True)
    cfg = StageConfig(f"rnd{idx}", dtype, hidden, hq, hkv, ffn, layers, tp, (rank,), batch=len(lens), seed=500 + idx)
    assert cfg.head_dim == d
    tol = TOL[dtype]
    w = [generate.layer_weights(cfg, l) for l in range(layers)]
    X = generate.hidden_rows(cfg, sum(lens))
    ora = make_oracle(cfg, rank, w)
    oc = ora.new_cache(len(lens))
    p_ref, h_ref = ora.prefill(oc, X, lens)
    st = make_gpu_stage(cfg, rank, w)
    kv = st.kv_cache_create(len(lens), max(lens) + 8)
    p, h = gpu_prefill(st, kv, cfg, X, lens)
    check(f"case {idx} prefill resid", h, h_ref, tol)
    check(f"case {idx} prefill partial", p, p_ref, tol)
    assert kv.get_lengths(len(lens)) == lens
    for k in range(3):
        x = generate.hidden_rows(cfg, len(lens), stream_id=1 + k)
        p_ref, h_ref = ora.decode(oc, x)
        p, h = gpu_decode(st, kv, cfg, k, x)
        check(f"case {idx} decode {k} resid", h, h_ref, tol)
        check(f"case {idx} decode {k} partial", p, p_ref, tol)
    s = int(np.argmax(lens))
    for layer in range(layers):
        kk, vv = kv.read(layer, s, 0, lens[s] + 3)
        check(f"case {idx} K layer {layer}", kk.numpy().reshape(-1, d), oc.k[layer][s].reshape(-1, d), tol)
        check(f"case {idx} V layer {layer}", vv.numpy().reshape(-1, d), oc.v[layer][s].reshape(-1, d), tol)
