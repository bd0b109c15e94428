"""CPU oracle for one GPU's share of a pipeline stage -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this module;
the product path never does.  It shares no code with the GPU library.

What it computes (float64 throughout, plain numpy, no blocking / fusion / caching tricks):
the forward pass of `n_layers` consecutive decoder layers, sharded Megatron-style at
tensor-parallel degree t, rank r (paper Section 2, "Parallelism in generative inference":
weights split column-wise then row-wise, two all-reduce points per layer), run as prefill and
then token-by-token decode against a KV cache (paper Section 2, prefill / decode equations:
K and V of earlier positions are kept, the new token's K, V are concatenated, and the same
attention + FFN formulas are evaluated for the new row).  The stage returns its
pre-all-reduce partial of the last layer plus the residual stream that partial is to be added to.

The paper's equations are a simplified transformer (multi-head attention, ReLU FFN, no
normalisation).  The model it actually serves is Llama-2 (70B) (Section 5.1), so the layer
here is that model's layer.  Readings taken where the paper is silent:
  * pre-norm RMSNorm before attention and before the FFN, eps inside the square root, gain
    applied after normalising;
  * softmax scale 1/sqrt(head_dim) (the paper's 1/sqrt(H) is single-head notation);
  * causal mask inside each sequence, no attention across sequences of a batch;
  * grouped-query attention: query head j reads KV head j // G, G = n_heads / n_kv_heads;
    rank r owns query heads [r*hq_l, (r+1)*hq_l) and KV heads [r*hkv_l, (r+1)*hkv_l);
  * rotary embedding in the rotate-half pairing (element i pairs with i + d/2), angle
    p * theta^(-2i/d), applied to q and k (not v); k is cached after rotation;
  * FFN is SwiGLU: silu(n W1) * (n W3), then W2;
  * the residual stream is replicated across ranks and never part of a partial;
  * reduce points on one device: "solo" adds the rank's own partial to the residual (what a
    single rank can compute alone), "group" adds the sum over all ranks (the all-reduce).
Weights use the paper's x . W convention: W is [in, out].

Pins (tests/test_oracle_pins.py): shard-sum == unsharded, decode == prefill row, causality,
brute-force dense attention without cache on the tiny stage, torch library routines for
attention / RMSNorm / SiLU / linear, RoPE closed forms.  Solo-mode semantics for t > 1 are
this build's own definition (no second device): parity unpinned by the paper; pinned only by
construction (solo(t, r) equals an unsharded stage whose weights are rank r's shard).
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

F64 = np.float64


def _f64(x) -> np.ndarray:
    if hasattr(x, "detach"):            # torch tensor
        x = x.detach().cpu().numpy()
    return np.asarray(x, dtype=F64)


def rmsnorm(h: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """n_c = h_c / sqrt(mean_c(h^2) + eps) * g_c, row by row."""
    ms = np.mean(h * h, axis=-1, keepdims=True)
    return h / np.sqrt(ms + eps) * g


def rope_cos_sin(pos: np.ndarray, d: int, theta: float) -> Tuple[np.ndarray, np.ndarray]:
    """cos, sin of the angle p * theta^(-2i/d), shape [len(pos), d/2]."""
    i = np.arange(d // 2, dtype=F64)
    inv_freq = theta ** (-2.0 * i / d)
    ang = np.asarray(pos, dtype=F64)[:, None] * inv_freq[None, :]
    return np.cos(ang), np.sin(ang)


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotate every head of x [n, heads, d] by its row's absolute position (rotate-half)."""
    d = x.shape[-1]
    c, s = rope_cos_sin(pos, d, theta)
    c, s = c[:, None, :], s[:, None, :]
    lo, hi = x[..., : d // 2], x[..., d // 2:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def silu(a: np.ndarray) -> np.ndarray:
    return a / (1.0 + np.exp(-a))


def softmax(s: np.ndarray) -> np.ndarray:
    e = np.exp(s - np.max(s))
    return e / np.sum(e)


class KVCache:
    """Per layer, per sequence: K and V rows [len, hkv_l, d] (K stored after rotation)."""

    def __init__(self, n_layers: int, batch: int, hkv_l: int, d: int):
        self.k = [[np.zeros((0, hkv_l, d), F64) for _ in range(batch)] for _ in range(n_layers)]
        self.v = [[np.zeros((0, hkv_l, d), F64) for _ in range(batch)] for _ in range(n_layers)]
        self.batch = batch

    def length(self, layer: int, seq: int) -> int:
        return self.k[layer][seq].shape[0]

    def append(self, layer: int, seq: int, k: np.ndarray, v: np.ndarray) -> None:
        self.k[layer][seq] = np.concatenate([self.k[layer][seq], k], axis=0)
        self.v[layer][seq] = np.concatenate([self.v[layer][seq], v], axis=0)

    def fill(self, layer: int, seq: int, k, v) -> None:
        """Install a synthetic context (replaces whatever the sequence held in that layer)."""
        self.k[layer][seq] = _f64(k).copy()
        self.v[layer][seq] = _f64(v).copy()


class OracleStage:
    def __init__(self, hidden: int, n_heads: int, n_kv_heads: int, ffn: int, n_layers: int,
                 tp_degree: int, tp_rank: int, rms_eps: float = 1e-5, rope_theta: float = 10000.0):
        assert hidden % n_heads == 0 and n_heads % n_kv_heads == 0
        assert n_heads % tp_degree == 0 and n_kv_heads % tp_degree == 0 and ffn % tp_degree == 0
        assert 0 <= tp_rank < tp_degree
        self.H, self.hq, self.hkv, self.F, self.L = hidden, n_heads, n_kv_heads, ffn, n_layers
        self.t, self.r = tp_degree, tp_rank
        self.d = hidden // n_heads
        self.hq_l, self.hkv_l, self.F_l = n_heads // tp_degree, n_kv_heads // tp_degree, ffn // tp_degree
        self.G = n_heads // n_kv_heads
        self.eps, self.theta = rms_eps, rope_theta
        self.layers: List[dict] = [None] * n_layers

    # ---- weights --------------------------------------------------------------------
    def load_layer(self, layer: int, g_attn, wq, wk, wv, wo, g_ffn, w1, w3, w2) -> None:
        """Takes GLOBAL [in, out] matrices and keeps rank r's shard: columns of W_Q/W_K/W_V/
        W1/W3 (column-parallel), rows of W_O/W2 (row-parallel)."""
        d, r = self.d, self.r
        qs = slice(r * self.hq_l * d, (r + 1) * self.hq_l * d)
        ks = slice(r * self.hkv_l * d, (r + 1) * self.hkv_l * d)
        fs = slice(r * self.F_l, (r + 1) * self.F_l)

        def cut(w, rows=slice(None), cols=slice(None)):
            if hasattr(w, "detach"):
                w = w.detach()[rows, cols].cpu().numpy()
            else:
                w = np.asarray(w)[rows, cols]
            return np.ascontiguousarray(w, dtype=F64)

        self.layers[layer] = dict(
            g_attn=_f64(g_attn), g_ffn=_f64(g_ffn),
            wq=cut(wq, cols=qs), wk=cut(wk, cols=ks), wv=cut(wv, cols=ks), wo=cut(wo, rows=qs),
            w1=cut(w1, cols=fs), w3=cut(w3, cols=fs), w2=cut(w2, rows=fs))

    def new_cache(self, batch: int) -> KVCache:
        return KVCache(self.L, batch, self.hkv_l, self.d)

    # ---- the two sub-layers; each returns this rank's pre-all-reduce partial ----------
    def attn_partial(self, layer: int, cache: KVCache, h: np.ndarray, seq_of_row: Sequence[int]) -> np.ndarray:
        """h [T,H]: rows of one call; row i belongs to sequence seq_of_row[i]; the rows of one
        sequence are consecutive positions starting at that sequence's current cache length."""
        W = self.layers[layer]
        T = h.shape[0]
        n = rmsnorm(h, W["g_attn"], self.eps)
        q = (n @ W["wq"]).reshape(T, self.hq_l, self.d)
        k = (n @ W["wk"]).reshape(T, self.hkv_l, self.d)
        v = (n @ W["wv"]).reshape(T, self.hkv_l, self.d)
        # absolute position of every row
        pos = np.zeros(T, dtype=np.int64)
        nxt = {}
        for i, s in enumerate(seq_of_row):
            p = nxt.get(s, cache.length(layer, s))
            pos[i] = p
            nxt[s] = p + 1
        q = rope(q, pos, self.theta)
        k = rope(k, pos, self.theta)
        for s in sorted(nxt):
            rows = [i for i, ss in enumerate(seq_of_row) if ss == s]
            cache.append(layer, s, k[rows], v[rows])          # the "Concat" of the decode equations
        o = np.zeros((T, self.hq_l, self.d), F64)
        scale = 1.0 / np.sqrt(float(self.d))
        for i, s in enumerate(seq_of_row):
            K = cache.k[layer][s][: pos[i] + 1]               # causal: positions 0..p only
            V = cache.v[layer][s][: pos[i] + 1]
            for j in range(self.hq_l):
                c = j // self.G
                w = softmax((K[:, c, :] @ q[i, j]) * scale)
                o[i, j] = w @ V[:, c, :]
        return o.reshape(T, self.hq_l * self.d) @ W["wo"]

    def ffn_partial(self, layer: int, h: np.ndarray) -> np.ndarray:
        W = self.layers[layer]
        n = rmsnorm(h, W["g_ffn"], self.eps)
        u = silu(n @ W["w1"]) * (n @ W["w3"])
        return u @ W["w2"]

    # ---- one layer, chosen output rows only (full-size workloads) ------------------------------------
    def layer_rows(self, layer: int, h_seq, rows: Sequence[int], split_ffn: bool = False):
        """Solo-mode output of `layer` for ONE sequence given the residual stream h_seq [S,H] entering the
        layer (positions 0..S-1), evaluated only at the positions in `rows`.  Same definition as
        attn_partial / ffn_partial: K and V are formed for every position (they are needed by later rows),
        the query, attention, W_O, residual and FFN only for the chosen rows.  Returns (h_out [len(rows),H]
        = residual stream after the layer, K [S,hkv_l,d] after rotation, V [S,hkv_l,d]); with split_ffn the
        first element is the pair (h_mid, P_ffn) a stage returns for its last layer instead of their sum."""
        W = self.layers[layer]
        h = _f64(h_seq)
        S = h.shape[0]
        n = rmsnorm(h, W["g_attn"], self.eps)
        pos = np.arange(S)
        K = rope((n @ W["wk"]).reshape(S, self.hkv_l, self.d), pos, self.theta)
        V = (n @ W["wv"]).reshape(S, self.hkv_l, self.d)
        rows = list(rows)
        q = rope((n[rows] @ W["wq"]).reshape(len(rows), self.hq_l, self.d), np.asarray(rows), self.theta)
        o = np.zeros((len(rows), self.hq_l, self.d), F64)
        scale = 1.0 / np.sqrt(float(self.d))
        for a, i in enumerate(rows):
            for j in range(self.hq_l):
                c = j // self.G
                w = softmax((K[: i + 1, c, :] @ q[a, j]) * scale)
                o[a, j] = w @ V[: i + 1, c, :]
        h_mid = h[rows] + o.reshape(len(rows), self.hq_l * self.d) @ W["wo"]
        p = self.ffn_partial(layer, h_mid)
        return ((h_mid, p) if split_ffn else h_mid + p), K, V

    # ---- solo mode: this rank alone ---------------------------------------------------
    def forward(self, cache: KVCache, hidden_in, seq_of_row: Sequence[int], taps: dict = None):
        """Returns (out_partial, out_resid): last layer's FFN partial (no residual inside) and the
        residual stream it would be added to.  `taps`, if a dict, receives the residual stream
        entering each layer (key = layer index)."""
        h = _f64(hidden_in).copy()
        for layer in range(self.L):
            if taps is not None:
                taps[layer] = h.copy()
            h = h + self.attn_partial(layer, cache, h, seq_of_row)
            p = self.ffn_partial(layer, h)
            if layer == self.L - 1:
                return p, h
            h = h + p

    def prefill(self, cache: KVCache, hidden_in, seq_lens: Sequence[int], taps: dict = None):
        seq_of_row = [s for s, n in enumerate(seq_lens) for _ in range(n)]
        return self.forward(cache, hidden_in, seq_of_row, taps)

    def decode(self, cache: KVCache, hidden_in, taps: dict = None):
        return self.forward(cache, hidden_in, list(range(cache.batch)), taps)


def group_forward(stages: Sequence[OracleStage], caches: Sequence[KVCache], hidden_in,
                  seq_of_row: Sequence[int]):
    """All t ranks of one stage with the all-reduce performed: at each reduce point the partials
    are summed in rank order.  Returns ([out_partial_r for r], out_resid)."""
    h = _f64(hidden_in).copy()
    L = stages[0].L
    for layer in range(L):
        h = h + sum(st.attn_partial(layer, c, h, seq_of_row) for st, c in zip(stages, caches))
        parts = [st.ffn_partial(layer, h) for st in stages]
        if layer == L - 1:
            return parts, h
        h = h + sum(parts)


def greedy_head(x_last: np.ndarray, g_final, w_lm, eps: float) -> Tuple[int, np.ndarray]:
    """Final RMSNorm + untied LM head on one hidden row; argmax, lowest index wins ties."""
    logits = rmsnorm(_f64(x_last)[None, :], _f64(g_final), eps)[0] @ _f64(w_lm)
    return int(np.argmax(logits)), logits


# ---- the model's two ends, adjacent to the first and the last stage (Section 2: the prompt enters as tokens and
# the output leaves as tokens, one per step) ------------------------------------------------------------------
def embed_rows(table, tokens) -> np.ndarray:
    """First stage: row `tokens[i]` of the embedding table [vocab, H] for every input token."""
    return _f64(table)[np.asarray(tokens, dtype=np.int64)]


def head_shard_greedy(x: np.ndarray, g_final, w_lm, eps: float, t: int, r: int) -> Tuple[np.ndarray, np.ndarray]:
    """Last stage, vocabulary-parallel over t ranks: rank r holds columns [r V/t, (r+1) V/t) of the LM head.
    For every row of x [rows, H]: final RMSNorm, the rank's logits, and the rank's best candidate as
    (GLOBAL token id, its logit); the lowest id wins ties."""
    w = _f64(w_lm)
    V = w.shape[1]
    assert V % t == 0
    lo = r * (V // t)
    logits = rmsnorm(_f64(x), _f64(g_final), eps) @ w[:, lo:lo + V // t]
    idx = np.argmax(logits, axis=1)
    return (idx + lo).astype(np.int64), logits[np.arange(logits.shape[0]), idx]


def merge_greedy(candidates) -> np.ndarray:
    """The group's choice from the ranks' (ids, logits) candidates, in rank order: largest logit, and since a
    lower rank holds lower ids, the first maximum keeps the lowest-id tie rule."""
    ids = np.stack([c[0] for c in candidates])          # [t, rows]
    val = np.stack([c[1] for c in candidates])
    best = np.argmax(val, axis=0)
    return ids[best, np.arange(ids.shape[1])]
