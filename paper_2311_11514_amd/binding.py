"""ctypes binding of libhexgen.so: argument marshalling only, same names as include/hexgen.h
(the paper's calls) and include/hexgen_bench.h (measurement-only entry points).

torch is used for device memory and streams; every step of the stage runs in the library's HIP
kernels.  There is no fallback: if the shared library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhexgen.so")

HEXGEN_F32, HEXGEN_BF16, HEXGEN_F16 = 0, 1, 2
_DTYPE_CODE = {"f32": HEXGEN_F32, "bf16": HEXGEN_BF16, "f16": HEXGEN_F16}
STATUS_NAMES = {0: "HEXGEN_OK", 1: "HEXGEN_ERR_INVALID_ARG", 2: "HEXGEN_ERR_SHAPE", 3: "HEXGEN_ERR_STATE",
                4: "HEXGEN_ERR_CAPACITY", 5: "HEXGEN_ERR_OOM", 6: "HEXGEN_ERR_DEVICE"}

# every symbol include/*.h declares: name -> (restype, argtypes)
_vp, _i, _i64, _f = C.c_void_p, C.c_int, C.c_int64, C.c_float
_ip = C.POINTER(C.c_int32)
_fp = C.POINTER(C.c_float)
SIGNATURES = {
    "hexgen_status_string": (C.c_char_p, [_i]),
    "hexgen_stage_create": (_i, [_i, _i, _i, _i, _i, _i, _i, _i, C.POINTER(_vp)]),
    "hexgen_stage_set_params": (_i, [_vp, _f, _f]),
    "hexgen_stage_destroy": (None, [_vp]),
    "hexgen_stage_load_layer": (_i, [_vp, _i] + [_vp] * 9),
    "hexgen_kv_cache_create": (_i, [_vp, _i, _i, C.POINTER(_vp)]),
    "hexgen_kv_cache_destroy": (None, [_vp]),
    "hexgen_kv_cache_reset": (_i, [_vp]),
    "hexgen_stage_prefill": (_i, [_vp, _vp, _vp, _ip, _i, _vp, _vp, _vp]),
    "hexgen_stage_decode": (_i, [_vp, _vp, _i, _vp, _vp, _vp, _vp]),
    "hexgen_stage_decode_static": (_i, [_vp, _vp, _i, _vp, _vp, _vp, _vp]),
    "hexgen_stage_decode_static_bytes": (_i64, [_vp, _i]),
    "hexgen_stage_run_sublayer": (_i, [_vp, _vp, _i, _i, _vp, _ip, _i, _vp, _vp]),
    "hexgen_kv_cache_commit": (_i, [_vp, _ip, _i]),
    "hexgen_accumulate_f32": (_i, [_vp, _vp, _i64, _vp]),
    "hexgen_kv_cache_read": (_i, [_vp, _i, _i, _i, _i, _fp, _fp]),
    "hexgen_kv_cache_fill": (_i, [_vp, _i, _i, _i, _fp, _fp]),
    "hexgen_kv_cache_set_lengths": (_i, [_vp, _ip, _i]),
    "hexgen_kv_cache_get_lengths": (_i, [_vp, _ip, _i]),
    "hexgen_stage_set_tap": (_i, [_vp, _i, _vp]),
    "hexgen_stage_weight_bytes": (_i64, [_vp]),
    "hexgen_stream_copy": (_i, [_vp, _vp, _i64, _i, _vp]),
    "hexgen_stream_read": (_i, [_vp, _vp, _i64, _i, _vp]),
    "hexgen_mfma_probe": (_i, [_i, _vp, _i, _i, _vp]),
    "hexgen_set_gemm_tile": (_i, [_i]),
    "hexgen_set_attn_split": (_i, [_i]),
    "hexgen_embed_rows": (_i, [_vp, _i, _i, _i, _vp, _i, _vp, _vp]),
    "hexgen_head_create": (_i, [_i, _i, _i, _i, _i, C.c_float, C.POINTER(_vp)]),
    "hexgen_head_load": (_i, [_vp, _vp, _vp]),
    "hexgen_head_greedy": (_i, [_vp, _vp, _vp, _i, _vp, _vp, _vp]),
    "hexgen_head_destroy": (None, [_vp]),
    "hexgen_cost_comp": (C.c_double, [_i, C.c_double, _i, _i, _i, _i, _i, _i, _vp, _vp]),
    "hexgen_cost_comp_prefill": (C.c_double, [_i, C.c_double, _i, _i, _i, _i, _i, _i, _vp, _vp]),
    "hexgen_cost_comp_decode": (C.c_double, [_i, C.c_double, _i, _i, _i, _i, _i, _i, _vp, _vp]),
    "hexgen_cost_comm_tp": (C.c_double, [_i, _i, _i, _i, _i, _i, _i, _vp, _vp]),
    "hexgen_cost_comm_pp": (C.c_double, [_i, _i, _i, _i, _i, _i, _i, _vp, _vp]),
    "hexgen_cost_mem": (C.c_double, [_i, C.c_double, _i, _i, _i, _i, _i, _i]),
    "hexgen_sched_pipeline_layout": (C.c_double, [_vp, _vp, _i, _vp, _i, _vp, _vp]),
    "hexgen_sched_merge": (_i, [_i, _vp, _vp, _vp]),
    "hexgen_sched_split": (_i, [_i, _vp, _vp, _vp]),
    "hexgen_sched_swap": (_i, [_i, _vp, _vp, _i]),
    "hexgen_sched_repartition_layers": (_i, [_i, _i, _vp, _vp]),
    "hexgen_sched_group_can_hold": (_i, [_i, _vp, _vp, C.c_double]),
    "hexgen_slo_attainment": (C.c_double, [_i, _vp, _vp, _i, _i, _vp, _vp, _vp]),
    "hexgen_sched_draw": (C.c_ulonglong, [C.c_ulonglong, C.c_ulonglong]),
    "hexgen_sched_initial_groups": (_i, [_vp, _vp]),
    "hexgen_sched_plan_group": (C.c_double, [_vp, _vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp]),
    "hexgen_sched_search": (C.c_double, [_vp, _vp, _vp, _i, _vp, C.c_double, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "hexgen_stage_profile_enable": (_i, [_vp, _i]),
    "hexgen_stage_profile_read": (_i, [_vp, _i, C.POINTER(C.c_double), C.POINTER(_i64)]),
    "hexgen_stage_time_w13_decode": (_i, [_vp, _i, C.POINTER(C.c_double), C.POINTER(_i64), _vp]),
}


def load_library(path: str = LIB_PATH) -> C.CDLL:
    if not os.path.exists(path):
        raise ImportError(f"{path} not found: build it first (python -m paper_2311_11514_amd.build); "
                          "there is no fallback path")
    lib = C.CDLL(path)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


lib = load_library()


class HexgenError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.hexgen_status_string(status).decode()
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({msg})")


def _check(status: int, where: str) -> None:
    if status != 0:
        raise HexgenError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous()
    return t.data_ptr()


def _i32(seq: Optional[Sequence[int]]):
    if seq is None:
        return None
    return (C.c_int32 * len(seq))(*[int(v) for v in seq])


def _stream_handle(stream: Optional[torch.cuda.Stream]) -> Optional[int]:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream or None


def _torch_dtype(dtype: int):
    return {HEXGEN_F32: torch.float32, HEXGEN_BF16: torch.bfloat16, HEXGEN_F16: torch.float16}[dtype]


def _dtype_code(dtype) -> int:
    if isinstance(dtype, str):
        return _DTYPE_CODE[dtype]
    if isinstance(dtype, torch.dtype):
        return {torch.float32: HEXGEN_F32, torch.bfloat16: HEXGEN_BF16, torch.float16: HEXGEN_F16}[dtype]
    return int(dtype)


class Stage:
    """Owns a hexgen_stage_t.  dtype: "f32" | "bf16" | "f16"."""

    def __init__(self, hidden, n_heads, n_kv_heads, ffn, n_layers, tp_degree, tp_rank, dtype,
                 rms_eps: float = 1e-5, rope_theta: float = 10000.0):
        self.dtype = _DTYPE_CODE[dtype] if isinstance(dtype, str) else int(dtype)
        h = C.c_void_p()
        _check(lib.hexgen_stage_create(hidden, n_heads, n_kv_heads, ffn, n_layers, tp_degree, tp_rank,
                                       self.dtype, C.byref(h)), "hexgen_stage_create")
        self.handle = h
        self.hidden, self.n_layers = hidden, n_layers
        self.head_dim = hidden // n_heads
        self.hkv_l = n_kv_heads // tp_degree
        _check(lib.hexgen_stage_set_params(self.handle, rms_eps, rope_theta), "hexgen_stage_set_params")
        self._taps = {}

    def close(self, _lib=lib):
        # the default argument keeps the library reachable when the module's globals are already torn down
        if getattr(self, "handle", None):
            _lib.hexgen_stage_destroy(self.handle)
            self.handle = None

    __del__ = close

    def load_layer(self, layer: int, g_attn, wq, wk, wv, wo, g_ffn, w1, w3, w2):
        """Global [in, out] tensors (host or device); converted to the stage's dtype if needed."""
        td = _torch_dtype(self.dtype)
        ts = [t.to(td).contiguous() for t in (g_attn, wq, wk, wv, wo, g_ffn, w1, w3, w2)]
        _check(lib.hexgen_stage_load_layer(self.handle, layer, *[t.data_ptr() for t in ts]),
               "hexgen_stage_load_layer")

    def kv_cache_create(self, max_batch: int, max_seq: int) -> "KVCache":
        return KVCache(self, max_batch, max_seq)

    def prefill(self, kv: "KVCache", hidden_in: torch.Tensor, seq_lens: Sequence[int],
                out_partial: torch.Tensor, out_resid: Optional[torch.Tensor] = None, stream=None):
        _check(lib.hexgen_stage_prefill(self.handle, kv.handle, _ptr(hidden_in), _i32(seq_lens), len(seq_lens),
                                        _ptr(out_partial), _ptr(out_resid), _stream_handle(stream)),
               "hexgen_stage_prefill")

    def decode(self, kv: "KVCache", step: int, hidden_in: torch.Tensor, out_partial: torch.Tensor,
               out_resid: Optional[torch.Tensor] = None, stream=None):
        _check(lib.hexgen_stage_decode(self.handle, kv.handle, step, _ptr(hidden_in), _ptr(out_partial),
                                       _ptr(out_resid), _stream_handle(stream)), "hexgen_stage_decode")

    def decode_static(self, kv: "KVCache", step: int, hidden_in: torch.Tensor, out_partial: torch.Tensor,
                      out_resid: Optional[torch.Tensor] = None, stream=None):
        """hexgen_stage_decode_static: the decode step for callers that cannot allocate."""
        _check(lib.hexgen_stage_decode_static(self.handle, kv.handle, step, _ptr(hidden_in), _ptr(out_partial),
                                              _ptr(out_resid), _stream_handle(stream)), "hexgen_stage_decode_static")

    def decode_static_bytes(self, batch: int) -> int:
        return int(lib.hexgen_stage_decode_static_bytes(self.handle, batch))

    def run_sublayer(self, kv: "KVCache", layer: int, which: int, h_in: torch.Tensor,
                     seq_lens: Optional[Sequence[int]], batch: int, partial_out: torch.Tensor, stream=None):
        _check(lib.hexgen_stage_run_sublayer(self.handle, kv.handle, layer, which, _ptr(h_in), _i32(seq_lens),
                                             batch, _ptr(partial_out), _stream_handle(stream)),
               "hexgen_stage_run_sublayer")

    def set_tap(self, layer: int, h_dump: Optional[torch.Tensor]):
        self._taps[layer] = h_dump          # keep the buffer alive
        _check(lib.hexgen_stage_set_tap(self.handle, layer, _ptr(h_dump)), "hexgen_stage_set_tap")

    def profile_enable(self, slot_mask):
        """slot_mask: bit i times slot i (True = all seven slots, False / 0 = off)."""
        mask = 127 if slot_mask is True else int(slot_mask)
        _check(lib.hexgen_stage_profile_enable(self.handle, mask), "hexgen_stage_profile_enable")

    def profile_read(self, slot: int):
        """(total milliseconds, number of timed launches) of a slot; see include/hexgen_bench.h."""
        ms, n = C.c_double(), C.c_int64()
        _check(lib.hexgen_stage_profile_read(self.handle, slot, C.byref(ms), C.byref(n)),
               "hexgen_stage_profile_read")
        return ms.value, n.value

    def time_w13_decode(self, reps: int, stream=None):
        """(total milliseconds, launches) of the W1/W3 decode projection of every layer, back to back, reps times."""
        ms, n = C.c_double(), C.c_int64()
        _check(lib.hexgen_stage_time_w13_decode(self.handle, reps, C.byref(ms), C.byref(n), _stream_handle(stream)),
               "hexgen_stage_time_w13_decode")
        return ms.value, n.value

    def weight_bytes(self) -> int:
        return int(lib.hexgen_stage_weight_bytes(self.handle))


class KVCache:
    def __init__(self, stage: Stage, max_batch: int, max_seq: int):
        h = C.c_void_p()
        _check(lib.hexgen_kv_cache_create(stage.handle, max_batch, max_seq, C.byref(h)), "hexgen_kv_cache_create")
        self.handle, self.stage = h, stage

    def close(self, _lib=lib):
        if getattr(self, "handle", None):
            _lib.hexgen_kv_cache_destroy(self.handle)
            self.handle = None

    __del__ = close

    def reset(self):
        _check(lib.hexgen_kv_cache_reset(self.handle), "hexgen_kv_cache_reset")

    def commit(self, seq_lens: Optional[Sequence[int]], batch: int):
        _check(lib.hexgen_kv_cache_commit(self.handle, _i32(seq_lens), batch), "hexgen_kv_cache_commit")

    def set_lengths(self, lens: Sequence[int]):
        _check(lib.hexgen_kv_cache_set_lengths(self.handle, _i32(lens), len(lens)), "hexgen_kv_cache_set_lengths")

    def get_lengths(self, batch: int):
        out = (C.c_int32 * batch)()
        _check(lib.hexgen_kv_cache_get_lengths(self.handle, out, batch), "hexgen_kv_cache_get_lengths")
        return list(out)

    def fill(self, layer: int, seq: int, k: torch.Tensor, v: torch.Tensor):
        """k, v: host fp32 [n, hkv_local, head_dim]."""
        k = k.to(torch.float32).contiguous().cpu()
        v = v.to(torch.float32).contiguous().cpu()
        _check(lib.hexgen_kv_cache_fill(self.handle, layer, seq, k.shape[0],
                                        C.cast(k.data_ptr(), _fp), C.cast(v.data_ptr(), _fp)), "hexgen_kv_cache_fill")

    def read(self, layer: int, seq: int, pos0: int, n: int):
        st = self.stage
        k = torch.empty(n, st.hkv_l, st.head_dim, dtype=torch.float32)
        v = torch.empty_like(k)
        _check(lib.hexgen_kv_cache_read(self.handle, layer, seq, pos0, n, C.cast(k.data_ptr(), _fp),
                                        C.cast(v.data_ptr(), _fp)), "hexgen_kv_cache_read")
        return k, v


def stream_copy(dst: torch.Tensor, src: torch.Tensor, blocks: int = 4096, stream=None):
    nbytes = src.numel() * src.element_size()
    _check(lib.hexgen_stream_copy(_ptr(dst), _ptr(src), nbytes, blocks, _stream_handle(stream)), "hexgen_stream_copy")


def stream_read(src: torch.Tensor, sink: torch.Tensor, blocks: int = 4096, stream=None):
    nbytes = src.numel() * src.element_size()
    _check(lib.hexgen_stream_read(_ptr(src), _ptr(sink), nbytes, blocks, _stream_handle(stream)), "hexgen_stream_read")


class Head:
    """Final RMSNorm + vocabulary-parallel LM head + greedy arg-max of one rank (hexgen_head_*)."""

    def __init__(self, hidden: int, vocab: int, tp_degree: int, tp_rank: int, dtype, rms_eps: float = 1e-5):
        self.dtype = _dtype_code(dtype)
        h = C.c_void_p()
        _check(lib.hexgen_head_create(hidden, vocab, tp_degree, tp_rank, self.dtype, rms_eps, C.byref(h)),
               "hexgen_head_create")
        self.handle, self.hidden, self.vocab = h, hidden, vocab

    def close(self, _lib=lib):
        if getattr(self, "handle", None):
            _lib.hexgen_head_destroy(self.handle)
            self.handle = None

    __del__ = close

    def load(self, g_final: torch.Tensor, w_lm: torch.Tensor):
        td = _torch_dtype(self.dtype)
        g, w = g_final.to(td).contiguous(), w_lm.to(td).contiguous()
        assert tuple(w.shape) == (self.hidden, self.vocab) and g.numel() == self.hidden
        _check(lib.hexgen_head_load(self.handle, _ptr(g), _ptr(w)), "hexgen_head_load")

    def greedy(self, hidden_a: torch.Tensor, hidden_b: Optional[torch.Tensor] = None, stream=None):
        """Returns (token ids int32 [n], logits float32 [n]) of this rank's candidates, on the device."""
        n = hidden_a.shape[0]
        tok = torch.empty(n, dtype=torch.int32, device=hidden_a.device)
        val = torch.empty(n, dtype=torch.float32, device=hidden_a.device)
        _check(lib.hexgen_head_greedy(self.handle, _ptr(hidden_a), _ptr(hidden_b) if hidden_b is not None else None, n,
                                      _ptr(tok), _ptr(val), _stream_handle(stream)), "hexgen_head_greedy")
        return tok, val


def embed_rows(table: torch.Tensor, tokens: torch.Tensor, stream=None) -> torch.Tensor:
    """rows[i] = table[tokens[i]] on the device (hexgen_embed_rows); tokens int32."""
    assert table.is_contiguous() and tokens.dtype == torch.int32
    out = torch.empty((tokens.numel(), table.shape[1]), dtype=table.dtype, device=table.device)
    _check(lib.hexgen_embed_rows(_ptr(table), _dtype_code(table.dtype), table.shape[1], table.shape[0], _ptr(tokens),
                                 tokens.numel(), _ptr(out), _stream_handle(stream)), "hexgen_embed_rows")
    return out


def _darr(values):
    flat = [float(v) for row in values for v in (row if isinstance(row, (list, tuple)) else [row])]
    return (C.c_double * len(flat))(*flat)


def cost_comp(hidden, bytes_per_elem, batch, s_in, s_out, layers, m_d, c_d, params_factor=12.0, phase="both") -> float:
    """Eq. 3 of the paper's cost model (hexgen_cost_comp*); phase = "both" | "prefill" | "decode"."""
    fn = {"both": lib.hexgen_cost_comp, "prefill": lib.hexgen_cost_comp_prefill, "decode": lib.hexgen_cost_comp_decode}[phase]
    return fn(hidden, params_factor, bytes_per_elem, batch, s_in, s_out, layers, len(m_d), _darr(m_d), _darr(c_d))


def cost_comm_tp(hidden, bytes_per_elem, batch, s_in, s_out, layers, alpha, beta) -> float:
    return lib.hexgen_cost_comm_tp(hidden, bytes_per_elem, batch, s_in, s_out, layers, len(alpha), _darr(alpha), _darr(beta))


def cost_comm_pp(hidden, bytes_per_elem, batch, s_in, s_out, alpha, beta) -> float:
    return lib.hexgen_cost_comm_pp(hidden, bytes_per_elem, batch, s_in, s_out, len(alpha), len(alpha[0]), _darr(alpha), _darr(beta))


def cost_mem(hidden, bytes_per_elem, batch, s_in, s_out, layers, n_dev, params_factor=12.0) -> float:
    return lib.hexgen_cost_mem(hidden, params_factor, bytes_per_elem, batch, s_in, s_out, layers, n_dev)


class _Pool(C.Structure):
    _fields_ = [("n_types", C.c_int), ("count", C.POINTER(C.c_int)), ("m_d", C.POINTER(C.c_double)),
                ("c_d", C.POINTER(C.c_double)), ("mem_bytes", C.POINTER(C.c_double)), ("tp_alpha", C.POINTER(C.c_double)),
                ("tp_beta", C.POINTER(C.c_double)), ("pp_alpha", C.POINTER(C.c_double)), ("pp_beta", C.POINTER(C.c_double))]


class _Task(C.Structure):
    _fields_ = [("hidden", C.c_int), ("params_factor", C.c_double), ("bytes_per_elem", C.c_int), ("batch", C.c_int),
                ("s_in", C.c_int), ("s_out", C.c_int)]


def _iarr(values):
    return (C.c_int * len(values))(*[int(v) for v in values])


def sched_pipeline_layout(pool: dict, task, layers, pow2_degrees_only: bool = False):
    """Algorithm 1 (hexgen_sched_pipeline_layout).  pool: dict with count, m, c, mem, tp_alpha, tp_beta (per type) and
    pp_alpha, pp_beta (type x type); task = (hidden, params_factor, bytes_per_elem, batch, s_in, s_out).
    Returns (cost seconds, [(type, degree) per stage])."""
    nt = len(pool["count"])
    keep = [_iarr(pool["count"]), _darr(pool["m"]), _darr(pool["c"]), _darr(pool["mem"]), _darr(pool["tp_alpha"]),
            _darr(pool["tp_beta"]), _darr(pool["pp_alpha"]), _darr(pool["pp_beta"])]
    p = _Pool(nt, keep[0], keep[1], keep[2], keep[3], keep[4], keep[5], keep[6], keep[7])
    t = _Task(int(task[0]), float(task[1]), int(task[2]), int(task[3]), int(task[4]), int(task[5]))
    ls = _iarr(layers)
    st, sc = (C.c_int * len(layers))(), (C.c_int * len(layers))()
    cost = lib.hexgen_sched_pipeline_layout(C.byref(p), C.byref(t), len(layers), ls, int(pow2_degrees_only), st, sc)
    return cost, [(st[j], sc[j]) for j in range(len(layers))]


class _Search(C.Structure):
    _fields_ = [("total_layers", C.c_int), ("model_bytes", C.c_double), ("max_stages", C.c_int),
                ("pow2_degrees_only", C.c_int), ("seed", C.c_ulonglong), ("n_iter", C.c_int), ("pop_size", C.c_int),
                ("max_group_states", C.c_long)]


def _pool_struct(pool: dict):
    keep = [_iarr(pool["count"]), _darr(pool["m"]), _darr(pool["c"]), _darr(pool["mem"]), _darr(pool["tp_alpha"]),
            _darr(pool["tp_beta"]), _darr(pool["pp_alpha"]), _darr(pool["pp_beta"])]
    return _Pool(len(pool["count"]), *keep), keep


def _task_struct(task):
    return _Task(int(task[0]), float(task[1]), int(task[2]), int(task[3]), int(task[4]), int(task[5]))


def slo_attainment(arrival, latency, deadline, cls=None, return_finish: bool = False):
    """hexgen_slo_attainment: latency[replica][class], deadline[class]; returns the share of requests served in time
    (and the finish times when asked)."""
    n, n_rep, n_cls = len(arrival), len(latency), len(deadline)
    fin = (C.c_double * max(n, 1))() if return_finish else None
    a = lib.hexgen_slo_attainment(n, _darr(arrival), None if cls is None else _iarr(cls), n_rep, n_cls,
                                  _darr([list(r) for r in latency]), _darr(deadline), fin)
    return (a, list(fin)[:n]) if return_finish else a


def sched_draw(seed: int, counter: int) -> int:
    return int(lib.hexgen_sched_draw(seed, counter))


def sched_initial_groups(pool: dict):
    """hexgen_sched_initial_groups: the K-means / elbow start of the search, a list of count vectors."""
    p, _keep = _pool_struct(pool)
    nt = len(pool["count"])
    out = (C.c_int * (nt * nt))()
    n = lib.hexgen_sched_initial_groups(C.byref(p), out)
    return [[out[g * nt + k] for k in range(nt)] for g in range(n)]


def sched_plan_group(pool: dict, task, tau, total_layers: int, max_stages: int, pow2_degrees_only: bool = False):
    """hexgen_sched_plan_group: (latency, layers per stage, [(type, degree) per stage]) of the group's best pipeline."""
    p, _keep = _pool_struct(pool)
    t = _task_struct(task)
    ns = C.c_int(0)
    lay, ty, cn = (C.c_int * max_stages)(), (C.c_int * max_stages)(), (C.c_int * max_stages)()
    cost = lib.hexgen_sched_plan_group(C.byref(p), C.byref(t), _iarr(tau), total_layers, max_stages, int(pow2_degrees_only),
                                       C.byref(ns), lay, ty, cn)
    return cost, [lay[j] for j in range(ns.value)], [(ty[j], cn[j]) for j in range(ns.value)]


def sched_search(pool: dict, task, total_layers: int, model_bytes: float, max_stages: int, arrival, deadline: float,
                 seed: int, n_iter: int, pop_size: int, pow2_degrees_only: bool = False, max_group_states: int = 1 << 14):
    """hexgen_sched_search: returns {"attainment", "groups": [{"tau", "latency", "layers", "stages"}], "history"}."""
    p, _keep = _pool_struct(pool)
    t = _task_struct(task)
    nt = len(pool["count"])
    cfg = _Search(total_layers, float(model_bytes), max_stages, int(pow2_degrees_only), seed, n_iter, pop_size,
                  max_group_states)
    max_groups = max(1, sum(pool["count"]))
    ng = C.c_int(0)
    tau = (C.c_int * (max_groups * nt))()
    lat = (C.c_double * max_groups)()
    gs = (C.c_int * max_groups)()
    lay, ty, cn = [(C.c_int * (max_groups * max_stages))() for _ in range(3)]
    hist = (C.c_double * max(n_iter, 1))()
    score = lib.hexgen_sched_search(C.byref(p), C.byref(t), C.byref(cfg), len(arrival), _darr(arrival), float(deadline),
                                    max_groups, C.byref(ng), tau, lat, gs, lay, ty, cn, hist)
    groups = []
    for g in range(ng.value):
        o = g * max_stages
        groups.append({"tau": [tau[g * nt + k] for k in range(nt)], "latency": lat[g],
                       "layers": [lay[o + j] for j in range(gs[g])],
                       "stages": [(ty[o + j], cn[o + j]) for j in range(gs[g])]})
    return {"attainment": score, "groups": groups, "history": list(hist)[:n_iter]}


def sched_merge(t1, t2):
    out = (C.c_int * len(t1))()
    assert lib.hexgen_sched_merge(len(t1), _iarr(t1), _iarr(t2), out)
    return list(out)


def sched_split(t):
    a, b = (C.c_int * len(t))(), (C.c_int * len(t))()
    assert lib.hexgen_sched_split(len(t), _iarr(t), a, b)
    return list(a), list(b)


def sched_swap(t1, t2, k):
    a, b = _iarr(t1), _iarr(t2)
    if not lib.hexgen_sched_swap(len(t1), a, b, k):
        raise ValueError("swap: the second group has no GPU of that type")
    return list(a), list(b)


def sched_group_can_hold(t, mem, model_bytes) -> bool:
    return bool(lib.hexgen_sched_group_can_hold(len(t), _iarr(t), _darr(mem), float(model_bytes)))


def sched_repartition_layers(total_layers, stage_mem):
    out = (C.c_int * len(stage_mem))()
    if not lib.hexgen_sched_repartition_layers(total_layers, len(stage_mem), _darr(stage_mem), out):
        raise ValueError("repartition_layers: invalid arguments")
    return list(out)


def set_gemm_tile(code: int):
    _check(lib.hexgen_set_gemm_tile(code), "hexgen_set_gemm_tile")


def set_attn_split(nsplit: int):
    _check(lib.hexgen_set_attn_split(nsplit), "hexgen_set_attn_split")


def mfma_probe(variant: int, sink: torch.Tensor, iters: int, blocks: int, stream=None):
    _check(lib.hexgen_mfma_probe(variant, _ptr(sink), iters, blocks, _stream_handle(stream)), "hexgen_mfma_probe")


def accumulate_f32(dst: torch.Tensor, src: torch.Tensor, stream=None):
    assert dst.dtype == torch.float32 and src.dtype == torch.float32 and dst.numel() == src.numel()
    _check(lib.hexgen_accumulate_f32(_ptr(dst), _ptr(src), dst.numel(), _stream_handle(stream)),
           "hexgen_accumulate_f32")
