"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and rejects bad
shapes and arguments without touching a GPU."""
import ctypes as C
import os
import math
import re

import pytest

import paper_2311_11514_amd as hx

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(inc, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(hexgen_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_symbols()
    assert len(names) >= 19
    raw = C.CDLL(hx.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), f"{n} declared in include/*.h but not exported"
        assert n in hx.SIGNATURES, f"{n} has no Python binding signature"
    assert sorted(hx.SIGNATURES) == names


def _create(*a):
    h = C.c_void_p()
    rc = hx.lib.hexgen_stage_create(*a, C.byref(h))
    if rc == 0:
        hx.lib.hexgen_stage_destroy(h)
    return rc


@pytest.mark.parametrize("args,status", [
    ((512, 8, 2, 1408, 2, 2, 0, 0), 0),
    ((8192, 64, 8, 28672, 8, 2, 0, 1), 0),
    ((8192, 64, 8, 28672, 8, 8, 3, 1), 0),
    ((512, 8, 2, 1408, 2, 3, 0, 0), 2),      # heads not divisible by tp
    ((512, 8, 2, 1408, 2, 4, 0, 0), 2),      # kv heads not divisible by tp
    ((512, 8, 2, 1409, 2, 2, 0, 0), 2),      # ffn not divisible
    ((512, 8, 3, 1408, 2, 1, 0, 0), 2),      # heads % kv heads
    ((500, 8, 2, 1408, 2, 2, 0, 0), 2),      # hidden % heads
    ((512, 8, 2, 1408, 2, 2, 2, 0), 2),      # rank out of range
    ((512, 16, 2, 1408, 2, 2, 0, 0), 2),     # head_dim 32 unsupported
    ((512, 8, 2, 1408, 0, 2, 0, 0), 1),      # no layers
    ((512, 8, 2, 1408, 2, 2, 0, 7), 1),      # unknown dtype
    ((1024, 8, 2, 1424, 2, 2, 0, 1), 2),     # bf16: local ffn 712 not a multiple of 32
    ((8192, 64, 8, 28672, 8, 4, 1, 2), 0),   # fp16 stage
    ((1024, 8, 2, 1424, 2, 2, 0, 2), 2),     # fp16: same alignment rules as bf16
    ((512, 8, 2, 1408, 2, 2, 0, 3), 1),      # first code past the enum
])
def test_stage_create_validation(args, status):
    assert _create(*args) == status


def test_null_and_range_arguments():
    assert hx.lib.hexgen_stage_create(512, 8, 2, 1408, 2, 2, 0, 0, None) == 1
    st = hx.Stage(512, 8, 2, 1408, 2, 2, 0, "f32")
    assert hx.lib.hexgen_stage_set_params(st.handle, -1.0, 1e4) == 1
    assert hx.lib.hexgen_stage_set_tap(st.handle, 5, None) == 1
    assert hx.lib.hexgen_stage_load_layer(st.handle, 0, *([None] * 9)) == 1
    assert hx.lib.hexgen_stage_weight_bytes(st.handle) == 0
    assert hx.lib.hexgen_status_string(4) == b"capacity exceeded"
    assert hx.lib.hexgen_accumulate_f32(None, None, 4, None) == 1
    st.close()


def test_fp16_workload_values_survive_the_storage_type():
    """Inputs drawn for an fp16 stage are fp16 values already, so the oracle (float64) and the stage (fp16 storage)
    start from identical numbers."""
    import torch
    from workloads import StageConfig, generate
    cfg = StageConfig("f16_probe", "f16", 512, 8, 4, 1408, 1, 1, (0,), batch=2, seed=42)
    for name, v in generate.layer_weights(cfg, 0).items():
        assert torch.equal(v, v.to(torch.float16).to(torch.float32)), name
    x = generate.hidden_rows(cfg, 7)
    assert torch.equal(x, x.to(torch.float16).to(torch.float32))
    assert hx.binding._dtype_code("f16") == hx.binding._dtype_code(torch.float16) == 2


# ---- cost model (host functions of the library) against the oracle ------------------------------------------------
def test_cost_model_functions_match_the_oracle():
    import math

    import numpy as np

    from oracle import cost_oracle as co
    rng = np.random.default_rng(3)
    for _ in range(50):
        n = int(rng.integers(1, 9))
        H, B, b = int(rng.choice([512, 4096, 8192])), int(rng.choice([2, 4])), int(rng.integers(1, 33))
        s_in, s_out, l = int(rng.integers(0, 2049)), int(rng.integers(0, 257)), int(rng.integers(0, 81))
        pf = float(rng.choice([12.0, 12.75]))
        m, c = list(rng.uniform(0.3e12, 8e12, n)), list(rng.uniform(50e12, 2500e12, n))
        for phase, ref in (("both", co.comp), ("prefill", co.comp_prefill), ("decode", co.comp_decode)):
            assert math.isclose(hx.cost_comp(H, B, b, s_in, s_out, l, m, c, pf, phase), ref(H, B, b, s_in, s_out, l, m, c, pf),
                                rel_tol=1e-12, abs_tol=0.0)
        al = rng.uniform(1e-6, 50e-6, (n, n)).tolist()
        be = rng.uniform(10e9, 400e9, (n, n)).tolist()
        assert math.isclose(hx.cost_comm_tp(H, B, b, s_in, s_out, l, al, be), co.comm_tp(H, B, b, s_in, s_out, l, al, be),
                            rel_tol=1e-12, abs_tol=0.0)
        n2 = int(rng.integers(1, 5))
        al2 = rng.uniform(1e-6, 50e-6, (n, n2)).tolist()
        be2 = rng.uniform(10e9, 400e9, (n, n2)).tolist()
        assert math.isclose(hx.cost_comm_pp(H, B, b, s_in, s_out, al2, be2), co.comm_pp(H, B, b, s_in, s_out, al2, be2),
                            rel_tol=1e-12)
        assert math.isclose(hx.cost_mem(H, B, b, s_in, s_out, l, n, pf), co.mem(H, B, b, s_in, s_out, l, n, pf), rel_tol=1e-12,
                            abs_tol=0.0)
    # invalid arguments give NaN, never a plausible number
    assert math.isnan(hx.cost_comp(0, 2, 1, 1, 1, 1, [1e12], [1e14]))
    assert math.isnan(hx.cost_comp(8192, 2, 1, 1, 1, 1, [0.0], [1e14]))
    assert math.isnan(hx.cost_comm_tp(8192, 2, 1, 1, 1, 1, [[0, 1e-6], [1e-6, 0]], [[1, 0.0], [1e9, 1]]))
    assert hx.cost_comm_tp(8192, 2, 1, 1, 1, 1, [[0.0]], [[1.0]]) == 0.0


def test_cost_model_library_on_the_hand_worked_comm_example():
    """The library's Eq. 4 / Eq. 5 on the non-uniform links worked by hand (tests/golden/cost_model_comm_worked_example.txt)."""
    from tests.test_oracle_pins import COMM_EXAMPLE as ex, _golden_cost
    gold = _golden_cost("cost_model_comm_worked_example.txt")
    t = ex["task"]
    args = (t["H"], t["B_type"], t["b"], t["s_in"], t["s_out"])
    assert math.isclose(hx.cost_comm_tp(*args, 3, ex["tp_alpha"], ex["tp_beta"]), gold["tp_total"], rel_tol=1e-12)
    assert math.isclose(hx.cost_comm_pp(*args, ex["pp_alpha"], ex["pp_beta"]), gold["pp_total"], rel_tol=1e-12)


# ---- pipeline layout DP and search operators against the oracle -------------------------------------------------
def test_pipeline_layout_dp_equals_brute_force():
    import math

    import numpy as np

    from oracle import sched_oracle as sch
    rng = np.random.default_rng(17)
    for trial in range(25):
        nt = int(rng.integers(1, 4))
        pool = {"count": [int(rng.integers(1, 5)) for _ in range(nt)],
                "m": list(rng.uniform(0.4e12, 6e12, nt)), "c": list(rng.uniform(60e12, 1500e12, nt)),
                "mem": list(rng.choice([16e9, 24e9, 48e9, 80e9, 192e9], nt)),
                "tp_alpha": list(rng.uniform(2e-6, 20e-6, nt)), "tp_beta": list(rng.uniform(20e9, 400e9, nt)),
                "pp_alpha": rng.uniform(5e-6, 200e-6, (nt, nt)).tolist(), "pp_beta": rng.uniform(1e9, 100e9, (nt, nt)).tolist()}
        task = (int(rng.choice([2048, 4096, 8192])), float(rng.choice([12.0, 12.75])), 2, int(rng.integers(1, 9)),
                int(rng.integers(16, 1025)), int(rng.integers(1, 129)))
        S = int(rng.integers(1, 4))
        layers = [int(rng.integers(1, 20)) for _ in range(S)]
        for pow2 in (False, True):
            ref, ref_asg = sch.best_layout_bruteforce(pool, task, layers, degrees={1, 2, 4, 8} if pow2 else None)
            cost, asg = hx.sched_pipeline_layout(pool, task, layers, pow2)
            if ref == math.inf:
                assert cost == math.inf
                continue
            assert math.isclose(cost, ref, rel_tol=1e-12), (trial, cost, ref)
            # the returned assignment is feasible and costs what the function says (ties may pick another optimum)
            used = [sum(n for k, n in asg if k == t) for t in range(nt)]
            assert all(u <= c for u, c in zip(used, pool["count"])) and all(n >= 1 for _, n in asg)
            total = sum(sch.stage_cost(pool, task, layers[j], k, n) for j, (k, n) in enumerate(asg))
            total += sum(sch.hop_cost(pool, task, asg[j][0], asg[j + 1][0]) for j in range(S - 1))
            assert math.isclose(total, cost, rel_tol=1e-12)


def test_search_operators_match_the_oracle():
    import numpy as np

    from oracle import sched_oracle as sch
    rng = np.random.default_rng(19)
    for _ in range(30):
        nt = int(rng.integers(1, 6))
        t1 = [int(v) for v in rng.integers(0, 9, nt)]
        t2 = [int(v) for v in rng.integers(0, 9, nt)]
        assert hx.sched_merge(t1, t2) == sch.merge(t1, t2)
        assert hx.sched_split(t1) == sch.split(t1)
        k = int(rng.integers(0, nt))
        if t2[k] >= 1:
            assert hx.sched_swap(t1, t2, k) == sch.swap(t1, t2, k)
        else:
            with pytest.raises(ValueError):
                hx.sched_swap(t1, t2, k)
        memt = [float(v) for v in rng.choice([24e9, 48e9, 80e9], nt)]
        model = float(rng.choice([13e9, 140e9, 400e9]))
        assert hx.sched_group_can_hold(t1, memt, model) == sch.group_can_hold(t1, memt, model)
        S = int(rng.integers(1, 7))
        memv = [float(v) for v in rng.choice([24e9, 48e9, 80e9, 160e9, 640e9], S)]
        L = int(rng.integers(S, 121))
        assert hx.sched_repartition_layers(L, memv) == sch.repartition_layers(L, memv)


def test_scheduler_functions_reject_invalid_arguments():
    import math
    pool = {"count": [2], "m": [1e12], "c": [1e14], "mem": [80e9], "tp_alpha": [1e-5], "tp_beta": [1e11],
            "pp_alpha": [[1e-5]], "pp_beta": [[1e10]]}
    task = (4096, 12.0, 2, 1, 128, 32)
    assert math.isnan(hx.sched_pipeline_layout(pool, task, [4, 0])[0])               # a stage without layers
    assert math.isnan(hx.sched_pipeline_layout(dict(pool, count=[-1]), task, [4])[0])
    assert math.isnan(hx.sched_pipeline_layout(dict(pool, count=[65]), task, [4])[0])
    # three stages cannot be served by two GPUs: no assignment, not an error
    assert hx.sched_pipeline_layout(pool, task, [2, 2, 2])[0] == math.inf
    # nothing fits the memory
    assert hx.sched_pipeline_layout(dict(pool, mem=[1e6]), task, [4])[0] == math.inf
    with pytest.raises(ValueError):
        hx.sched_repartition_layers(2, [1.0, 1.0, 1.0])                             # fewer layers than stages
    with pytest.raises(ValueError):
        hx.sched_repartition_layers(8, [1.0, 0.0])


def test_pipeline_layout_dp_at_sizes_enumeration_cannot_reach():
    """Larger pools (4 types, up to 8 GPUs each, 6 stages): the returned layout is feasible, re-prices (with the
    oracle's stage and hop costs) to the returned cost, and no randomly drawn feasible layout is cheaper."""
    import math

    import numpy as np

    from oracle import sched_oracle as sch
    rng = np.random.default_rng(23)
    for trial in range(6):
        nt = 4
        pool = {"count": [int(rng.integers(2, 9)) for _ in range(nt)],
                "m": list(rng.uniform(0.4e12, 6e12, nt)), "c": list(rng.uniform(60e12, 1500e12, nt)),
                "mem": list(rng.choice([24e9, 48e9, 80e9, 192e9], nt)),
                "tp_alpha": list(rng.uniform(2e-6, 20e-6, nt)), "tp_beta": list(rng.uniform(20e9, 400e9, nt)),
                "pp_alpha": rng.uniform(5e-6, 200e-6, (nt, nt)).tolist(), "pp_beta": rng.uniform(1e9, 100e9, (nt, nt)).tolist()}
        task = (8192, 12.75, 2, int(rng.integers(1, 5)), int(rng.integers(64, 1025)), int(rng.integers(1, 65)))
        S = 6
        layers = sch.repartition_layers(80, [1.0] * S)
        cost, asg = hx.sched_pipeline_layout(pool, task, layers, False)
        if cost == math.inf:
            continue
        used = [sum(n for k, n in asg if k == t) for t in range(nt)]
        assert all(u <= c for u, c in zip(used, pool["count"]))
        total = sum(sch.stage_cost(pool, task, layers[j], k, n) for j, (k, n) in enumerate(asg))
        total += sum(sch.hop_cost(pool, task, asg[j][0], asg[j + 1][0]) for j in range(S - 1))
        assert math.isclose(total, cost, rel_tol=1e-12)
        for _ in range(200):
            left = list(pool["count"])
            cand = []
            for j in range(S):
                k = int(rng.integers(0, nt))
                if left[k] == 0:
                    break
                n = int(rng.integers(1, left[k] + 1))
                left[k] -= n
                cand.append((k, n))
            if len(cand) < S:
                continue
            c2 = sum(sch.stage_cost(pool, task, layers[j], k, n) for j, (k, n) in enumerate(cand))
            c2 += sum(sch.hop_cost(pool, task, cand[j][0], cand[j + 1][0]) for j in range(S - 1))
            assert c2 >= cost * (1 - 1e-12)


# ---- SLO attainment and the search over deployments: product against the oracles -----------------------------------
def test_slo_attainment_equals_oracle():
    import numpy as np

    from oracle import slo_oracle as slo
    from workloads import serving
    rng = np.random.default_rng(23)
    for trial in range(30):
        n, n_rep, n_cls = int(rng.integers(1, 400)), int(rng.integers(1, 7)), int(rng.integers(1, 4))
        arrival = serving.poisson_arrivals(float(rng.uniform(0.2, 5.0)), n, trial)
        if trial % 5 == 0:
            arrival = sorted(float(round(a, 1)) for a in arrival)           # bursts: several requests at one instant
        latency = rng.uniform(0.2, 3.0, (n_rep, n_cls)).tolist()
        if trial % 3 == 0:
            latency[-1] = list(latency[0])                                   # identical replicas: ties
        deadline = rng.uniform(0.5, 6.0, n_cls).tolist()
        cls = None if n_cls == 1 else [int(c) for c in rng.integers(0, n_cls, n)]
        got, fin = hx.slo_attainment(arrival, latency, deadline, cls, return_finish=True)
        assert fin == slo.simulate(arrival, latency, cls)                    # same sums in the same order: bit-identical
        assert got == slo.attainment(arrival, latency, deadline, cls)


def test_slo_attainment_rejects_invalid_arguments():
    import math
    assert math.isnan(hx.slo_attainment([], [[1.0]], [1.0]))
    assert math.isnan(hx.slo_attainment([1.0, 0.5], [[1.0]], [1.0]))               # unsorted
    assert math.isnan(hx.slo_attainment([-1.0], [[1.0]], [1.0]))
    assert math.isnan(hx.slo_attainment([0.0], [[0.0]], [1.0]))                    # a latency of zero
    assert math.isnan(hx.slo_attainment([0.0], [[1.0]], [1.0], cls=[1]))           # class out of range
    assert math.isnan(hx.slo_attainment([float("nan")], [[1.0]], [1.0]))
    assert hx.slo_attainment([0.0], [[1.0]], [1.0]) == 1.0


def _check_plan(pool, task, tau, n_layers, cost, layers, stages, ref):
    """The plan is the oracle's, or (two stages of equal cost swapped: several plans are optimal) another feasible plan
    of the group that the oracle's cost functions price the same."""
    from oracle import sched_oracle as sch
    if layers == ref[1] and stages == [tuple(s) for s in ref[2]]:
        return
    assert sum(layers) == n_layers and min(layers) >= 1 and len(layers) == len(stages)
    assert all(sum(n for k, n in stages if k == t) <= tau[t] for t in range(len(tau))) and all(n >= 1 for _, n in stages)
    total = sum(sch.stage_cost(pool, task, layers[j], k, n) for j, (k, n) in enumerate(stages))
    total += sum(sch.hop_cost(pool, task, stages[j][0], stages[j + 1][0]) for j in range(len(stages) - 1))
    assert abs(total - ref[0]) <= 1e-12 * ref[0] and abs(total - cost) <= 1e-12 * cost


def test_search_pieces_equal_oracle():
    import math

    import numpy as np

    from oracle import search_oracle as srch
    from workloads import serving
    for seed in (0, 99, 12345, 2 ** 63 + 5):
        assert [hx.sched_draw(seed, c) for c in range(50)] == [srch.draw(seed, c) for c in range(50)]
    for kind in ("full_price", "half_price"):
        pool = serving.hetero_pool(kind)
        assert hx.sched_initial_groups(pool) == srch.initial_groups(pool)
    rng = np.random.default_rng(3)
    for seed in range(12):
        pool = serving.tiny_pool(seed, int(rng.integers(1, 6)), 4, two_regions=bool(seed % 3))
        assert hx.sched_initial_groups(pool) == srch.initial_groups(pool)
    assert hx.sched_initial_groups(dict(serving.tiny_pool(1, 3), count=[0, 0, 0])) == []
    task = (4096, 12.0, 2, 1, 128, 32)
    for seed in range(6):
        pool = serving.tiny_pool(seed, 3, 3)
        pool["mem"] = [m / 8 for m in pool["mem"]]
        for tau in (pool["count"], [1, 1, 0], [0, 1, 1], [pool["count"][0], 0, 1]):
            for pow2 in (False, True):
                ref = srch.plan_group(pool, task, tau, 16, 3, degrees={1, 2, 4} if pow2 else None)
                cost, layers, stages = hx.sched_plan_group(pool, task, tau, 16, 3, pow2)
                if ref[0] == math.inf:
                    assert cost == math.inf and layers == []
                    continue
                assert abs(cost - ref[0]) <= 1e-12 * ref[0]
                _check_plan(pool, task, tau, 16, cost, layers, stages, ref)


def test_search_equals_oracle():
    import math

    from oracle import search_oracle as srch
    from workloads import serving
    task = (4096, 12.0, 2, 1, 128, 32)
    n_layers = 16
    model_bytes = n_layers * 12 * 4096 ** 2 * 2
    improved = 0
    for seed in (1, 2, 4, 5, 7):
        pool = serving.tiny_pool(seed, 3, 3)
        pool["mem"] = [m / 8 for m in pool["mem"]]
        whole = hx.sched_plan_group(pool, task, pool["count"], n_layers, 3)[0]
        arrival = serving.poisson_arrivals(1.2 / whole, 150, seed)
        for pop in (1, 4):
            ref = srch.search(pool, task, n_layers, model_bytes, 3, arrival, 2.5 * whole, seed, 60, pop)
            got = hx.sched_search(pool, task, n_layers, model_bytes, 3, arrival, 2.5 * whole, seed, 60, pop)
            assert got["history"] == ref["history"] and got["attainment"] == ref["attainment"]
            assert [g["tau"] for g in got["groups"]] == [g["tau"] for g in ref["groups"]]
            for a, b in zip(got["groups"], ref["groups"]):
                assert abs(a["latency"] - b["latency"]) <= 1e-12 * b["latency"]
                _check_plan(pool, task, a["tau"], n_layers, a["latency"], a["layers"], a["stages"],
                            (b["latency"], b["layers"], b["stages"]))
            improved += ref["history"][-1] > ref["history"][0] or ref["history"][0] == 1.0
    assert improved >= 4
    # unusable hop links are rejected (the K-means features would not be numbers)
    bad = serving.tiny_pool(1, 2, 2)
    bad["pp_beta"][0][1] = 0.0
    assert hx.sched_initial_groups(bad) == []
    assert math.isnan(hx.sched_search(bad, task, n_layers, model_bytes, 3, [0.0, 1.0], 1.0, 0, 5, 2)["attainment"])
    # a pool that cannot hold the model at all
    pool = serving.tiny_pool(1, 2, 2)
    assert math.isnan(hx.sched_search(pool, task, n_layers, 1e15, 3, [0.0, 1.0], 1.0, 0, 5, 2)["attainment"])


def test_search_on_the_large_pool_keeps_its_invariants():
    from workloads import serving
    pool = serving.hetero_pool("half_price")
    task = (8192, 12.0, 2, 1, 128, 32)
    n_layers, model_bytes = 80, 80 * 12 * 8192 ** 2 * 2
    start = hx.sched_initial_groups(pool)
    lat0 = [hx.sched_plan_group(pool, task, g, n_layers, 8, True)[0] for g in start]
    arrival = serving.poisson_arrivals(0.5, 300, 7)
    res = hx.sched_search(pool, task, n_layers, model_bytes, 8, arrival, 5 * min(lat0), 11, 150, 8, True)
    groups = [g["tau"] for g in res["groups"]]
    assert [sum(g[k] for g in groups) for k in range(3)] == pool["count"]
    assert all(b >= a for a, b in zip(res["history"], res["history"][1:]))
    assert res["attainment"] == res["history"][-1] >= hx.slo_attainment(arrival, [[x] for x in lat0], [5 * min(lat0)])
    for g in res["groups"]:
        assert sum(g["layers"]) == n_layers and all(n in (1, 2, 4, 8) for _, n in g["stages"])
        used = [sum(n for k, n in g["stages"] if k == t) for t in range(3)]
        assert all(u <= c for u, c in zip(used, g["tau"]))
        # the group's latency is what the layout routine gives for its plan
        cost, _ = hx.sched_pipeline_layout(dict(pool, count=g["tau"]), task, g["layers"], True)
        assert abs(cost - g["latency"]) <= 1e-12 * cost
    assert res["attainment"] == hx.slo_attainment(arrival, [[g["latency"]] for g in res["groups"]], [5 * min(lat0)])


def test_bench_refuses_more_than_one_gpu_and_a_missing_gpu():
    """bench.py measures one GPU: `--gpus 2` ends with a message and a non-zero status before anything is imported, and
    without a GPU the default run fails loudly instead of timing anything on the CPU."""
    import os
    import subprocess
    import sys
    import torch
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=root)
    assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout.strip() == ""
    if not torch.cuda.is_available():
        p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "1", "--warmup", "0"], capture_output=True,
                           text=True, cwd=root)
        assert p.returncode != 0 and "needs a GPU" in p.stderr and p.stdout.strip() == ""
