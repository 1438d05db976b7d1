"""Host side of the library vs the oracle, bit-exact, and the C-ABI surface.
CPU only: no GPU call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2604_25080_amd as cf
from oracle import planner as P
from oracle.pagetable import PageTable
from workloads import churn_script, hand_cost_model, make_batch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def both_cost(d):
    return P.CostModel(**d), cf.cost_model(**d)


def both_opts(chunk, l_delta, n_layers, kvb, mode=-1, key=0, kv_only=0, boundary=0):
    return (P.PlanOpts(chunk, l_delta, n_layers, kvb, mode, key, kv_only, boundary),
            cf.plan_opts(chunk, l_delta, n_layers, kvb, mode, key, kv_only, boundary))


# ------------------------------------------------------------------ C-ABI surface
def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "cacheflow.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(cf_[a-z0-9_]+)\s*\(", hdr))
    assert declared, "no declarations found"
    assert declared == set(cf.binding.EXPORTS)
    for name in declared:
        assert hasattr(cf.lib, name), name


def test_struct_sizes_match_the_header_layout():
    assert ctypes.sizeof(cf.cf_cost_model) == 56
    assert ctypes.sizeof(cf.cf_plan_opts) == 32
    assert ctypes.sizeof(cf.cf_split) == 12
    assert ctypes.sizeof(cf.cf_plan_stats) == 32
    assert ctypes.sizeof(cf.cf_model_desc) == 40
    assert ctypes.sizeof(cf.cf_request) == 48
    assert ctypes.sizeof(cf.cf_timing) == 64
    assert ctypes.sizeof(cf.cf_dynamic_stats) == 40
    assert ctypes.sizeof(cf.cf_dynamic_opts) == 24
    assert ctypes.sizeof(cf.cf_overlap_model) == 8
    assert ctypes.sizeof(cf.cf_batch_plan_opts) == 28
    assert ctypes.sizeof(cf.cf_batch_plan) == 72


def test_status_strings():
    assert cf.lib.cf_status_str(0) == b"ok"
    assert b"pages" in cf.lib.cf_status_str(cf.CF_ERR_OUT_OF_PAGES)


# --------------------------------------------------------------------- planner
def test_planner_matches_oracle_on_random_batches():
    rng = np.random.default_rng(41)
    for trial in range(1500):
        d = dict(f_c=int(rng.integers(0, 50_000_000)), alpha=int(rng.integers(1, 2_000_000)),
                 beta=int(rng.integers(0, 60_000)), f_io=int(rng.integers(0, 20_000_000)),
                 gamma=int(rng.integers(1, 900_000_000)),
                 s_c=int(rng.choice([0, 0, 3_000_000_000])), s_io=int(rng.choice([0, 0, 400_000_000])))
        ocm, ccm = both_cost(d)
        chunk = 16 * int(rng.integers(1, 40))
        oo, co = both_opts(chunk, int(rng.choice([0, 300, 2000, 10 ** 6])), int(rng.integers(1, 40)),
                           int(rng.choice([512, 4096, 1024])), int(rng.integers(-1, 2)),
                           int(rng.integers(0, 3)), int(rng.choice([0, 0, 115, 98, 1000])),
                           int(rng.choice([0, 0, 512, 16384, 32768])))
        n_ctx = [int(rng.integers(0, 6000)) for _ in range(int(rng.integers(1, 12)))]
        otrace = []
        osplits, ostats = P.plan(ocm, oo, n_ctx, trace=otrace)
        csplits, cstats, ctrace = cf.restore_plan(ccm, co, n_ctx, trace_cap=100000)
        assert csplits == osplits, (trial, n_ctx)
        assert cstats == ostats
        assert ctrace == otrace


@pytest.mark.parametrize("cfg", ["cfg2", "cfg3", "cfg4", "cfg5"])
def test_planner_matches_oracle_on_benchmark_batches(cfg):
    b = make_batch(cfg)
    s = b.shape
    for kind in ("mi355x_like", "balanced", "slow_io", "startup"):
        ocm, ccm = both_cost(hand_cost_model(kind))
        oo, co = both_opts(b.chunk_tokens, 2048, s.n_layers, s.kv_bytes_per_token_layer, b.forced_mode)
        otrace = []
        osplits, ostats = P.plan(ocm, oo, b.n_ctx, trace=otrace)
        csplits, cstats, ctrace = cf.restore_plan(ccm, co, b.n_ctx, trace_cap=len(otrace) + 5)
        assert (csplits, cstats, ctrace) == (osplits, ostats, otrace)


def test_plan_eval_and_l_delta_match_oracle():
    rng = np.random.default_rng(42)
    for _ in range(100):
        d = hand_cost_model(str(rng.choice(["mi355x_like", "balanced", "slow_io", "uniform", "startup"])))
        ocm, ccm = both_cost(d)
        oo, co = both_opts(64 * int(rng.integers(1, 9)), 0, int(rng.integers(1, 33)), 4096, int(rng.integers(0, 2)),
                           boundary=int(rng.choice([0, 16384])))
        n_ctx = [int(rng.integers(1, 5000)) for _ in range(3)]
        splits, _ = P.plan(ocm, oo, n_ctx)
        units = [(-(-s[1] // oo.chunk_tokens) if s[0] == 0 else s[2]) for s in splits]
        assert cf.plan_eval(ccm, co, n_ctx, splits) == P.split_times(ocm, oo, n_ctx, units)
    for kind in ("mi355x_like", "balanced", "slow_io"):
        ocm, ccm = both_cost(hand_cost_model(kind))
        oo, co = both_opts(512, 0, 32, 4096)
        assert cf.derive_l_delta(ccm, co, 20000) == P.derive_l_delta(ocm, oo, 20000)


def test_prefill_cost_matches_oracle_and_the_formula_by_hand():
    cm_kw = hand_cost_model("balanced")
    ocm, ccm = P.CostModel(**cm_kw), cf.cost_model(**cm_kw)
    rng = np.random.default_rng(4)
    for _ in range(20):
        B = int(rng.integers(1, 9))
        n_ctx = [int(x) for x in rng.integers(0, 20000, size=B)]
        n_new = [int(x) for x in rng.integers(0, 600, size=B)]
        L = int(rng.integers(1, 81))
        assert cf.prefill_cost(ccm, L, n_ctx, n_new) == P.prefill_cost(ocm, L, n_ctx, n_new)
    # by hand: 3 tokens from position 10 through 2 layers: pairs = 3*10 + 3*4/2 = 36 -> 1 block
    want = 2 * (ocm.f_c + 3 * ocm.alpha + 1 * ocm.beta)
    assert cf.prefill_cost(ccm, 2, [10], [3]) == want == P.prefill_cost(ocm, 2, [10], [3])
    assert cf.prefill_cost(ccm, 2, [10], [0]) == 0


def test_cost_feedback_matches_oracle_and_balances_a_contended_plan():
    rng = np.random.default_rng(43)
    for _ in range(200):
        d = dict(f_c=int(rng.integers(0, 10 ** 8)), alpha=int(rng.integers(1, 10 ** 6)), beta=int(rng.integers(0, 10 ** 5)),
                 f_io=int(rng.integers(0, 10 ** 8)), gamma=int(rng.integers(1, 10 ** 9)),
                 s_c=int(rng.integers(0, 10 ** 10)), s_io=int(rng.integers(0, 10 ** 9)))
        ocm, ccm = both_cost(d)
        args = [int(rng.integers(0, 10 ** 12)) for _ in range(4)]
        want = P.cost_feedback(ocm, *args)
        cf.cost_feedback(ccm, *args)
        assert (ccm.f_c, ccm.alpha, ccm.beta, ccm.f_io, ccm.gamma, ccm.s_c, ccm.s_io) == \
               (want.f_c, want.alpha, want.beta, want.f_io, want.gamma, want.s_c, want.s_io)
    # hand case: compute ran 20 % slower than predicted, I/O as predicted
    ccm = cf.cost_model(0, 1000, 10, 0, 2000, 500, 100)
    cf.cost_feedback(ccm, 1_000_000, 1_200_000, 5_000, 5_000)
    assert (ccm.alpha, ccm.beta, ccm.s_c, ccm.gamma, ccm.s_io) == (1200, 12, 600, 2000, 100)
    # a world where compute is really 1.5x slower than the model says: a few rounds of
    # feedback move the split until predicted compute and I/O times balance under the truth
    true = P.CostModel(**hand_cost_model("startup"))
    true = P.CostModel(true.f_c, true.alpha * 3 // 2, true.beta * 3 // 2, true.f_io, true.gamma, true.s_c, true.s_io)
    model = cf.cost_model(**hand_cost_model("startup"))
    opts_o, opts_c = both_opts(512, 0, 32, 4096, 0)
    n_ctx = make_batch("cfg2").n_ctx
    for _ in range(4):
        splits, st, _ = cf.restore_plan(model, opts_c, n_ctx)
        units = [-(-s[1] // 512) for s in splits]
        t_c, t_io = P.split_times(true, opts_o, n_ctx, units)          # what "really" happens
        cf.cost_feedback(model, st["t_comp"], t_c, st["t_io"], t_io)
    assert abs(t_c - t_io) < 0.1 * max(t_c, t_io)


def test_planning_policy_matches_oracle_on_random_batches_and_hand_cases():
    """cf_plan_batch / cf_plan_feedback against their oracle twins: splits, plan kind, every
    predicted time and the corrected models, bit for bit, over random cost tables, contention
    factors, model widths, join modes, new turns and stages."""
    from workloads import SHAPES
    rng = np.random.default_rng(47)
    kinds = [0, 0, 0]
    for trial in range(600):
        d = dict(f_c=int(rng.integers(0, 50_000_000)), alpha=int(rng.integers(1, 2_000_000)),
                 beta=int(rng.integers(0, 60_000)), f_io=int(rng.integers(0, 20_000_000)),
                 gamma=int(rng.integers(1_000_000, 900_000_000)), s_c=int(rng.integers(0, 10 ** 10)),
                 s_io=int(rng.integers(0, 10 ** 9)))
        if trial % 3 == 0:          # around the point where the three candidates are close
            d = dict(hand_cost_model("startup"))
            d["gamma"] = int(d["gamma"] * rng.uniform(0.3, 30))
        ocm, ccm = both_cost(d)
        sh = SHAPES[("8b", "70b-tp8", "mini-bf16", "tiny")[trial % 4]]
        model = (sh.n_layers, sh.d_model, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.d_ffn, sh.elem_bytes)
        desc = cf.model_desc(sh)
        ov = (int(rng.integers(500, 3000)), int(rng.integers(500, 3000))) if trial % 5 else (1000, 1000)
        B = int(rng.integers(1, 7))
        n_ctx = [int(x) for x in rng.integers(0, 6000, size=B)]
        n_new = [int(x) for x in rng.integers(0, 300, size=B)] if trial % 4 else None
        chunk = int(rng.choice([16, 256, 512]))
        l_delta = int(rng.choice([0, 1024, 4096]))
        mode, key, piped = int(rng.integers(-1, 2)), int(rng.integers(0, 3)), bool(rng.integers(0, 2))
        stage = int(rng.integers(1, sh.n_layers + 1)) if trial % 7 == 0 or trial % 11 == 0 else 0
        first = int(rng.integers(0, sh.n_layers - stage + 1)) if stage else 0
        want_sp, want = P.plan_batch(ocm, ov, model, chunk, l_delta, mode, key, piped, n_ctx, n_new, stage, first)
        cov = cf.overlap_model(*ov)
        got_sp, info = cf.plan_batch(ccm, cov, desc, cf.batch_plan_opts(chunk, l_delta, mode, key, piped, stage, first),
                                     n_ctx, n_new)
        assert got_sp == want_sp, (trial, got_sp, want_sp)
        got = info.as_dict()
        got.pop("reserved")
        assert got == want, (trial, got, want)
        kinds[want["kind"]] += 1
        meas = [int(rng.integers(0, 4 * max(want["ttft"], 1))) for _ in range(3)]
        meas.append(int(rng.integers(0, meas[0] + 1)) if trial % 2 else 0)
        ocm2, ov2 = P.plan_feedback(ocm, ov, want, *meas)
        cf.lib.cf_plan_feedback(ccm, cov, info, *meas)
        assert (cov.comp_permille, cov.io_permille) == ov2
        assert (ccm.f_c, ccm.alpha, ccm.beta, ccm.f_io, ccm.gamma, ccm.s_c, ccm.s_io) == \
               (ocm2.f_c, ocm2.alpha, ocm2.beta, ocm2.f_io, ocm2.gamma, ocm2.s_c, ocm2.s_io)
    assert min(kinds) >= 20, kinds          # all three outcomes occur
    # argument errors are codes, not crashes
    sh = SHAPES["8b"]
    with pytest.raises(cf.CfError):
        cf.plan_batch(cf.cost_model(**hand_cost_model("startup")), cf.overlap_model(100, 1000), cf.model_desc(sh),
                      cf.batch_plan_opts(512, 0), [4096])
    with pytest.raises(cf.CfError):
        cf.plan_batch(cf.cost_model(**hand_cost_model("startup")), cf.overlap_model(), cf.model_desc(sh),
                      cf.batch_plan_opts(512, 0, stage_layers=33), [4096])
    with pytest.raises(cf.CfError):         # the stage must lie inside the model
        cf.plan_batch(cf.cost_model(**hand_cost_model("startup")), cf.overlap_model(), cf.model_desc(sh),
                      cf.batch_plan_opts(512, 0, stage_layers=8, stage_first_layer=25), [4096])
    with pytest.raises(cf.CfError):
        cf.restore_plan(cf.cost_model(**hand_cost_model("startup")), cf.plan_opts(512, 0, 32, 4096, boundary_bytes_per_token=-1), [4096])


def test_run_time_scheduling_calls_match_oracle_on_random_states():
    rng = np.random.default_rng(44)
    n_cases = n_multi = n_given_back = 0
    for it in range(400):
        d = dict(f_c=int(rng.integers(0, 50_000_000)), alpha=int(rng.integers(100_000, 2_000_000)),
                 beta=int(rng.integers(0, 60_000)), f_io=int(rng.integers(0, 20_000_000)),
                 gamma=int(rng.integers(5_000_000, 900_000_000)))
        ocm, ccm = both_cost(d)
        mode = int(rng.integers(-1, 2))
        key = int(rng.integers(0, 3))
        opts_o, opts_c = both_opts(int(rng.choice([16, 64, 512])), int(rng.integers(0, 3000)),
                                   int(rng.integers(1, 9)), 4096, mode, key, int(rng.integers(0, 400)))
        b = int(rng.integers(1, 7))
        n = [int(x) for x in rng.integers(0, 4000, size=b)]
        m = [len(P.unit_costs(ocm, opts_o, x, P.request_mode(opts_o, x))[0]) for x in n]
        pc = [int(rng.integers(0, mi + 1)) for mi in m]
        pio = [int(rng.integers(-1, mi)) if mi else -1 for mi in m]
        closed = [bool(rng.integers(0, 4) == 0) for _ in range(b)]
        backlog = int(rng.integers(0, 3 * 10 ** 10))
        busy = int(rng.integers(0, 10 ** 10))
        sc, sio = int(rng.integers(250, 4001)), int(rng.integers(250, 4001))
        fixed = int(rng.integers(0, 2) * rng.integers(0, 10 ** 10))
        cap = int(rng.integers(0, 2) * rng.integers(0, 10 ** 10))
        order = int(rng.integers(0, 2))
        later = int(rng.integers(0, 2) * rng.integers(0, 10 ** 10))
        max_units = int(rng.choice([0, 1, 1, 2, 3]))
        alone = int(rng.integers(0, 2) * rng.integers(250, 4001))
        want_take, want_a = P.dynamic_claim(ocm, opts_o, n, pc, pio, closed, backlog, sc, sio, fixed, cap, order, later,
                                            max_units, alone)
        got_take, got_a = cf.dynamic_claim(ccm, opts_c, n, pc, pio, closed, backlog, sc, sio, fixed, cap, order, later,
                                           max_units, alone)
        assert (got_take, got_a) == (want_take, want_a), (it, n, pc, pio, max_units, alone)
        n_multi += max(want_take, default=0) > 1 and any(t > 2 for t in want_take)
        n_given_back += alone > 0 and not any(want_take) and any(
            P.dynamic_claim(ocm, opts_o, n, pc, pio, closed, backlog, sc, sio, fixed, cap, order, later, max_units, 0)[0])
        want = P.io_pick(ocm, opts_o, n, pc, pio, closed, backlog, busy, sc, sio)
        got = cf.dynamic_io_pick(ccm, opts_c, n, pc, pio, closed, backlog, busy, sc, sio)
        assert got == want, (it, n, pc, pio)
        n_cases += any(want_take) + (want >= 0)
    assert n_cases > 200         # the states are not all trivial
    assert n_multi > 10 and n_given_back > 10     # steps with several chunks of a request; units given back
    cm = cf.cost_model(**hand_cost_model("balanced"))
    with pytest.raises(cf.CfError) as e:
        cf.dynamic_claim(cm, cf.plan_opts(512, 0, 32, 4096), [1000], [3], [1], None, 0)    # 2 units only
    assert e.value.status == cf.CF_ERR_INVALID_ARG
    with pytest.raises(cf.CfError):
        cf.dynamic_io_pick(cm, cf.plan_opts(512, 0, 32, 4096), [1000], [0], [1], None, -1, 0)
    with pytest.raises(cf.CfError):
        cf.dynamic_claim(cm, cf.plan_opts(512, 0, 32, 4096), [1000], [0], [1], None, 0, 0, 1000)


def test_planner_rejects_bad_arguments():
    cm = cf.cost_model(**hand_cost_model("balanced"))
    with pytest.raises(cf.CfError) as e:
        cf.restore_plan(cm, cf.plan_opts(0, 0, 32, 4096), [100])
    assert e.value.status == cf.CF_ERR_INVALID_ARG
    with pytest.raises(cf.CfError):
        cf.restore_plan(cm, cf.plan_opts(512, 0, 32, 4096), [-1])
    with pytest.raises(cf.CfError) as e:
        cf.plan_eval(cm, cf.plan_opts(512, 0, 32, 4096), [100], [(0, 101, 32)])
    assert e.value.status == cf.CF_ERR_INVALID_PLAN
    assert cf.restore_plan(cm, cf.plan_opts(512, 0, 32, 4096), [])[0] == []


def test_planner_is_fast_enough_for_the_serving_path():
    import time
    b = make_batch("cfg4")
    cm = cf.cost_model(**hand_cost_model("mi355x_like"))
    o = cf.plan_opts(512, 2048, 32, 4096)
    t0 = time.perf_counter()
    for _ in range(20):
        cf.restore_plan(cm, o, b.n_ctx)
    assert (time.perf_counter() - t0) / 20 < 5e-3


# ------------------------------------------------------------------ page table
def test_page_table_matches_oracle_under_churn():
    for seed in range(8):
        n_pages = 96
        page_bytes = 2 * 2 * 16 * 64 * 4
        c = cf.Cache(0, n_pages * 3 * page_bytes + 17, 3, 2, 64, cf.CF_F32)
        o = PageTable(n_pages)
        assert c.n_pages == n_pages and c.page_bytes == page_bytes
        for op in churn_script(seed, n_pages, n_ops=120):
            if op[0] == "alloc":
                c.alloc(op[1], op[2])
                assert c.page_table(op[1]) == o.alloc(op[1], op[2])
            else:
                c.free(op[1])
                o.release(op[1])
            assert c.n_free == o.n_free()
        for rid in o.tables:
            assert c.page_table(rid) == o.table(rid)


def test_page_table_errors():
    c = cf.Cache(0, 4 * 2 * 1 * 16 * 64 * 2 * 2, 2, 1, 64, cf.CF_BF16)
    assert c.n_pages == 4
    c.alloc(7, 40)
    with pytest.raises(cf.CfError) as e:
        c.alloc(7, 1)
    assert e.value.status == cf.CF_ERR_UNKNOWN_REQUEST
    with pytest.raises(cf.CfError) as e:
        c.alloc(8, 2 * 16 + 1)
    assert e.value.status == cf.CF_ERR_OUT_OF_PAGES
    with pytest.raises(cf.CfError) as e:
        c.free(9)
    assert e.value.status == cf.CF_ERR_UNKNOWN_REQUEST
    c.alloc(8, 0)
    assert c.page_table(8) == []
    c.free(7)
    assert c.n_free == 4


def test_host_kv_bytes_follows_the_size_formula():
    # 2 * L * Hkv * hd * N elements (Sec. 2), rounded up to whole 16-token pages
    assert cf.host_kv_bytes(32, 8, 128, cf.CF_BF16, 4096) == 2 * 32 * 8 * 128 * 4096 * 2
    assert cf.host_kv_bytes(2, 4, 64, cf.CF_F32, 17) == 2 * 2 * 4 * 64 * 32 * 4


def test_workspace_and_ctx_argument_checks_need_no_gpu():
    from workloads import SHAPES
    d = cf.model_desc(SHAPES["tiny"])
    assert cf.workspace_bytes(d, cf.ctx_opts(2, 256, 256)) > 0
    bad = cf.model_desc(SHAPES["tiny"])
    bad.head_dim = 96
    with pytest.raises(cf.CfError) as e:
        cf.workspace_bytes(bad, cf.ctx_opts(2, 256, 256))
    assert e.value.status == cf.CF_ERR_UNSUPPORTED


def test_bench_refuses_more_than_one_gpu_with_a_message():
    """The benchmark runs on one GPU; asking for more ends with a message, before any GPU work."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
