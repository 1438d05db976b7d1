"""Pins for oracle/planner.py: Eq. 1 closed forms, brute force on tiny
batches, structural properties of Algorithm 1 (Sec. 3.1-3.3).  CPU only."""
import numpy as np
import pytest

from oracle import planner as P
from workloads import hand_cost_model


def cm_of(kind):
    return P.CostModel(**hand_cost_model(kind))


def rand_cm(rng, overheads=True, startups=False):
    return P.CostModel(
        s_c=int(rng.integers(0, 400_000_000)) if startups else 0,
        s_io=int(rng.integers(0, 100_000_000)) if startups else 0,
        f_c=int(rng.integers(0, 50_000_000)) if overheads else 0,
        alpha=int(rng.integers(100_000, 2_000_000)),
        beta=int(rng.integers(0, 60_000)),
        f_io=int(rng.integers(0, 20_000_000)) if overheads else 0,
        gamma=int(rng.integers(5_000_000, 900_000_000)))


# ------------------------------------------------------------ Algorithm 1 init
def test_mode_rule_and_pointer_init():
    opts = P.PlanOpts(512, 2048, 32, 4096)
    assert P.request_mode(opts, 2048) == P.TOKEN_WISE       # N_c >= L_delta
    assert P.request_mode(opts, 2047) == P.LAYER_WISE
    a, b, tok = P.unit_costs(cm_of("balanced"), opts, 1300, P.TOKEN_WISE)
    assert len(a) == 3 and tok == [512, 512, 276]           # ceil(N_c / C) chunks
    a, b, tok = P.unit_costs(cm_of("balanced"), opts, 1300, P.LAYER_WISE)
    assert len(a) == 32 and tok == [1300] * 32              # L units


def test_cost_formula_by_hand():
    cm = P.CostModel(f_c=7, alpha=3, beta=5, f_io=11, gamma=13)
    # 2 layers, 4 tokens starting at position 6: pairs = 4*6 + 4*5/2 = 34 -> ceil(34/1024)=1
    assert P.compute_cost(cm, 2, 4, 6) == 2 * (7 + 3 * 4 + 5 * 1)
    assert P.compute_cost(cm, 1, 2048, 0) == 7 + 3 * 2048 + 5 * ((2048 * 2049 // 2 + 1023) // 1024)
    assert P.io_cost(cm, 1 << 20) == 11 + 13
    assert P.io_cost(cm, (1 << 20) + 1) == 11 + 14           # ceil


def test_later_chunks_cost_more_to_recompute_not_to_load():
    a, b, _ = P.unit_costs(cm_of("mi355x_like"), P.PlanOpts(512, 0, 32, 4096), 8192, P.TOKEN_WISE)
    assert all(a[i] < a[i + 1] for i in range(len(a) - 1))   # quadratic attention term
    assert len(set(b)) == 1                                  # I/O linear in bytes


# ------------------------------------------------------------------ Eq. 1 pins
@pytest.mark.parametrize("ratio", [0.25, 1.0, 3.0])
def test_single_request_uniform_costs_meet_at_the_closed_form_split(ratio):
    # layer-wise, uniform units: a per layer = alpha*n, b per layer = gamma*bytes/2^20
    L, n = 64, 1024
    alpha = 1_000_000
    per_layer_bytes = 1 << 20
    gamma = int(alpha * n * ratio)          # T_io / T_comp = ratio
    cm = P.CostModel(0, alpha, 0, 0, gamma)
    opts = P.PlanOpts(512, 0, L, per_layer_bytes // n, P.LAYER_WISE)
    splits, st = P.plan(cm, opts, [n])
    t_comp, t_io = L * alpha * n, L * gamma
    l_star = L * t_io / (t_comp + t_io)                      # Eq. 1
    t_star = t_comp * t_io / (t_comp + t_io)
    assert abs(splits[0][2] - l_star) <= 1
    assert splits[0][1] == n
    unit = max(alpha * n, gamma)
    assert t_star <= st["makespan"] <= t_star + unit
    assert st["makespan"] <= min(t_comp, t_io)               # T* <= min(T_comp, T_io)


def test_makespan_tends_to_the_harmonic_mean_as_units_shrink():
    alpha, gamma_total = 1_000_000, 3_000_000 * 4096
    gaps = []
    for L in (8, 64, 512):
        cm = P.CostModel(0, alpha * 512 // L, 0, 0, gamma_total // L)
        opts = P.PlanOpts(512, 0, L, (1 << 20) // 4096, P.LAYER_WISE)
        _, st = P.plan(cm, opts, [4096])
        t_comp, t_io = P.split_times(cm, opts, [4096], [L])[0], P.split_times(cm, opts, [4096], [0])[1]
        t_star = t_comp * t_io / (t_comp + t_io)
        gaps.append(st["makespan"] / t_star - 1.0)
    assert gaps[0] >= gaps[1] >= gaps[2] and gaps[2] < 0.01


# ------------------------------------------------------------- brute force pins
def test_single_request_matches_brute_force_exactly():
    rng = np.random.default_rng(21)
    for trial in range(300):
        cm = rand_cm(rng, startups=trial % 2 == 1)
        mode = int(rng.integers(0, 2))
        opts = P.PlanOpts(16 * int(rng.integers(1, 5)), 0, int(rng.integers(1, 9)),
                          int(rng.choice([512, 4096])), mode,
                          kv_only_permille=int(rng.choice([0, 115, 1000])))
        n = int(rng.integers(1, 16 * 40))
        _, st = P.plan(cm, opts, [n])
        best, _ = P.brute_force(cm, opts, [n])
        assert st["makespan"] == best, (trial, cm, opts, n)


def test_last_recomputed_layer_costs_only_its_kv_projection():
    """With kv_only_permille set, a request's LAST recomputed layer is priced f_c + alpha*t*p/1000
    (no attention).  By hand: token-wise chunk = L-1 full layers + one K/V-only layer; layer-wise
    c claimed layers = c-1 full + one K/V-only, whichever c (each claim completes the layer below
    it); permille 1000 with beta = 0 is the old pricing; the plan never recomputes less."""
    cm = P.CostModel(f_c=7, alpha=1000, beta=13, f_io=5, gamma=10 ** 6)
    full = lambda t, p0: 7 + 1000 * t + 13 * -(-(t * p0 + t * (t + 1) // 2) // 1024)
    kvo = lambda t, p: 7 + -(-(1000 * p * t) // 1000)
    o = P.PlanOpts(32, 0, 5, 4096, P.TOKEN_WISE, kv_only_permille=115)
    a, b, tok = P.unit_costs(cm, o, 80, P.TOKEN_WISE)
    assert a == [4 * full(32, 0) + kvo(32, 115), 4 * full(32, 32) + kvo(32, 115), 4 * full(16, 64) + kvo(16, 115)]
    a, b, tok = P.unit_costs(cm, o, 80, P.LAYER_WISE)
    assert a == [kvo(80, 115)] + [full(80, 0)] * 4
    for c in range(1, 6):
        assert sum(a[:c]) == (c - 1) * full(80, 0) + kvo(80, 115)
    flat = P.CostModel(f_c=7, alpha=1000, beta=0, f_io=5, gamma=10 ** 6)
    for mode in (P.TOKEN_WISE, P.LAYER_WISE):
        old = P.unit_costs(flat, P.PlanOpts(32, 0, 5, 4096, mode), 80, mode)
        new = P.unit_costs(flat, P.PlanOpts(32, 0, 5, 4096, mode, kv_only_permille=1000), 80, mode)
        assert old == new
    rng = np.random.default_rng(8)
    for _ in range(100):
        cmr = rand_cm(rng)
        n_ctx = [int(rng.integers(1, 3000)) for _ in range(int(rng.integers(1, 6)))]
        mode = int(rng.integers(0, 2))
        s0, _ = P.plan(cmr, P.PlanOpts(64, 0, 8, 4096, mode), n_ctx)
        s1, _ = P.plan(cmr, P.PlanOpts(64, 0, 8, 4096, mode, kv_only_permille=115), n_ctx)
        assert sum(k * c for _, k, c in s1) >= sum(k * c for _, k, c in s0)


def test_boundary_rows_of_a_stage_above_layer_0_cost_the_channel_hand_cases():
    """A stage above layer 0 recomputes from cached stage-input rows that cross the same link
    as the KV (Sec. 3.2).  gamma = 2^20 makes a byte cost 1: by hand, a token-wise chunk costs
    the channel tokens * bytes when it is RECOMPUTED, a layer-wise request all its rows at the
    first layer it recomputes and nothing after.  Hand trace, one request, 4 units of 16 tokens,
    a = 100 each, b = 16 tokens * 1 layer * 6 B = 96 each, boundary 2 B per token -> 32 per
    recomputed chunk:
      (0,0)   compute 100 vs I/O 96   -> I/O takes unit 3        t_io  96
      (0,96)  100 vs 192              -> compute takes unit 0    t_c 100, t_io 96 + 32 = 128
      (100,128) 200 vs 224            -> compute takes unit 1    t_c 200, t_io 160
      (200,160) 300 vs 256            -> I/O takes unit 2        t_io 256
    Without the term the fourth step is the same but the channel ends at 192."""
    cm = P.CostModel(f_c=4, alpha=6, beta=0, f_io=0, gamma=1 << 20)
    o = P.PlanOpts(16, 0, 3, 2, P.TOKEN_WISE, boundary_bytes_per_token=2)
    assert P.boundary_costs(cm, o, 40, P.TOKEN_WISE) == [32, 32, 16]
    assert P.boundary_costs(cm, o, 40, P.LAYER_WISE) == [80, 0, 0]
    odd = P.CostModel(f_c=4, alpha=6, beta=0, f_io=9, gamma=(1 << 20) + 1)
    assert P.boundary_costs(odd, o, 40, P.TOKEN_WISE) == [33, 33, 17]     # ceil, no f_io
    assert P.boundary_costs(cm, P.PlanOpts(16, 0, 3, 2, P.TOKEN_WISE), 40, P.TOKEN_WISE) == [0, 0, 0]
    a, b, _ = P.unit_costs(P.CostModel(f_c=0, alpha=0, beta=0, f_io=0, gamma=1 << 20), o, 64, P.TOKEN_WISE)
    assert b == [96] * 4
    # a = 100 per unit: f_c = 100 with ONE layer; b = 16 tokens * 1 layer * 6 B = 96
    cm1 = P.CostModel(f_c=100, alpha=0, beta=0, f_io=0, gamma=1 << 20)
    o1 = P.PlanOpts(16, 0, 1, 6, P.TOKEN_WISE, boundary_bytes_per_token=2)
    trace = []
    splits, st = P.plan(cm1, o1, [64], trace)
    assert trace == [(1, 0, 3), (0, 0, 0), (0, 0, 1), (1, 0, 2)]
    assert splits == [(P.TOKEN_WISE, 32, 1)] and (st["t_comp"], st["t_io"]) == (200, 256)
    assert P.split_times(cm1, o1, [64], [2]) == (200, 256)
    assert P.split_times(cm1, o1, [64], [4]) == (400, 128)    # all recomputed: the rows still travel
    assert P.split_times(cm1, o1, [64], [0]) == (0, 384)
    o0 = P.PlanOpts(16, 0, 1, 6, P.TOKEN_WISE)
    splits, st = P.plan(cm1, o0, [64])
    assert splits == [(P.TOKEN_WISE, 32, 1)] and (st["t_comp"], st["t_io"]) == (200, 192)
    # layer-wise, 3 layers of 40 tokens: the first recomputed layer brings 80, the next nothing
    ol = P.PlanOpts(16, 0, 3, 2, P.LAYER_WISE, boundary_bytes_per_token=2)
    assert P.split_times(cm1, ol, [40], [1]) == (100, 2 * 80 + 80)
    assert P.split_times(cm1, ol, [40], [2]) == (200, 80 + 80)
    assert P.split_times(cm1, ol, [40], [3]) == (300, 80)


def test_boundary_rows_plans_are_consistent_and_near_brute_force():
    """The plan's clocks are those of its own splits; with boundary rows cheaper than the KV
    they replace (any stage of two layers or more at these sizes) the two-pointer schedule stays
    within one unit of the brute-force optimum; zero bytes change nothing."""
    rng = np.random.default_rng(29)
    n_equal = 0
    trials = 300
    for trial in range(trials):
        cm = rand_cm(rng, startups=trial % 3 == 0)
        L = int(rng.integers(2, 5))
        kvb = int(rng.choice([512, 4096]))
        bb = int(rng.integers(1, kvb * L)) if trial % 5 else 0
        opts = P.PlanOpts(32, int(rng.choice([0, 64, 10_000])), L, kvb, boundary_bytes_per_token=bb)
        n_ctx = [int(rng.integers(1, 32 * 5)) for _ in range(int(rng.integers(1, 4)))]
        splits, st = P.plan(cm, opts, n_ctx)
        units = [(-(-k // 32) if m == P.TOKEN_WISE else c) for (m, k, c) in splits]
        assert P.split_times(cm, opts, n_ctx, units) == (st["t_comp"], st["t_io"]), (trial, n_ctx)
        if bb == 0:
            o0 = P.PlanOpts(32, opts.l_delta, L, kvb)
            assert P.plan(cm, o0, n_ctx) == (splits, st)
        best, _ = P.brute_force(cm, opts, n_ctx)
        worst = 0
        for n in n_ctx:
            mode = P.request_mode(opts, n)
            a, b, _ = P.unit_costs(cm, opts, n, mode)
            worst = max(worst, max(a), max(b) + max(P.boundary_costs(cm, opts, n, mode)))
        assert best <= st["makespan"] <= best + worst, (trial, n_ctx, cm, opts)
        n_equal += st["makespan"] == best
    assert n_equal > trials // 5


def test_tiny_batches_shared_model_full_chunks_match_brute_force():
    rng = np.random.default_rng(22)
    for trial in range(400):
        cm = rand_cm(rng, overheads=False)
        c = 64
        opts = P.PlanOpts(c, 0, 4, 4096, P.TOKEN_WISE)
        n_ctx = [c * int(rng.integers(1, 7)) for _ in range(int(rng.integers(1, 5)))]
        _, st = P.plan(cm, opts, n_ctx)
        best, _ = P.brute_force(cm, opts, n_ctx)
        # one shared cost model, full chunks, equal I/O unit cost: compute takes the
        # cheapest units first and I/O the dearest first, so the batch behaves as one
        # global two-pointer and the schedule is optimal
        assert st["makespan"] == best, (trial, n_ctx, cm)


def test_tiny_batches_general_are_within_one_unit_of_brute_force():
    rng = np.random.default_rng(23)
    n_equal = 0
    trials = 300
    for trial in range(trials):
        cm = rand_cm(rng)
        opts = P.PlanOpts(32, int(rng.choice([0, 64, 10_000])), 3, 4096)
        n_ctx = [int(rng.integers(1, 32 * 5)) for _ in range(int(rng.integers(1, 5)))]
        splits, st = P.plan(cm, opts, n_ctx)
        best, _ = P.brute_force(cm, opts, n_ctx)
        worst_unit = 0
        for n in n_ctx:
            a, b, _ = P.unit_costs(cm, opts, n, P.request_mode(opts, n))
            worst_unit = max(worst_unit, max(a), max(b))
        assert best <= st["makespan"] <= best + worst_unit, (trial, n_ctx, cm)
        n_equal += st["makespan"] == best
    assert n_equal > trials // 4


# ------------------------------------------------------------ structure of plans
def _check_structure(cm, opts, n_ctx):
    trace = []
    splits, st = P.plan(cm, opts, n_ctx, trace=trace)
    claimed = {}
    for eng, i, u in trace:
        assert (i, u) not in claimed                          # every unit claimed once
        claimed[(i, u)] = eng
    for i, n in enumerate(n_ctx):
        mode = P.request_mode(opts, n)
        m = len(P.unit_costs(cm, opts, n, mode)[0])
        engines = [claimed[(i, u)] for u in range(m)]         # ... and every unit is claimed
        assert engines == sorted(engines)                     # recomputed prefix, loaded suffix
        n_comp = engines.count(0)
        assert splits[i][0] == mode
        if mode == P.TOKEN_WISE:
            assert splits[i][1] == min(n_comp * opts.chunk_tokens, n) and splits[i][2] == opts.n_layers
        else:
            assert splits[i][1] == n and splits[i][2] == n_comp
    t_c, t_io = P.split_times(cm, opts, n_ctx,
                              [sum(1 for (j, u), e in claimed.items() if j == i and e == 0)
                               for i in range(len(n_ctx))])
    assert (t_c, t_io) == (st["t_comp"], st["t_io"])
    all_c = P.split_times(cm, opts, n_ctx, [10 ** 9] * len(n_ctx))[0]
    all_io = P.split_times(cm, opts, n_ctx, [0] * len(n_ctx))[1]
    assert st["makespan"] <= min(all_c, all_io) or min(all_c, all_io) == 0
    return splits, st, trace


def test_structure_on_random_batches():
    rng = np.random.default_rng(24)
    for _ in range(200):
        cm = rand_cm(rng)
        opts = P.PlanOpts(64, int(rng.choice([0, 256, 100_000])), int(rng.integers(1, 12)), 4096,
                          io_key=int(rng.integers(0, 3)))
        n_ctx = [int(rng.integers(0, 2000)) for _ in range(int(rng.integers(1, 9)))]
        _check_structure(cm, opts, n_ctx)


def test_structure_on_benchmark_shaped_batch():
    from workloads import make_batch
    b = make_batch("cfg4")
    opts = P.PlanOpts(512, 2048, 32, 4096)
    splits, st, _ = _check_structure(cm_of("mi355x_like"), opts, b.n_ctx)
    assert any(s[0] == P.LAYER_WISE for s in splits) and any(s[0] == P.TOKEN_WISE for s in splits)


def test_io_goes_to_the_request_with_most_remaining_recompute():
    cm = cm_of("balanced")
    opts = P.PlanOpts(512, 0, 32, 4096, P.TOKEN_WISE)
    trace = []
    P.plan(cm, opts, [2048, 16384, 4096], trace=trace)
    first_io = next(t for t in trace if t[0] == 1)
    assert first_io[1:] == (1, 31)                            # longest request, its last chunk
    # I/O claims first under a fast link, with both requests untouched: the
    # tie on remaining cost and on length goes to the lower index
    trace = []
    P.plan(cm_of("mi355x_like"), opts, [4096, 4096], trace=trace)
    assert trace[0] == (1, 0, 7)
    # after compute took chunk 0 of request 0, request 1 has more left to recompute
    trace = []
    P.plan(cm, opts, [4096, 4096], trace=trace)
    assert trace[0] == (0, 0, 0) and next(t for t in trace if t[0] == 1)[1] == 1


def test_slower_io_never_shrinks_the_recomputed_part():
    rng = np.random.default_rng(25)
    for _ in range(60):
        cm = rand_cm(rng)
        opts = P.PlanOpts(64, 0, 4, 4096, P.TOKEN_WISE)
        n = [int(rng.integers(64, 3000))]
        k_prev = -1
        for scale in (1, 2, 4, 8, 16):
            cm2 = P.CostModel(cm.f_c, cm.alpha, cm.beta, cm.f_io * scale, cm.gamma * scale)
            k = P.plan(cm2, opts, n)[0][0][1]
            assert k >= k_prev
            k_prev = k


def test_degenerate_inputs():
    cm = cm_of("balanced")
    opts = P.PlanOpts(512, 0, 32, 4096)
    splits, st = P.plan(cm, opts, [])
    assert splits == [] and st["makespan"] == 0
    splits, st = P.plan(cm, opts, [0, 5])
    assert splits[0] == (P.TOKEN_WISE, 0, 32) and st["n_claims"] == 1
    assert splits[1][1] in (0, 5)


def test_l_delta_is_the_first_grid_point_where_token_wise_wins():
    cm = cm_of("balanced")
    opts = P.PlanOpts(512, 0, 32, 4096)
    ld = P.derive_l_delta(cm, opts, 32768)
    assert ld % 512 == 0 and 512 < ld <= 32768

    def j(n, mode):
        return P.plan(cm, P.PlanOpts(512, 0, 32, 4096, mode), [n])[1]["makespan"]
    assert j(ld, P.TOKEN_WISE) <= j(ld, P.LAYER_WISE)
    for n in range(512, ld, 512):
        assert j(n, P.TOKEN_WISE) > j(n, P.LAYER_WISE)


def test_baseline_plans():
    opts = P.PlanOpts(512, 0, 32, 4096)
    assert P.all_recompute(opts, [5, 7]) == [(0, 5, 32), (0, 7, 32)]
    assert P.all_load(opts, [5, 7]) == [(0, 0, 32), (0, 0, 32)]


# ------------------------------------------------ run-time scheduling (Sec. 3.3)
def test_dynamic_claim_hand_cases():
    # uniform costs: one token-wise request of 4 chunks, a = 2048 * alpha-ish each, b fixed
    cm = P.CostModel(f_c=0, alpha=10, beta=0, f_io=0, gamma=1 << 20)     # a = L*10*t, b = bytes
    opts = P.PlanOpts(16, 0, 2, 1, P.TOKEN_WISE)                         # unit: 16 tokens, 2 layers
    a, b, _ = P.unit_costs(cm, opts, 64, P.TOKEN_WISE)
    assert a == [320] * 4 and b == [32] * 4
    # the channel alone needs 4*32 = 128 < 320: compute takes nothing
    assert P.dynamic_claim(cm, opts, [64], [0], [3]) == ([0], 0)
    # with a backlog of 192 the channel needs 320: a step of 320 ends no later -> taken
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=192) == ([1], 320)
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=191) == ([0], 0)
    # loads that turn out 3x slower than modelled tip the same state over
    assert P.dynamic_claim(cm, opts, [64], [0], [3], scale_io=3000) == ([1], 320)
    # two requests: each unit taken shortens what is left to the channel, the second does not fit
    take, a_sum = P.dynamic_claim(cm, opts, [64, 64], [0, 0], [3, 3], io_backlog=100)
    assert (take, a_sum) == ([1, 0], 320)       # R = 100 + 256; 320 <= 356, then 640 > 356 - 32
    # a finished request is never a candidate
    assert P.dynamic_claim(cm, opts, [64, 64], [4, 0], [3, 3], io_backlog=10 ** 6)[0] == [0, 1]
    # work the step carries anyway counts against what it can take on top
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=192, step_fixed=1) == ([0], 1)
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=200, step_fixed=8) == ([1], 328)
    # so does work that waits for the compute engine after the step, without lengthening the step
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=200, compute_later=8) == ([1], 320)
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=200, compute_later=9) == ([0], 0)


def test_dynamic_claim_step_cap_and_shortest_first_order():
    cm = P.CostModel(f_c=0, alpha=10, beta=0, f_io=0, gamma=1 << 20)
    opts = P.PlanOpts(16, 0, 2, 1, P.TOKEN_WISE)            # a = 320, b = 32 per full chunk
    n = [64, 32, 48]                                        # 4, 2 and 3 chunks
    big = 10 ** 6
    # no cap: every live request's next chunk goes into the step
    assert P.dynamic_claim(cm, opts, n, [0, 0, 0], [3, 1, 2], io_backlog=big) == ([1, 1, 1], 960)
    # capped at one chunk's worth: the step stops after its first candidate -- by index under
    # the cost-ratio order (all equal here), the request with least ahead of it under the other
    assert P.dynamic_claim(cm, opts, n, [0, 0, 0], [3, 1, 2], io_backlog=big, step_cap=320) == ([1, 0, 0], 320)
    assert P.dynamic_claim(cm, opts, n, [0, 0, 0], [3, 1, 2], io_backlog=big, step_cap=320,
                           order=P.ORDER_SHORTEST) == ([0, 1, 0], 320)
    assert P.dynamic_claim(cm, opts, n, [0, 0, 0], [3, 1, 2], io_backlog=big, step_cap=321,
                           order=P.ORDER_SHORTEST) == ([0, 1, 1], 640)
    # the cap never starves a step: work it carries anyway does not count as its first unit
    assert P.dynamic_claim(cm, opts, n, [0, 0, 0], [3, 1, 2], io_backlog=big, step_fixed=500,
                           step_cap=320)[0] == [1, 0, 0]
    # shortest first finishes requests one after the other
    pc, pio = [0, 0, 0], [3, 1, 2]
    finished = []
    for _ in range(9):
        take, _ = P.dynamic_claim(cm, opts, n, pc, pio, io_backlog=big, step_cap=320, order=P.ORDER_SHORTEST)
        i = take.index(1)
        pc[i] += 1
        if pc[i] > pio[i]:
            finished.append(i)
    assert finished == [1, 2, 0]


def test_dynamic_claim_several_chunks_of_a_request_and_units_given_back_hand_cases():
    """Hand values for the two later parts of the rule: a step may hold consecutive chunks of one
    request, and what it chose is given back unless it pays for the contention it causes."""
    cm = P.CostModel(f_c=0, alpha=10, beta=1024, f_io=0, gamma=1 << 20)
    opts = P.PlanOpts(16, 0, 2, 1, P.TOKEN_WISE)             # unit: 16 tokens through 2 layers
    a, b, _ = P.unit_costs(cm, opts, 64, P.TOKEN_WISE)
    # chunk u costs 2 * (10 * 16 + 1024 * ceil(pairs / 1024)), pairs = 16 * 16u + 136 -> 1 block each
    assert a == [2368] * 4 and b == [32] * 4
    big = 10 ** 6
    # one unit per request (the default), two, no limit: the chunks are taken from the pointer on
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=big) == ([1], 2368)
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=big, max_units=2) == ([2], 4736)
    assert P.dynamic_claim(cm, opts, [64], [1], [3], io_backlog=big, max_units=0) == ([3], 7104)
    # the test runs unit by unit: R = 5000 + 4 * 32 = 5128; 2368 <= 5128; 4736 <= 5128 - 32;
    # 7104 > 5128 - 64
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=5000, max_units=0) == ([2], 4736)
    # two requests, the cheaper ratio first: request 1's chunks are short (8 tokens: a = 2 * (80 +
    # 1024) = 2208, b = 16; 2208 / 16 > 2368 / 32), so request 0 is walked to its end first
    n2 = [64, 8]
    a1, b1, _ = P.unit_costs(cm, opts, 8, P.TOKEN_WISE)
    assert a1 == [2208] and b1 == [16]
    assert P.dynamic_claim(cm, opts, n2, [0, 0], [3, 0], io_backlog=big, max_units=0) == ([4, 1], 4 * 2368 + 2208)
    assert P.dynamic_claim(cm, opts, n2, [0, 0], [3, 0], io_backlog=big, max_units=0, step_cap=4736) == ([2, 0], 4736)
    # a cap reached inside a request stops the whole step, the other request is not started
    assert P.dynamic_claim(cm, opts, n2, [0, 0], [3, 0], io_backlog=big, max_units=3, step_cap=4737)[0] == [3, 0]
    # contention.  Beside a recomputing engine the channel runs at scale 2000, alone at 1000:
    # R = 5000 + 4 * 64 = 5256 beside, R_alone = 5000 + 4 * 32 = 5128.  Two units are chosen
    # (2368 <= 5256, 4736 <= 5256 - 64, 7104 > 5256 - 128); with them the restoration ends at
    # max(4736, 5256 - 128) = 5128, not before the 5128 of the channel alone: given back
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=5000, scale_io=2000, max_units=0) == ([2], 4736)
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=5000, scale_io=2000, max_units=0,
                           io_alone=1000) == ([0], 0)
    # one picosecond less alone-time to beat is still a tie; a channel that is slower on its own
    # (scale 1032: R_alone = 5000 + 4 * 33 = 5132) is beaten by 5128 and the units stay
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=5000, scale_io=2000, max_units=0,
                           io_alone=1032) == ([2], 4736)
    # work that waits after the step counts on both sides: 4736 + 400 = 5136 > 5132 loses ...
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=5000, scale_io=2000, max_units=0,
                           io_alone=1032, compute_later=400) == ([0], 0)
    # A capped step is the first of several: whether recomputing pays is judged on everything
    # the engine would take (the two units above), not on the one unit the cap lets through --
    # which by itself, max(2368, 5256 - 64) = 5192, would not beat the 5132 of the channel alone
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=5000, scale_io=2000, max_units=0,
                           io_alone=1032, step_cap=2368) == ([1], 2368)
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=5000, scale_io=2000, max_units=1,
                           io_alone=1032) == ([1], 2368)
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=5000, scale_io=2000, max_units=1,
                           io_alone=1000) == ([0], 0)
    # ... and the step's fixed work is reported when the units are given back
    assert P.dynamic_claim(cm, opts, [64], [0], [3], io_backlog=5000, scale_io=2000, max_units=0,
                           io_alone=1000, step_fixed=7) == ([0], 7)


def test_dynamic_claim_layer_wise_group_and_last_layer_mark():
    cm = P.CostModel(f_c=0, alpha=10, beta=0, f_io=0, gamma=1 << 20)
    opts = P.PlanOpts(16, 0, 4, 1, P.LAYER_WISE)            # units: 4 layers over all tokens
    n = [32, 16]                                            # a per layer 320 / 160, b 32 / 16
    # plenty of backlog: the group takes layer 0 and expects to take layer 1 too
    assert P.dynamic_claim(cm, opts, n, [0, 0], [3, 3], io_backlog=10 ** 6) == ([1, 1], 480)
    # room for exactly one layer: R = 480 + 4*48 = 672; 480 <= 672, next 960 > 672 - 48
    assert P.dynamic_claim(cm, opts, n, [0, 0], [3, 3], io_backlog=480) == ([2, 2], 480)
    # the last unclaimed layer of the group is always marked as its last
    assert P.dynamic_claim(cm, opts, n, [3, 3], [3, 3], io_backlog=10 ** 6)[0] == [2, 2]
    # with a K/V-only price for a request's last layer (here 1/4 of the linear part): layer 0 is
    # priced 80 + 40, the step that runs it in full is reported at 320 + 160
    kvo = P.PlanOpts(16, 0, 4, 1, P.LAYER_WISE, kv_only_permille=250)
    assert P.dynamic_claim(cm, kvo, n, [0, 0], [3, 3], io_backlog=10 ** 6) == ([1, 1], 480)
    # ... and a last layer further up is priced in full (it completes the layer below) but runs
    # only its K/V projection
    assert P.dynamic_claim(cm, kvo, n, [3, 3], [3, 3], io_backlog=10 ** 6) == ([2, 2], 120)
    # closed requests are not offered to the compute engine, whatever the backlog
    assert P.dynamic_claim(cm, opts, n, [1, 1], [3, 3], closed=[True, True], io_backlog=10 ** 9) == ([0, 0], 0)


def test_io_pick_declines_when_compute_gets_there_first():
    cm = P.CostModel(f_c=0, alpha=10, beta=0, f_io=0, gamma=1 << 20)
    opts = P.PlanOpts(16, 0, 2, 1, P.TOKEN_WISE)            # a = 320, b = 32 per unit
    # longest remaining recomputation first (Sec. 3.3), ties to the longer context
    assert P.io_pick(cm, opts, [64, 128], [0, 0], [3, 7]) == 1
    assert P.io_pick(cm, opts, [64, 128], [0, 4], [3, 7]) == 1     # equal remaining: longer context
    assert P.io_pick(cm, opts, [64, 128], [0, 5], [3, 7]) == 0
    assert P.io_pick(cm, opts, [64, 128], [4, 8], [3, 7]) == -1    # nothing live
    # one unit left, costs 320 to recompute: the channel takes it unless its backlog is longer
    assert P.io_pick(cm, opts, [64], [3], [3], io_backlog=288) == 0
    assert P.io_pick(cm, opts, [64], [3], [3], io_backlog=289) == -1
    assert P.io_pick(cm, opts, [64], [3], [3], io_backlog=289, compute_busy=1) == 0
    assert P.io_pick(cm, opts, [64], [3], [3], closed=[True], io_backlog=10 ** 9) == 0
    # never both decline: whatever the state, with the compute engine idle one of them takes a unit
    rng = np.random.default_rng(7)
    for _ in range(300):
        cm = rand_cm(rng)
        mode = int(rng.integers(-1, 2))
        opts = P.PlanOpts(64, 600, 4, 4096, mode, kv_only_permille=int(rng.integers(0, 300)))
        n = [int(x) for x in rng.integers(1, 1500, size=int(rng.integers(1, 5)))]
        m = [len(P.unit_costs(cm, opts, x, P.request_mode(opts, x))[0]) for x in n]
        pc = [int(rng.integers(0, mi + 1)) for mi in m]
        pio = [int(rng.integers(pc[i] - 1, m[i])) for i in range(len(n))]
        if opts.force_mode != P.TOKEN_WISE:           # layer-wise requests share their pointers
            lw = [i for i in range(len(n)) if P.request_mode(opts, n[i]) == P.LAYER_WISE]
            for i in lw:
                pc[i], pio[i] = pc[lw[0]], max(pio[lw[0]], pc[lw[0]] - 1)
        if all(pc[i] > pio[i] for i in range(len(n))):
            continue
        backlog = int(rng.integers(0, 10 ** 10))
        sc, sio = int(rng.integers(250, 4001)), int(rng.integers(250, 4001))
        take, _ = P.dynamic_claim(cm, opts, n, pc, pio, None, backlog, sc, sio)
        pick = P.io_pick(cm, opts, n, pc, pio, None, backlog, 0, sc, sio)
        assert any(take) or pick >= 0


@pytest.mark.parametrize("kind", ["mi355x_like", "balanced", "slow_io", "uniform"])
@pytest.mark.parametrize("mode,n_ctx", [(P.TOKEN_WISE, [9000, 5000, 16000, 2100]),
                                        (P.LAYER_WISE, [4096, 3000, 1000]),
                                        (-1, [16384, 9000, 1500, 800])])
def test_simulated_run_time_scheduling_tracks_the_static_plan_and_adapts(kind, mode, n_ctx):
    cm = cm_of(kind)
    opts = P.PlanOpts(512, 2048, 32, 4096, mode, kv_only_permille=120)
    splits, st = P.plan(cm, opts, n_ctx)
    dsplits, makespan, n_steps = P.simulate_dynamic(cm, opts, n_ctx)
    for (m, k, c), n in zip(dsplits, n_ctx):              # a valid split for every request
        assert 0 <= k <= n and 0 <= c <= 32 and (k == n if m == P.LAYER_WISE else c == 32)
    # the world behaves as modelled: deciding at run time costs at most a few percent
    assert makespan <= 1.03 * st["makespan"]
    # compute really runs 1.5x slower than modelled: the static split is stuck with its plan,
    # the run-time scheduler sees the slow steps and leaves more to the channel
    slow = P.CostModel(cm.f_c * 3 // 2, cm.alpha * 3 // 2, cm.beta * 3 // 2, cm.f_io, cm.gamma)
    units = [(-(-k // 512) if m == P.TOKEN_WISE else c) for m, k, c in splits]
    t_c, t_io = P.split_times(slow, opts, n_ctx, units, [s[0] for s in splits])
    _, makespan_slow, _ = P.simulate_dynamic(cm, opts, n_ctx, true_cm=slow)
    assert makespan_slow <= max(t_c, t_io)
    # and it never does worse than the better of the two extremes by more than one step
    all_io = sum(sum(P.unit_costs(slow, opts, n, P.request_mode(opts, n))[1]) for n in n_ctx)
    assert makespan_slow <= 1.05 * all_io
    # short steps that finish the short requests first: a different order of the same work
    _, capped, n_capped = P.simulate_dynamic(cm, opts, n_ctx, step_cap=st["makespan"] // 20,
                                             order=P.ORDER_SHORTEST)
    assert capped <= 1.06 * st["makespan"] and n_capped >= n_steps


def test_simulated_run_time_scheduling_against_brute_force():
    rng = np.random.default_rng(31)
    for _ in range(25):
        cm = rand_cm(rng, overheads=False)
        opts = P.PlanOpts(64, 0, 3, 4096, P.TOKEN_WISE)
        n_ctx = [int(x) for x in rng.integers(64, 400, size=2)]
        best, _ = P.brute_force(cm, opts, n_ctx)
        _, makespan, _ = P.simulate_dynamic(cm, opts, n_ctx, lookahead=0)
        costs = [P.unit_costs(cm, opts, n, P.TOKEN_WISE) for n in n_ctx]
        biggest = max(max(a + b) for a, b, _ in costs)
        # list scheduling: within one (largest) unit per engine of the optimum
        assert makespan <= best + 2 * biggest


def test_sweep_batches_are_what_their_name_says():
    from workloads import make_batch
    b = make_batch("sweep:4:2048:1")
    assert b.n_ctx == [2048] * 4 and b.n_new == [128] * 4 and b.forced_mode == 1 and b.shape.name == "8b"
    assert all(len(t) == 2048 and t.max() < b.shape.vocab for t in b.ctx_tokens)
    assert make_batch("sweep:1:512").forced_mode == -1
    # seeded: the same name gives the same tokens
    assert np.array_equal(make_batch("sweep:4:2048:1").ctx_tokens[3], b.ctx_tokens[3])


# ------------------------------------------------------------------ feedback and policy pins
def test_cost_feedback_hand_values():
    """Ratios measured/predicted scale each side; clamped to [1/4, 4]; round to nearest; alpha
    and gamma never drop below 1; a side with no prediction or no measurement is left alone."""
    cm = P.CostModel(f_c=7, alpha=1000, beta=10, f_io=9, gamma=2000, s_c=500, s_io=100)
    out = P.cost_feedback(cm, 1_000_000, 1_200_000, 5_000, 5_000)           # compute 20 % slower
    assert (out.f_c, out.alpha, out.beta, out.s_c) == (8, 1200, 12, 600)     # 7 * 1.2 = 8.4 -> 8
    assert (out.f_io, out.gamma, out.s_io) == (9, 2000, 100)
    out = P.cost_feedback(cm, 1_000, 9_000, 1_000, 100)                      # 9x and 0.1x: clamped
    assert (out.f_c, out.alpha, out.beta, out.s_c) == (28, 4000, 40, 2000)
    assert (out.f_io, out.gamma, out.s_io) == (2, 500, 25)                   # 9/4 = 2.25 -> 2
    out = P.cost_feedback(cm, 2, 3, 2, 3)                                    # 1.5x: halves round up
    assert (out.f_c, out.alpha, out.beta, out.s_c) == (11, 1500, 15, 750)    # 10.5 -> 11
    tiny = P.CostModel(0, 1, 0, 0, 3, 0, 0)
    out = P.cost_feedback(tiny, 4, 1, 4, 1)                                  # a quarter of 1 and of 3
    assert (out.alpha, out.gamma) == (1, 1)
    out = P.cost_feedback(cm, 0, 5, 7, 0)
    assert out == cm


def test_prefill_cost_hand_value():
    """16 new tokens from position 2048 through 2 layers: 16*2048 + 16*17/2 = 32904 pairs =
    33 blocks of 1024 -> per layer 10 + 3*16 + 1000*33 = 33058."""
    cm = P.CostModel(f_c=10, alpha=3, beta=1000, f_io=0, gamma=1)
    assert P.prefill_cost(cm, 2, [2048], [16]) == 66116
    assert P.prefill_cost(cm, 2, [2048, 77], [16, 0]) == 66116              # no new turn, no cost
    assert P.prefill_cost(cm, 2, [0], [1]) == 2 * (10 + 3 + 1000)            # one pair


# A model small enough to price by hand: 2 layers, d 16, 2 query heads / 1 KV head of 8, FFN 16,
# 2-byte elements.  K/V-projection share: 2*16*(2+2)*8 = 1024 of 1024 + 2*2*8*16 + 6*16*16 =
# 3072 linear FLOPs -> 333 permille.  KV bytes per token and layer: 2*1*8*2 = 32.
HAND_MODEL = (2, 16, 2, 1, 8, 16, 2)
# alpha 1000 ps per token and layer, nothing else on the compute side; gamma = 20 * 2^20, i.e.
# 20 ps per byte.  One request of 64 tokens, chunks of 16: four units, each
#   a = 1 full layer (16000) + the top layer's K/V share ceil(1000*333*16/1000) = 5328 -> 21328
#   b = 16 tokens * 2 layers * 32 B * 20 = 20480
HAND_COST = P.CostModel(f_c=0, alpha=1000, beta=0, f_io=0, gamma=20 << 20)


def test_policy_kv_share_of_the_8b_layer():
    # 2*4096*6144 of 436207616 linear FLOPs = 11.54 %
    assert P.kv_share_permille(4096, 32, 8, 128, 14336) == 115
    assert P.kv_share_permille(16, 2, 1, 8, 16) == 333


def test_policy_hybrid_without_contention_and_all_load_under_heavy_contention():
    """No new turn.  Isolated costs: I/O takes unit 3 (20480 < 21328), compute unit 0, I/O unit 2
    (40960 < 42656), compute unit 1: k = 32, t_comp 42656, t_io 40960 -- against 81920 for
    loading everything and 85312 for recomputing everything.  With both engines twice as slow
    side by side the same hybrid ends at 85312 and loses to loading everything."""
    splits, info = P.plan_batch(HAND_COST, (1000, 1000), HAND_MODEL, 16, 0, 0, 0, True, [64])
    assert splits == [(0, 32, 2)]
    assert info["kind"] == P.PLAN_HYBRID and info["kv_only_permille"] == 333
    assert (info["t_comp"], info["t_io"], info["ttft"]) == (42656, 40960, 42656)
    assert (info["ttft_hybrid"], info["ttft_all_load"], info["ttft_all_recompute"]) == (42656, 81920, 85312)
    # contention 1.5x: a = 31992, b = 30720 -> t_comp 63984: still ahead of 81920
    splits, info = P.plan_batch(HAND_COST, (1500, 1500), HAND_MODEL, 16, 0, 0, 0, True, [64])
    assert splits == [(0, 32, 2)] and info["kind"] == P.PLAN_HYBRID and info["ttft"] == 63984
    splits, info = P.plan_batch(HAND_COST, (2000, 2000), HAND_MODEL, 16, 0, 0, 0, True, [64])
    assert splits == [(0, 0, 2)]
    assert info["kind"] == P.PLAN_ALL_LOAD and info["ttft_hybrid"] == 85312 and info["ttft"] == 81920
    assert (info["t_comp"], info["t_io"]) == (0, 81920)
    # contention on the compute side only can make recomputing everything the plan when loads are dear
    dear = P.CostModel(0, 1000, 0, 0, 200 << 20)             # b = 204800 per unit
    splits, info = P.plan_batch(dear, (1000, 1000), HAND_MODEL, 16, 0, 0, 0, True, [64])
    assert splits == [(0, 64, 2)] and info["kind"] == P.PLAN_ALL_RECOMPUTE and info["ttft"] == 85312


def test_policy_new_turn_on_the_compute_clock():
    """16 new tokens behind the 64: prefill = 2 layers * 16 * 1000 = 32000.  Pipelined join: the
    compute clock starts there, so I/O takes units 3 and 2 (20480, 40960 < 53328), compute unit 0
    (53328 < 61440), I/O unit 1 (61440 < 74656): k = 16; one layer of the new turn (16000) is
    left when the last load lands -> 77440.  Sequential join: the plan of the test above, then
    the new turn as a pass of its own: 42656 + 32000."""
    splits, info = P.plan_batch(HAND_COST, (1000, 1000), HAND_MODEL, 16, 0, 0, 0, True, [64], [16])
    assert splits == [(0, 16, 2)] and info["kind"] == P.PLAN_HYBRID and info["prefill_ps"] == 32000
    assert (info["t_comp"], info["t_io"], info["ttft"]) == (53328, 61440, 77440)
    assert (info["ttft_all_load"], info["ttft_all_recompute"]) == (97920, 117312)
    splits, info = P.plan_batch(HAND_COST, (1000, 1000), HAND_MODEL, 16, 0, 0, 0, False, [64], [16])
    assert splits == [(0, 32, 2)]
    assert (info["t_comp"], info["t_io"], info["ttft"]) == (42656, 40960, 74656)
    assert (info["ttft_all_load"], info["ttft_all_recompute"]) == (113920, 117312)
    # a start-up of 1000 is paid once by a pipelined pass, twice when the new turn runs on its own
    su = P.CostModel(0, 1000, 0, 0, 20 << 20, s_c=1000)
    _, info = P.plan_batch(su, (1000, 1000), HAND_MODEL, 16, 0, 0, 0, True, [64], [16])
    assert info["ttft_all_recompute"] == 1000 + 85312 + 32000
    _, info = P.plan_batch(su, (1000, 1000), HAND_MODEL, 16, 0, 0, 0, False, [64], [16])
    assert info["ttft_all_recompute"] == (1000 + 85312) + (1000 + 32000)
    # a pipeline stage of one of the two layers: half the start-up, no new turn of its own
    _, info = P.plan_batch(su, (1000, 1000), HAND_MODEL, 16, 0, 0, 0, True, [64], [16], stage_layers=1)
    assert info["prefill_ps"] == 0 and info["ttft_all_recompute"] == 500 + 4 * 5328
    # the same stage as the model's SECOND layer recomputes from float32 boundary rows (64 B per
    # token, 16 * 64 * 20 = 20480 per chunk) over the link its KV (10240 per chunk) would take:
    # every recomputed chunk costs the channel twice what loading it would, so recompute always
    # wins the next claim, the channel ends at 4 * 20480, and loading everything (40960) is chosen
    sp, info = P.plan_batch(su, (1000, 1000), HAND_MODEL, 16, 0, 0, 0, True, [64], [16], stage_layers=1,
                            stage_first_layer=1)
    assert info["ttft_all_recompute"] == 81920 and info["ttft_hybrid"] == 81920
    assert info["kind"] == P.PLAN_ALL_LOAD and info["ttft"] == 40960 and sp == [(0, 0, 1)]


def test_policy_feedback_hand_values():
    info = dict(kind=P.PLAN_HYBRID, pipelined_join=1, t_comp=53328, t_io=61440)
    # the call ended well after the copy stream: its end is the compute measurement
    cm, ov = P.plan_feedback(HAND_COST, (1000, 1000), info, 60000, 61440, 64000)
    assert cm == HAND_COST and ov == (1200, 1000)            # 64000 / 53328 = 1.2001
    # ... not with the sequential join, and not when both streams ended together
    _, ov = P.plan_feedback(HAND_COST, (1000, 1000), dict(info, pipelined_join=0), 60000, 61440, 64000)
    assert ov == (1125, 1000)                                 # 60000 / 53328 = 1.1251
    _, ov = P.plan_feedback(HAND_COST, (1000, 1000), info, 60000, 61440, 62000)
    assert ov == (1125, 1000)
    # time the compute stream stood waiting for loads is taken off: (64000 - 10672) / 53328 = 1
    _, ov = P.plan_feedback(HAND_COST, (1000, 1000), info, 60000, 61440, 64000, 10672)
    assert ov == (1000, 1000)
    # one batch moves a factor by 5/4 or 4/5 at most (80000 / 53328 = 1.5: taken as 1.25) ...
    _, ov = P.plan_feedback(HAND_COST, (1000, 1000), info, 60000, 61440, 80000)
    assert ov == (1250, 1000)
    _, ov = P.plan_feedback(HAND_COST, (1100, 1000), info, 30000, 30720, 30000)
    assert ov == (880, 800)
    # ... and the factors stay in [500, 8000]
    _, ov = P.plan_feedback(HAND_COST, (7000, 3000), info, 533280, 614400, 533280)
    assert ov == (8000, 3750)
    _, ov = P.plan_feedback(HAND_COST, (600, 1000), info, 53, 61, 53)
    assert ov == (500, 800)
    # an extreme corrects the coefficients of the engine that ran alone
    cm, ov = P.plan_feedback(HAND_COST, (1200, 1300), dict(kind=P.PLAN_ALL_LOAD, pipelined_join=1, t_comp=0, t_io=81920),
                             0, 98304, 98304)
    assert ov == (1150, 1225) and cm.gamma == (20 << 20) * 6 // 5 and cm.alpha == 1000     # 200/4, 300/4 back
    cm, ov = P.plan_feedback(HAND_COST, (1200, 1300), dict(kind=P.PLAN_ALL_RECOMPUTE, pipelined_join=1, t_comp=85312, t_io=0),
                             85312, 0, 127968)
    assert cm.alpha == 1500 and cm.gamma == 20 << 20 and ov == (1150, 1225)
    _, ov = P.plan_feedback(HAND_COST, (600, 1000), dict(kind=P.PLAN_ALL_LOAD, pipelined_join=1, t_comp=0, t_io=81920),
                            0, 81920, 81920)
    assert ov == (700, 1000)


def test_simulated_run_time_scheduling_hand_traces():
    """Two runs of the event-driven simulator traced by hand (true costs = the model's, so every
    ratio measured/predicted stays 1000).
    (1) One token-wise request of four 16-token chunks, recompute 32 per chunk, load 24 (units
    of 10^6 ps).  t=0: the channel takes chunk 3 (0+24 <= 128 of recompute left) and chunk 2
    (24+24 <= 96), declines chunk 1 (48+24 > 64); compute takes chunk 0 (32 <= 48 backlog + 48
    unclaimed loads).  t=24: chunk 3 has landed; the channel declines chunk 1 again (24+24 > 8
    left of the step + 32).  t=32: compute takes chunk 1 (32 <= 24 + 24).  t=48: chunk 2 has
    landed.  t=64: done -- the split and the makespan of the static plan.
    (2) Two layer-wise requests (32 and 16 tokens, 3 layers), loaded and recomputed as a group:
    per layer recompute 32+16 = 48, load 24+12 = 36.  t=0: the channel takes layer 2 (36 <= 144)
    and layer 1 (36+36 <= 96), declines layer 0 (72+36 > 48); compute takes layer 0 of the group
    (48 <= 72 + 36) as its last layer (there is no layer left to go on to): both requests are
    closed with cut 1.  Loads land at 36 and 72: makespan 72."""
    M = 1_000_000
    cm = P.CostModel(f_c=0, alpha=M, beta=0, f_io=0, gamma=1_536 * M)        # 24 M per 16 tokens x 2 x 512 B
    opts = P.PlanOpts(chunk_tokens=16, l_delta=0, n_layers=2, kv_bytes_per_token_layer=512, force_mode=P.TOKEN_WISE)
    assert P.unit_costs(cm, opts, 64, P.TOKEN_WISE)[:2] == ([32 * M] * 4, [24 * M] * 4)
    tr = []
    splits, makespan, n_steps = P.simulate_dynamic(cm, opts, [64], trace=tr)
    assert tr == [(0, 1, 0, 3), (0, 1, 0, 2), (0, 0, 0, 0), (32 * M, 0, 0, 1)]
    assert (splits, makespan, n_steps) == ([(P.TOKEN_WISE, 32, 2)], 64 * M, 2)
    assert P.plan(cm, opts, [64])[0] == splits and P.plan(cm, opts, [64])[1]["makespan"] == makespan
    opts = P.PlanOpts(chunk_tokens=16, l_delta=0, n_layers=3, kv_bytes_per_token_layer=512, force_mode=P.LAYER_WISE)
    assert P.unit_costs(cm, opts, 32, P.LAYER_WISE)[:2] == ([32 * M] * 3, [24 * M] * 3)
    assert P.unit_costs(cm, opts, 16, P.LAYER_WISE)[:2] == ([16 * M] * 3, [12 * M] * 3)
    tr = []
    splits, makespan, n_steps = P.simulate_dynamic(cm, opts, [32, 16], trace=tr)
    assert tr == [(0, 1, 0, 2), (0, 1, 0, 1), (0, 0, 0, 0)]
    assert (splits, makespan, n_steps) == ([(P.LAYER_WISE, 32, 1), (P.LAYER_WISE, 16, 1)], 72 * M, 1)
    # a slower channel (48 per chunk) still takes chunks 3 and 2 at t=0 (48+48 <= 96, the test is
    # "no later than"), compute chunks 0 and 1 (32 <= 96 + 96, then 32 <= 96 + 48); the loads
    # land at 48 and 96: the channel, not compute, ends the restoration
    slow = P.CostModel(0, M, 0, 0, 3_072 * M)
    opts = P.PlanOpts(16, 0, 2, 512, P.TOKEN_WISE)
    tr = []
    splits, makespan, n_steps = P.simulate_dynamic(slow, opts, [64], trace=tr)
    assert tr == [(0, 1, 0, 3), (0, 1, 0, 2), (0, 0, 0, 0), (32 * M, 0, 0, 1)]
    assert (splits, makespan, n_steps) == ([(P.TOKEN_WISE, 32, 2)], 96 * M, 2)
