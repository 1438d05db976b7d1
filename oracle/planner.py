"""Oracle: batch-aware two-pointer restoration scheduler (Algorithm 1,
Sec. 3.3) over an integer cost model, its brute-force optimum, and the
strategy threshold L_delta (Sec. 3.1).

TEST INFRASTRUCTURE ONLY (see package docstring).  Pure Python integers.

Units (Sec. 3.1).  A token-wise request of n tokens has M = ceil(n / C)
units; unit u is the chunk of tokens [u*C, min((u+1)*C, n)) through all L
layers.  A layer-wise request has M = L units; unit u is layer u over all n
tokens.  A request is token-wise iff n >= L_delta (Algorithm 1, mode rule).
Pointers start at (0, M-1); compute walks up, I/O walks down.

Readings taken where the text leaves room (each is listed in the design
notes of this repository):
 * a request stays live while p_comp <= p_io, so the unit where the pointers
   meet is restored by exactly one engine (the text's "meet ... without
   redundant work"; the printed termination test would drop that unit when
   the unit count is odd);
 * the lock-step loop is simulated event-driven with one compute clock and one
   I/O clock (single source => one serial channel): at every step the compute
   candidate is the next live request in round-robin index order at its
   p_comp, the I/O candidate is the live request with the largest remaining
   recompute cost at its p_io (re-evaluated after every claim, the
   "progressive, chunk-level" update), and the engine whose candidate would
   finish earlier claims it; a tie goes to compute;
 * I/O priority ties go to the longer context, then to the lower index.
"""
from dataclasses import dataclass
from fractions import Fraction
from functools import cmp_to_key
from itertools import product

TOKEN_WISE = 0
LAYER_WISE = 1

KEY_REMAINING_COST = 0     # Sec. 3.3: "largest remaining recomputation cost"
KEY_REMAINING_CELLS = 1    # "(i.e., longest length to restore)"
KEY_MARGINAL = 2           # abstract: highest marginal reduction per I/O time


@dataclass
class CostModel:
    """All picoseconds.  Per layer of recompute over t tokens starting at
    position p0:  f_c + alpha*t + beta*ceil(pairs/1024)  with
    pairs = t*p0 + t*(t+1)/2 causal (query, key) pairs.  Per copied unit:
    f_io + ceil(bytes*gamma / 2^20).  An engine that does any work at all pays
    its start-up s_c / s_io once, before its first unit."""
    f_c: int
    alpha: int
    beta: int
    f_io: int
    gamma: int
    s_c: int = 0      # one-time start-up of the compute engine (clock starts here)
    s_io: int = 0     # one-time start-up of the I/O channel


@dataclass
class PlanOpts:
    chunk_tokens: int
    l_delta: int
    n_layers: int
    kv_bytes_per_token_layer: int
    force_mode: int = -1            # -1: by l_delta; 0 token-wise; 1 layer-wise
    io_key: int = KEY_REMAINING_COST
    kv_only_permille: int = 0       # > 0: the last recomputed layer of a request costs only
                                    # its K/V projection, this many permille of alpha*t
    boundary_bytes_per_token: int = 0   # > 0: a pipeline stage above layer 0 (Sec. 3.2) recomputes
                                    # from cached stage-input hidden states that cross the same
                                    # link as the KV: a recompute claim also costs the channel


def ceil_div(a, b):
    return -(-a // b)


def compute_cost(cm, n_layers, t, p0):
    pairs = t * p0 + t * (t + 1) // 2
    return n_layers * (cm.f_c + cm.alpha * t + cm.beta * ceil_div(pairs, 1024))


def kv_only_cost(cm, permille, t):
    """The last recomputed layer of a request stops after its K/V write (nothing downstream
    reads its attention or MLP output): fixed part plus a fraction of the linear part."""
    return cm.f_c + (cm.alpha * permille * t + 999) // 1000


def io_cost(cm, n_bytes):
    return cm.f_io + ceil_div(n_bytes * cm.gamma, 1 << 20)


def request_mode(opts, n):
    if opts.force_mode in (TOKEN_WISE, LAYER_WISE):
        return opts.force_mode
    return TOKEN_WISE if n >= opts.l_delta else LAYER_WISE


def unit_costs(cm, opts, n, mode):
    """(a[u], b[u], tokens[u]) for the M units of one request."""
    a, b, tok = [], [], []
    if n <= 0:
        return a, b, tok
    if mode == TOKEN_WISE:
        c = opts.chunk_tokens
        for u in range(ceil_div(n, c)):
            t = min((u + 1) * c, n) - u * c
            if opts.kv_only_permille > 0:
                # all layers but the top one in full, the top one K/V only
                a.append(compute_cost(cm, opts.n_layers - 1, t, u * c) +
                         kv_only_cost(cm, opts.kv_only_permille, t))
            else:
                a.append(compute_cost(cm, opts.n_layers, t, u * c))
            b.append(io_cost(cm, t * opts.n_layers * opts.kv_bytes_per_token_layer))
            tok.append(t)
    else:
        for l in range(opts.n_layers):
            # claiming layer l turns layer l-1 from K/V-only into a full layer and adds a
            # K/V-only layer l: the first layer costs K/V only, every further one a full layer
            if opts.kv_only_permille > 0 and l == 0:
                a.append(kv_only_cost(cm, opts.kv_only_permille, n))
            else:
                a.append(compute_cost(cm, 1, n, 0))
            b.append(io_cost(cm, n * opts.kv_bytes_per_token_layer))
            tok.append(n)
    return a, b, tok


def boundary_costs(cm, opts, n, mode):
    """c[u]: channel time a RECOMPUTE claim of unit u costs -- the boundary-activation rows of the
    tokens it recomputes, ceil(tokens * bytes * gamma / 2^20), no per-transfer term.  A
    token-wise chunk brings its own tokens; a layer-wise request brings all its tokens with the
    first layer it recomputes and nothing after that."""
    if n <= 0:
        return []
    bb = opts.boundary_bytes_per_token
    cost = lambda t: ceil_div(t * bb * cm.gamma, 1 << 20) if bb > 0 else 0
    if mode == TOKEN_WISE:
        c = opts.chunk_tokens
        return [cost(min((u + 1) * c, n) - u * c) for u in range(ceil_div(n, c))]
    return [cost(n)] + [0] * (opts.n_layers - 1)


def _split_of(opts, n, mode, p_comp):
    if mode == TOKEN_WISE:
        return (mode, min(p_comp * opts.chunk_tokens, n), opts.n_layers)
    return (mode, n, p_comp)


def plan(cm, opts, n_ctx, trace=None):
    """Run the scheduler.  Returns (splits, stats): splits[i] =
    (mode, k_tokens, layer_cut); stats = dict(t_comp, t_io, makespan,
    n_claims).  If `trace` is a list, every claim is appended to it as
    (engine, request, unit) with engine 0 = compute, 1 = I/O."""
    b_req = len(n_ctx)
    modes = [request_mode(opts, n) for n in n_ctx]
    costs = [unit_costs(cm, opts, n_ctx[i], modes[i]) for i in range(b_req)]
    bcost = [boundary_costs(cm, opts, n_ctx[i], modes[i]) for i in range(b_req)]
    p_comp = [0] * b_req
    p_io = [len(costs[i][0]) - 1 for i in range(b_req)]
    t_c, t_io = cm.s_c, cm.s_io        # each engine's clock starts after its start-up
    n_c = n_io = n_boundary = 0
    rr = 0
    n_claims = 0

    def live(i):
        return p_comp[i] <= p_io[i]

    def remaining_cost(i):
        return sum(costs[i][0][p_comp[i]:p_io[i] + 1])

    def remaining_cells(i):
        per = opts.n_layers if modes[i] == TOKEN_WISE else 1
        return sum(costs[i][2][p_comp[i]:p_io[i] + 1]) * per

    while any(live(i) for i in range(b_req)):
        # compute candidate: round-robin
        ic = next((rr + d) % b_req for d in range(b_req) if live((rr + d) % b_req))
        # I/O candidate: highest priority key
        best = None
        for i in range(b_req):
            if not live(i):
                continue
            if best is None:
                best = i
                continue
            if opts.io_key == KEY_REMAINING_COST:
                ki, kb = remaining_cost(i), remaining_cost(best)
            elif opts.io_key == KEY_REMAINING_CELLS:
                ki, kb = remaining_cells(i), remaining_cells(best)
            else:  # a_i/b_i vs a_best/b_best by cross-multiplication
                ki = costs[i][0][p_io[i]] * costs[best][1][p_io[best]]
                kb = costs[best][0][p_io[best]] * costs[i][1][p_io[i]]
            if ki > kb or (ki == kb and n_ctx[i] > n_ctx[best]):
                best = i
        iio = best
        fin_c = t_c + costs[ic][0][p_comp[ic]]
        fin_io = t_io + costs[iio][1][p_io[iio]]
        if fin_c <= fin_io:
            if trace is not None:
                trace.append((0, ic, p_comp[ic]))
            t_c = fin_c
            # the boundary rows of what is recomputed travel over the channel
            t_io += bcost[ic][p_comp[ic]]
            n_boundary += bcost[ic][p_comp[ic]] > 0
            n_c += 1
            p_comp[ic] += 1
            rr = (ic + 1) % b_req
        else:
            if trace is not None:
                trace.append((1, iio, p_io[iio]))
            t_io = fin_io
            n_io += 1
            p_io[iio] -= 1
        n_claims += 1

    if n_c == 0:
        t_c = 0            # an engine that claimed nothing never started
    if n_io == 0 and n_boundary == 0:
        t_io = 0

    splits = [_split_of(opts, n_ctx[i], modes[i], p_comp[i]) for i in range(b_req)]
    stats = dict(t_comp=t_c, t_io=t_io, makespan=max(t_c, t_io), n_claims=n_claims)
    return splits, stats


def split_times(cm, opts, n_ctx, unit_splits, modes=None):
    """(t_comp, t_io) if request i recomputes its first unit_splits[i] units
    and loads the rest."""
    t_c = t_io = 0
    any_c = any_io = False
    for i, n in enumerate(n_ctx):
        mode = request_mode(opts, n) if modes is None else modes[i]
        a, b, _ = unit_costs(cm, opts, n, mode)
        c_b = sum(boundary_costs(cm, opts, n, mode)[:unit_splits[i]])
        t_c += sum(a[:unit_splits[i]])
        t_io += sum(b[unit_splits[i]:]) + c_b
        any_c |= len(a[:unit_splits[i]]) > 0
        any_io |= len(b[unit_splits[i]:]) > 0 or c_b > 0
    return (t_c + cm.s_c if any_c else 0), (t_io + cm.s_io if any_io else 0)


def brute_force(cm, opts, n_ctx):
    """Minimum over all split vectors of max(sum claimed a, sum claimed b).
    Exponential; tiny batches only.  Returns (best_makespan, best_vector)."""
    modes = [request_mode(opts, n) for n in n_ctx]
    ms = [len(unit_costs(cm, opts, n, m)[0]) for n, m in zip(n_ctx, modes)]
    best, arg = None, None
    for vec in product(*[range(m + 1) for m in ms]):
        t_c, t_io = split_times(cm, opts, n_ctx, vec, modes)
        j = max(t_c, t_io)
        if best is None or j < best:
            best, arg = j, vec
    return best, arg


def derive_l_delta(cm, opts, n_max):
    """L_delta = min{N : T_token(N) <= T_layer(N)} (Sec. 3.1) on the grid of
    multiples of C up to n_max, with T_* the single-request makespans under
    the cost model.  Returns n_max + C if token-wise never wins."""
    c = opts.chunk_tokens
    n = c
    while n <= n_max:
        j = []
        for mode in (TOKEN_WISE, LAYER_WISE):
            o = PlanOpts(opts.chunk_tokens, 0, opts.n_layers,
                         opts.kv_bytes_per_token_layer, mode, opts.io_key)
            j.append(plan(cm, o, [n])[1]["makespan"])
        if j[0] <= j[1]:
            return n
        n += c
    return n_max + c


def all_recompute(opts, n_ctx):
    return [(TOKEN_WISE, n, opts.n_layers) for n in n_ctx]


def all_load(opts, n_ctx):
    return [(TOKEN_WISE, 0, opts.n_layers) for n in n_ctx]


def prefill_cost(cm, n_layers, n_ctx, n_new):
    """Compute-clock cost of the new-turn prefill of a batch: request i runs its n_new[i] new
    tokens from position n_ctx[i] through all layers (the cost formula of a recompute unit,
    Sec. 3.1, applied to those rows).  With the pipelined join this work rides on the compute
    stream beside the recompute, so the caller adds it to the compute start-up s_c before
    planning; the paper's TTFT = restoration + this."""
    return sum(compute_cost(cm, n_layers, m, n) for n, m in zip(n_ctx, n_new) if m > 0)


def cost_feedback(cm, pred_comp, meas_comp, pred_io, meas_io):
    """Closed-loop correction of the cost model after an executed batch: compute-side
    coefficients times measured/predicted compute time, I/O-side ones times
    measured/predicted I/O time, each ratio clamped to [1/4, 4], round to nearest."""
    def scale(v, num, den):
        if num > 4 * den:
            num, den = 4, 1
        if 4 * num < den:
            num, den = 1, 4
        return (v * num + den // 2) // den
    out = CostModel(cm.f_c, cm.alpha, cm.beta, cm.f_io, cm.gamma, cm.s_c, cm.s_io)
    if pred_comp > 0 and meas_comp > 0:
        out.f_c = scale(cm.f_c, meas_comp, pred_comp)
        out.alpha = max(1, scale(cm.alpha, meas_comp, pred_comp))
        out.beta = scale(cm.beta, meas_comp, pred_comp)
        out.s_c = scale(cm.s_c, meas_comp, pred_comp)
    if pred_io > 0 and meas_io > 0:
        out.f_io = scale(cm.f_io, meas_io, pred_io)
        out.gamma = max(1, scale(cm.gamma, meas_io, pred_io))
        out.s_io = scale(cm.s_io, meas_io, pred_io)
    return out


# --------------------------------------------------------------------------
# Planning policy around Algorithm 1 (Sec. 3.3 names contention on shared
# resources and adaptation to evolving availability; Sec. 4.1 names the two
# extremes a hybrid has to beat: recompute everything, load everything).  The
# paper gives no formulas for these; the reading taken: while both engines run,
# every compute cost counts comp_permille/1000 and every load cost
# io_permille/1000 of its isolated value; the new turn's prefill is priced with
# the recompute formula and, under a per-layer pipelined join, rides on the
# compute clock with one layer of it left when the last load lands; the plan
# returned is the candidate (hybrid / all-load / all-recompute) with the
# smallest predicted time to first token.

PLAN_HYBRID, PLAN_ALL_LOAD, PLAN_ALL_RECOMPUTE = 0, 1, 2


def _permille(v, p):
    return (v * p + 500) // 1000


def kv_share_permille(d_model, n_q_heads, n_kv_heads, head_dim, d_ffn):
    """K/V-projection share of one layer's linear FLOPs, in permille, rounded to nearest."""
    qkv = 2 * d_model * (n_q_heads + 2 * n_kv_heads) * head_dim
    lin = qkv + 2 * n_q_heads * head_dim * d_model + 6 * d_model * d_ffn
    return (1000 * qkv + lin // 2) // lin


def plan_batch(cm, overlap, model, chunk_tokens, l_delta, force_mode, io_key, pipelined_join, n_ctx,
               n_new=None, stage_layers=0, stage_first_layer=0):
    """overlap = (comp_permille, io_permille); model = (n_layers, d_model, n_q_heads, n_kv_heads,
    head_dim, d_ffn, elem_bytes).  A stage above layer 0 recomputes from float32 boundary rows of
    d_model values, charged to the channel.  Returns (splits, info dict)."""
    n_layers, d_model, hq, hkv, hd, ffn, esz = model
    comp_pm, io_pm = overlap
    L = stage_layers if stage_layers > 0 else n_layers
    opts = PlanOpts(chunk_tokens, l_delta, L, 2 * hkv * hd * esz, force_mode, io_key,
                    kv_share_permille(d_model, hq, hkv, hd, ffn),
                    4 * d_model if stage_layers > 0 and stage_first_layer > 0 else 0)
    base = CostModel(cm.f_c, cm.alpha, cm.beta, cm.f_io, cm.gamma, cm.s_c, cm.s_io)
    if stage_layers > 0:
        base.s_c = cm.s_c * L // n_layers
    pre = 0
    if n_new is not None and stage_layers == 0:
        pre = prefill_cost(base, L, n_ctx, n_new)

    def times(s_c, p, comp, t_io):
        nt = s_c + p if p > 0 else 0
        if pipelined_join:
            t_comp = comp if comp > 0 else nt
            return t_comp, max(t_comp, t_io + p // L)
        return comp, max(comp, t_io) + nt

    # hybrid: Algorithm 1 under contention
    hy = CostModel(_permille(base.f_c, comp_pm), max(1 if base.alpha > 0 else 0, _permille(base.alpha, comp_pm)),
                   _permille(base.beta, comp_pm), _permille(base.f_io, io_pm),
                   max(1 if base.gamma > 0 else 0, _permille(base.gamma, io_pm)), _permille(base.s_c, comp_pm),
                   _permille(base.s_io, io_pm))
    pre_h = _permille(pre, comp_pm)
    run = CostModel(hy.f_c, hy.alpha, hy.beta, hy.f_io, hy.gamma, hy.s_c + (pre_h if pipelined_join else 0), hy.s_io)
    sp_h, st_h = plan(run, opts, n_ctx)
    recomputes = any(k > 0 and c > 0 for _, k, c in sp_h)
    loads = any(n > 0 and (k < n or c < L) for (_, k, c), n in zip(sp_h, n_ctx))
    th = times(hy.s_c, pre_h, st_h["t_comp"], st_h["t_io"])
    # the extremes, each engine alone, under the isolated costs
    modes = [request_mode(opts, n) for n in n_ctx]
    n_units = [len(unit_costs(base, opts, n, m)[0]) for n, m in zip(n_ctx, modes)]
    _, l_io = split_times(base, opts, n_ctx, [0] * len(n_ctx), modes)
    r_c, r_io = split_times(base, opts, n_ctx, n_units, modes)     # r_io: boundary rows, if any
    tl = times(base.s_c, pre, 0, l_io)
    tr = times(base.s_c, pre, (r_c + (pre if pipelined_join else 0)) if r_c > 0 else 0, r_io)
    sp_l = [(m, 0, L) if m == TOKEN_WISE else (m, n, 0) for m, n in zip(modes, n_ctx)]
    sp_r = [(m, n, L) for m, n in zip(modes, n_ctx)]
    kind = PLAN_HYBRID if (recomputes and loads) else (PLAN_ALL_LOAD if not recomputes else PLAN_ALL_RECOMPUTE)
    best = (th, tl, tr)[kind][1]
    if tl[1] < best:
        kind, best = PLAN_ALL_LOAD, tl[1]
    if tr[1] < best:
        kind, best = PLAN_ALL_RECOMPUTE, tr[1]
    info = dict(kind=kind, kv_only_permille=opts.kv_only_permille, pipelined_join=1 if pipelined_join else 0,
                prefill_ps=pre, t_comp=(th, tl, tr)[kind][0], t_io=(st_h["t_io"], l_io, r_io)[kind], ttft=best,
                ttft_hybrid=th[1], ttft_all_load=tl[1], ttft_all_recompute=tr[1])
    return (sp_h, sp_l, sp_r)[kind], info


def plan_feedback(cm, overlap, info, meas_compute, meas_copy, meas_total, meas_wait=0):
    """-> (cost model, overlap) after an executed batch.  A hybrid's ratios measured/predicted
    correct the overlap factors (one batch moves a factor by at most 5/4 or 4/5 -- the first
    hybrid after a cold start can measure far off on both engines at once --, factors stay in
    [500, 8000]); an extreme's ratio corrects the coefficients of the engine that ran alone
    (cost_feedback) and lets the overlap factors relax towards 1000."""
    def ratio(v, num, den):
        if 4 * num > 5 * den:
            num, den = 5, 4
        if 5 * num < 4 * den:
            num, den = 4, 5
        return (v * num + den // 2) // den
    meas_comp = meas_total if (info["pipelined_join"] and meas_total * 100 > meas_copy * 102) else meas_compute
    meas_comp = max(0, meas_comp - meas_wait)     # time the compute stream stood waiting for loads is not compute
    comp_pm, io_pm = overlap
    if info["kind"] == PLAN_HYBRID:
        if info["t_comp"] > 0 and meas_comp > 0:
            comp_pm = min(8000, max(500, ratio(comp_pm, meas_comp, info["t_comp"])))
        if info["t_io"] > 0 and meas_copy > 0:
            io_pm = min(8000, max(500, ratio(io_pm, meas_copy, info["t_io"])))
        return cm, (comp_pm, io_pm)
    # an extreme teaches nothing about contention: what was learned ages, a quarter of the way
    # back to 1000 per such batch (nothing measures the factors while an extreme is chosen)
    relax = lambda pm: pm - (pm - 1000) // 4 if pm >= 1000 else pm + (1000 - pm) // 4
    overlap = (relax(comp_pm), relax(io_pm))
    if info["kind"] == PLAN_ALL_LOAD:
        return cost_feedback(cm, 0, 0, info["t_io"], meas_copy), overlap
    return cost_feedback(cm, info["t_comp"], meas_comp, 0, 0), overlap


# --------------------------------------------------------------------------
# Run-time scheduling (Sec. 3.3: the scheduler works progressively, chunk by
# chunk, and re-ranks after every processed chunk).  The two decisions below
# are what an executor asks whenever one of its engines runs dry; costs are
# the cost model's, multiplied by the ratios measured/predicted seen so far
# (permille, products rounded down per unit).  The paper gives no mechanism;
# the reading taken here: an engine takes a unit only if its own finish time
# with it is no later than the time the other engine would need for everything
# still unclaimed, so that taking it cannot delay the end of the restoration.

def _scaled_units(cm, opts, n_ctx, scale_c, scale_io):
    out = []
    for n in n_ctx:
        mode = request_mode(opts, n)
        a, b, tok = unit_costs(cm, opts, n, mode)
        out.append((mode, [x * scale_c // 1000 for x in a], [x * scale_io // 1000 for x in b], a, tok, b))
    return out


def _io_candidate(opts, n_ctx, units, p_comp, p_io):
    """The live request with the largest I/O priority key (Sec. 3.3), ties to the longer
    context, then the lower index; None if no request is live."""
    best, best_key = None, None
    for i, n in enumerate(n_ctx):
        if p_comp[i] > p_io[i]:
            continue
        mode, _, _, a_raw, tok, _ = units[i]
        if opts.io_key == KEY_REMAINING_COST:
            key = Fraction(sum(a_raw[p_comp[i]:p_io[i] + 1]))
        elif opts.io_key == KEY_REMAINING_CELLS:
            per = opts.n_layers if mode == TOKEN_WISE else 1
            key = Fraction(sum(tok[p_comp[i]:p_io[i] + 1]) * per)
        else:
            key = Fraction(a_raw[p_io[i]], units[i][5][p_io[i]])
        if best is None or (key, n) > best_key:
            best, best_key = i, (key, n)
    return best


def io_pick(cm, opts, n_ctx, p_comp, p_io, closed=None, io_backlog=0, compute_busy=0,
            scale_c=1000, scale_io=1000):
    """Request whose far-end unit the I/O channel loads next, or -1 (none live, or the unit
    is better left to the compute engine): the candidate passes iff
    io_backlog + b <= compute_busy + (recompute cost of every unclaimed unit of requests the
    compute engine has not closed), or if its request is closed.  Layer-wise requests are
    loaded one layer of all of them at a time, so b sums over the live layer-wise ones."""
    closed = closed or [False] * len(n_ctx)
    units = _scaled_units(cm, opts, n_ctx, scale_c, scale_io)
    best = _io_candidate(opts, n_ctx, units, p_comp, p_io)
    if best is None:
        return -1
    if closed[best]:
        return best
    c_rem = compute_busy
    for i in range(len(n_ctx)):
        if not closed[i]:
            c_rem += sum(units[i][1][p_comp[i]:p_io[i] + 1])
    if units[best][0] == LAYER_WISE:
        b = sum(units[i][2][p_io[i]] for i in range(len(n_ctx))
                if p_comp[i] <= p_io[i] and units[i][0] == LAYER_WISE)
    else:
        b = units[best][2][p_io[best]]
    return best if io_backlog + b <= c_rem else -1


ORDER_CHEAPEST = 0     # least recompute cost per load cost saved first
ORDER_SHORTEST = 1     # least recomputation still ahead of the request first


def dynamic_claim(cm, opts, n_ctx, p_comp, p_io, closed=None, io_backlog=0, scale_c=1000,
                  scale_io=1000, step_fixed=0, step_cap=0, order=ORDER_CHEAPEST, compute_later=0,
                  max_units=1, io_alone=0):
    """Which live, open requests' next units the compute engine takes for its next step.

    R = io_backlog + load cost of every unclaimed unit: the time the I/O channel needs if
    compute takes nothing.  Candidates: each open token-wise request's next unit -- the unit
    behind the ones the step already holds of it, as long as the step holds fewer than
    `max_units` of that request (0: no limit) -- and all open layer-wise requests together as
    one candidate, once per step (they advance as a packed batch, one layer per step).
    The candidates are ranked by `order` (recompute cost per load cost, or the recomputation
    the request still has ahead of it; ascending, ties by index) and the first in rank with
        A + a + compute_later <= R - Bs
    is taken (A, Bs: recompute and load cost of what the step holds; A starts at
    `step_fixed`, the cost of work the step carries in any case; `compute_later` is work the
    compute engine has to do after this step whatever it takes now): the step, and what
    follows it, end no later than the channel would finish what the step leaves to it.  A
    request whose candidate fails is out for this step (its later units cost no less).  This
    repeats until no candidate passes or, with step_cap > 0, A has reached the cap (the first
    unit always goes in).

    Contention (Sec. 3.3, evolving resource availability): scale_io prices the channel while
    the compute engine recomputes beside it; `io_alone` > 0 is the channel's scale when the
    compute engine takes nothing.  Nothing is taken (take all 0) unless recomputing pays for
    the slowdown it causes:  max(A* + compute_later, R - Bs*) < max(step_fixed +
    compute_later, R_alone), with R_alone = R at the scale io_alone and A*, Bs* the totals of
    everything the same rule would take from this state without step_cap and max_units, the
    layer-wise group layer after layer (a capped step is the first of several: what counts
    is where the engine ends up, not what one step holds).

    Returns (take, step cost): take[i] = units taken of token-wise request i; for layer-wise
    requests 1 or 2, 2 marking that the group should stop this layer after its K/V write
    because the test fails for the group's next layer.  The step cost counts the group's layer
    at what the step really runs -- the whole layer (1) or its K/V projection (2) -- whereas the
    unit prices used for the decision charge a layer's attention and MLP to the following
    unit."""
    b_req = len(n_ctx)
    closed = closed or [False] * b_req
    units = _scaled_units(cm, opts, n_ctx, scale_c, scale_io)
    live = [i for i in range(b_req) if p_comp[i] <= p_io[i]]
    r_total = io_backlog + sum(sum(units[i][2][p_comp[i]:p_io[i] + 1]) for i in live)
    open_ = [i for i in live if not closed[i]]
    group = [i for i in open_ if units[i][0] == LAYER_WISE]
    front = list(p_comp)                       # next unit of each token-wise request

    def ahead(i):       # unscaled recomputation between the pointers
        return sum(units[i][3][front[i]:p_io[i] + 1])

    def before(x, y):
        if order == ORDER_SHORTEST:
            if x[4] != y[4]:
                return -1 if x[4] < y[4] else 1
        else:
            lhs, rhs = x[0] * y[1], y[0] * x[1]       # a_x/b_x against a_y/b_y
            if lhs != rhs:
                return -1 if lhs < rhs else 1
        return (x[2] > y[2]) - (x[2] < y[2])

    def greedy(cap, limit, group_depth):
        """One pass of the rule.  group_depth: how many layers of the layer-wise group a pass may
        take (a step runs one; the contention test looks at everything the engine would take)."""
        nonlocal front
        front = list(p_comp)
        take = [0] * b_req
        a_sum, b_sum = step_fixed, 0
        out = set()                            # requests (or the group's first member) that failed
        g_taken = 0
        g_open = bool(group)
        while True:
            if cap > 0 and a_sum >= cap and a_sum > step_fixed:
                break
            cands = [(units[i][1][front[i]], units[i][2][front[i]], i, False, ahead(i))
                     for i in open_ if units[i][0] == TOKEN_WISE and i not in out and front[i] <= p_io[i]
                     and (limit <= 0 or take[i] < limit)]
            if g_open and g_taken < group_depth and all(p_comp[i] + g_taken <= p_io[i] for i in group):
                cands.append((sum(units[i][1][p_comp[i] + g_taken] for i in group),
                              sum(units[i][2][p_comp[i] + g_taken] for i in group), group[0], True,
                              sum(sum(units[i][3][p_comp[i] + g_taken:p_io[i] + 1]) for i in group)))
            if not cands:
                break
            cands.sort(key=cmp_to_key(before))
            a, b, first, is_group, _ = cands[0]
            if a_sum + a + compute_later <= r_total - b_sum:
                a_sum += a
                b_sum += b
                if is_group:
                    g_taken += 1
                else:
                    take[first] += 1
                    front[first] += 1
            elif is_group:
                g_open = False
            else:
                out.add(first)
        return take, a_sum, b_sum, g_taken

    if io_alone > 0:
        # everything the compute engine would take from here on, steps and unit limits aside
        _, a_all, b_all, g_all = greedy(0, 0, 1 << 30)
        if a_all > step_fixed or g_all:
            alone = _scaled_units(cm, opts, n_ctx, scale_c, io_alone)
            r_alone = io_backlog + sum(sum(alone[i][2][p_comp[i]:p_io[i] + 1]) for i in live)
            if max(a_all + compute_later, r_total - b_all) >= max(step_fixed + compute_later, r_alone):
                return [0] * b_req, step_fixed
    take, a_sum, b_sum, g_taken = greedy(step_cap, max_units, 1)
    group_taken = g_taken > 0
    if group_taken:
        more = all(p_comp[i] + 1 <= p_io[i] for i in group)
        if more:
            more = a_sum + sum(units[i][1][p_comp[i] + 1] for i in group) + compute_later <= r_total - b_sum
        for i in group:
            take[i] = 1 if more else 2
        ran = 0
        for i in group:
            full = compute_cost(cm, 1, n_ctx[i], 0)
            kv = kv_only_cost(cm, opts.kv_only_permille, n_ctx[i]) if opts.kv_only_permille > 0 else full
            ran += (full if more else kv) * scale_c // 1000
        a_sum += ran - sum(units[i][1][p_comp[i]] for i in group)
    return take, a_sum


def simulate_dynamic(cm, opts, n_ctx, true_cm=None, lookahead=2_000_000_000, max_depth=4,
                     step_cap=0, order=ORDER_CHEAPEST, trace=None):
    """Event-driven model of an executor that schedules at run time with `io_pick` and
    `dynamic_claim`: the I/O channel holds one claimed unit plus more while less than
    `lookahead` of predicted work is queued (at most `max_depth`); the compute engine asks
    for a step whenever it is idle and the state has changed.  Durations come from
    `true_cm` (default: the model itself), predictions from `cm` times the ratios
    measured/predicted so far.  A step lasts the sum of its units' true costs.
    If `trace` is a list, every claim is appended to it as (time, engine, request, unit) with
    engine 0 = compute, 1 = I/O (a layer-wise group's claim names its first member).
    Returns (splits, makespan, n_steps)."""
    true_cm = true_cm or cm
    b_req = len(n_ctx)
    modes = [request_mode(opts, n) for n in n_ctx]
    pred = [unit_costs(cm, opts, n_ctx[i], modes[i]) for i in range(b_req)]
    true = [unit_costs(true_cm, opts, n_ctx[i], modes[i]) for i in range(b_req)]
    p_comp = [0] * b_req
    p_io = [len(pred[i][0]) - 1 for i in range(b_req)]
    closed = [False] * b_req
    group = [i for i in range(b_req) if modes[i] == LAYER_WISE and n_ctx[i] > 0]
    now = 0
    io_queue = []            # (true duration, predicted) of claimed loads, oldest first
    io_head_done = 0         # when the load at the head of the queue completes
    io_pred_done = 0
    io_busy_from = None
    step_end, step_start, step_pred = None, 0, 0
    c_pred_done = c_true_done = 0
    scale_c = scale_io = 1000
    n_steps = 0
    ask = True
    force_io = False

    def clamp(num, den):
        return min(4000, max(250, (num * 1000 + den // 2) // den))

    while True:
        progressed = False
        while len(io_queue) < max_depth:
            backlog = sum(d * scale_io // 1000 for _, d in io_queue)
            if io_queue and backlog >= lookahead:
                break
            busy = max(0, step_pred - (now - step_start)) if step_end is not None else 0
            if force_io:
                busy = 1 << 62
            force_io = False
            i = io_pick(cm, opts, n_ctx, p_comp, p_io, closed, backlog, busy, scale_c, scale_io)
            if i < 0:
                break
            members = group if modes[i] == LAYER_WISE else [i]
            u = p_io[i]
            d_true = sum(true[j][1][u] for j in members)
            d_pred = sum(pred[j][1][u] for j in members)
            for j in members:
                p_io[j] -= 1
            if trace is not None:
                trace.append((now, 1, members[0], u))
            if not io_queue:
                io_head_done = now + d_true
            if io_busy_from is None:
                io_busy_from = now
            io_queue.append((d_true, d_pred))
            ask = progressed = True
        if step_end is None and ask:
            ask = False
            backlog = sum(d * scale_io // 1000 for _, d in io_queue)
            take, a_pred = dynamic_claim(cm, opts, n_ctx, p_comp, p_io, closed, backlog, scale_c, scale_io,
                                         0, step_cap, order)
            dur = 0
            for i in range(b_req):
                if take[i]:
                    if trace is not None and (modes[i] == TOKEN_WISE or i == group[0]):
                        trace.append((now, 0, i, p_comp[i]))
                    dur += true[i][0][p_comp[i]]
                    p_comp[i] += 1
                    if take[i] == 2:
                        closed[i] = True
            if any(take):
                step_start, step_end, step_pred = now, now + dur, a_pred
                c_true_done += dur
                n_steps += 1
                progressed = True
        events = ([io_head_done] if io_queue else []) + ([step_end] if step_end is not None else [])
        if not events:
            if all(p_comp[i] > p_io[i] for i in range(b_req)):
                break
            if not progressed:
                if force_io:
                    raise AssertionError("scheduler stalled with live requests")
                force_io = True
            continue
        now = min(events)
        if io_queue and io_head_done == now:
            _, d_pred = io_queue.pop(0)
            io_pred_done += d_pred
            if io_queue:
                io_head_done = now + io_queue[0][0]
            if io_pred_done > 0 and now > io_busy_from:
                scale_io = clamp(now - io_busy_from, io_pred_done)
            ask = True
        if step_end is not None and step_end == now:
            step_end = None
            c_pred_done += step_pred
            if c_pred_done > 0:
                scale_c = clamp(c_true_done, c_pred_done)
            ask = True
    splits = [_split_of(opts, n_ctx[i], modes[i], p_comp[i]) for i in range(b_req)]
    return splits, now, n_steps
