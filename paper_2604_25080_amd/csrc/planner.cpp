// Batch-aware two-pointer restoration scheduler (Algorithm 1, Sec. 3.3) over
// an integer cost model.  Host only.
//
// Each request is cut into units: chunks of C tokens through all layers
// (token-wise, Sec. 3.1) or single layers over all tokens (layer-wise).  A
// compute pointer climbs from unit 0, an I/O pointer descends from the last
// unit; the request is finished when they have crossed.  The batch shares one
// compute engine and one I/O channel, each with its own clock.  At every step
// the compute engine's candidate is the next unfinished request in round-robin
// order, the I/O channel's candidate is the unfinished request with the most
// recomputation still ahead of it (Sec. 3.3), and whichever engine would be
// done with its candidate first takes it (ties: compute).  Priorities are
// re-evaluated after every unit (the "progressive, chunk-level" update).
#include <algorithm>
#include <vector>

#include "cf_common.h"

namespace {

struct Units {
    int mode = CF_TOKEN_WISE;
    int n = 0;                      // context tokens
    std::vector<int64_t> a_prefix;  // a_prefix[u] = sum of recompute cost of units < u
    std::vector<int64_t> b;         // load cost per unit
    std::vector<int64_t> c_io;      // channel time a RECOMPUTE claim of the unit costs (boundary rows)
    std::vector<int64_t> tok_prefix;
    int m() const { return (int)b.size(); }
    int64_t a(int u) const { return a_prefix[u + 1] - a_prefix[u]; }
};

int64_t layer_pass_cost(const cf_cost_model& cm, int64_t layers, int64_t t, int64_t p0) {
    int64_t pairs = t * p0 + t * (t + 1) / 2;
    return layers * (cm.f_c + cm.alpha * t + cm.beta * cf::ceil_div(pairs, 1024));
}

// The last recomputed layer of a request stops after its K/V write: fixed part plus
// kv_only_permille / 1000 of the linear part, no attention.
int64_t kv_only_cost(const cf_cost_model& cm, int64_t permille, int64_t t) {
    return cm.f_c + (cm.alpha * permille * t + 999) / 1000;
}

int64_t load_cost(const cf_cost_model& cm, int64_t bytes) {
    // bytes*gamma can exceed 2^63 only for absurd inputs; use 128-bit to be exact
    __int128 num = (__int128)bytes * cm.gamma;
    __int128 q = (num + ((__int128)1 << 20) - 1) >> 20;
    return cm.f_io + (int64_t)q;
}

// channel time of `tokens` boundary-activation rows (no per-transfer term: they ride with the
// step's metadata)
int64_t boundary_cost(const cf_cost_model& cm, const cf_plan_opts& o, int64_t tokens) {
    if (o.boundary_bytes_per_token <= 0) return 0;
    __int128 num = (__int128)tokens * o.boundary_bytes_per_token * cm.gamma;
    return (int64_t)((num + ((__int128)1 << 20) - 1) >> 20);
}

int mode_of(const cf_plan_opts& o, int n) {
    if (o.force_mode == CF_TOKEN_WISE || o.force_mode == CF_LAYER_WISE) return o.force_mode;
    return n >= o.l_delta ? CF_TOKEN_WISE : CF_LAYER_WISE;
}

Units make_units(const cf_cost_model& cm, const cf_plan_opts& o, int n, int mode) {
    Units u;
    u.mode = mode;
    u.n = n;
    u.a_prefix.push_back(0);
    u.tok_prefix.push_back(0);
    if (n <= 0) return u;
    if (mode == CF_TOKEN_WISE) {
        int c = o.chunk_tokens;
        for (int64_t s = 0; s < n; s += c) {
            int64_t t = (s + c <= n) ? c : n - s;
            int64_t a = o.kv_only_permille > 0
                            ? layer_pass_cost(cm, o.n_layers - 1, t, s) + kv_only_cost(cm, o.kv_only_permille, t)
                            : layer_pass_cost(cm, o.n_layers, t, s);
            u.a_prefix.push_back(u.a_prefix.back() + a);
            u.b.push_back(load_cost(cm, t * o.n_layers * (int64_t)o.kv_bytes_per_token_layer));
            u.c_io.push_back(boundary_cost(cm, o, t));
            u.tok_prefix.push_back(u.tok_prefix.back() + t * o.n_layers);
        }
    } else {
        for (int l = 0; l < o.n_layers; ++l) {
            // claiming layer l makes layer l-1 a full layer and adds a K/V-only layer l
            int64_t a = (o.kv_only_permille > 0 && l == 0) ? kv_only_cost(cm, o.kv_only_permille, n)
                                                           : layer_pass_cost(cm, 1, n, 0);
            u.a_prefix.push_back(u.a_prefix.back() + a);
            u.b.push_back(load_cost(cm, (int64_t)n * o.kv_bytes_per_token_layer));
            u.c_io.push_back(l == 0 ? boundary_cost(cm, o, n) : 0);
            u.tok_prefix.push_back(u.tok_prefix.back() + n);
        }
    }
    return u;
}

int check(const cf_cost_model* cm, const cf_plan_opts* o, int32_t B, const int32_t* n_ctx,
          const char* who) {
    if (!cm || !o || B < 0 || (B > 0 && !n_ctx))
        return cf::fail(CF_ERR_INVALID_ARG, "%s: null argument or negative batch", who);
    if (o->chunk_tokens <= 0 || o->n_layers <= 0 || o->kv_bytes_per_token_layer <= 0)
        return cf::fail(CF_ERR_INVALID_ARG, "%s: chunk_tokens, n_layers and KV bytes must be > 0",
                        who);
    if (o->kv_only_permille < 0 || o->kv_only_permille > 1000)
        return cf::fail(CF_ERR_INVALID_ARG, "%s: kv_only_permille %d not in 0..1000", who, o->kv_only_permille);
    if (o->boundary_bytes_per_token < 0)
        return cf::fail(CF_ERR_INVALID_ARG, "%s: boundary_bytes_per_token < 0", who);
    if (o->io_key < 0 || o->io_key > CF_KEY_MARGINAL || o->force_mode < -1 || o->force_mode > 1)
        return cf::fail(CF_ERR_INVALID_ARG, "%s: bad io_key or force_mode", who);
    if (cm->f_c < 0 || cm->alpha < 0 || cm->beta < 0 || cm->f_io < 0 || cm->gamma < 0 ||
        cm->s_c < 0 || cm->s_io < 0)
        return cf::fail(CF_ERR_INVALID_ARG, "%s: negative cost coefficient", who);
    for (int i = 0; i < B; ++i)
        if (n_ctx[i] < 0) return cf::fail(CF_ERR_INVALID_ARG, "%s: n_ctx[%d] < 0", who, i);
    return CF_OK;
}

// The I/O channel's candidate: the live request (p_comp <= p_io) with the largest key -- by
// default the recomputation still ahead of it (Sec. 3.3); ties go to the longer context, then
// to the lower index.  -1 if no request is live.
int pick_io(const std::vector<Units>& req, const std::vector<int>& pc, const std::vector<int>& pio,
            const int32_t* n_ctx, int io_key) {
    int best = -1;
    for (int i = 0; i < (int)req.size(); ++i) {
        if (pc[i] > pio[i]) continue;
        if (best < 0) { best = i; continue; }
        bool gt, eq;
        if (io_key == CF_KEY_MARGINAL) {
            __int128 ki = (__int128)req[i].a(pio[i]) * req[best].b[pio[best]];
            __int128 kb = (__int128)req[best].a(pio[best]) * req[i].b[pio[i]];
            gt = ki > kb; eq = ki == kb;
        } else {
            const auto& pi = io_key == CF_KEY_REMAINING_COST ? req[i].a_prefix : req[i].tok_prefix;
            const auto& pb = io_key == CF_KEY_REMAINING_COST ? req[best].a_prefix : req[best].tok_prefix;
            int64_t ki = pi[pio[i] + 1] - pi[pc[i]];
            int64_t kb = pb[pio[best] + 1] - pb[pc[best]];
            gt = ki > kb; eq = ki == kb;
        }
        if (gt || (eq && n_ctx[i] > n_ctx[best])) best = i;
    }
    return best;
}

// Shared argument check of the run-time scheduling calls: pointers of every request must lie
// in [0, units] x [-1, units-1].
int check_pointers(const std::vector<Units>& req, const int32_t* p_comp, const int32_t* p_io,
                   const char* who) {
    for (int i = 0; i < (int)req.size(); ++i)
        if (p_comp[i] < 0 || p_comp[i] > req[i].m() || p_io[i] < -1 || p_io[i] >= req[i].m())
            return cf::fail(CF_ERR_INVALID_ARG, "%s: pointers of request %d outside its %d units", who, i,
                            req[i].m());
    return CF_OK;
}

}  // namespace

extern "C" int cf_restore_plan(const cf_cost_model* cost, const cf_plan_opts* opts, int32_t B,
                               const int32_t* n_ctx, cf_split* out, cf_plan_stats* stats,
                               cf_claim* trace, int32_t trace_cap) {
    int rc = check(cost, opts, B, n_ctx, "cf_restore_plan");
    if (rc) return rc;
    if (B > 0 && !out) return cf::fail(CF_ERR_INVALID_ARG, "cf_restore_plan: null out_splits");
    if (trace_cap < 0 || (trace_cap > 0 && !trace))
        return cf::fail(CF_ERR_INVALID_ARG, "cf_restore_plan: bad trace buffer");

    std::vector<Units> req(B);
    std::vector<int> pc(B, 0), pio(B);
    int n_live = 0;
    for (int i = 0; i < B; ++i) {
        req[i] = make_units(*cost, *opts, n_ctx[i], mode_of(*opts, n_ctx[i]));
        pio[i] = req[i].m() - 1;
        n_live += pc[i] <= pio[i];
    }
    int64_t t_c = cost->s_c, t_io = cost->s_io;   // clocks start after the engines' start-up
    int n_c = 0, n_io = 0;
    bool boundary_moved = false;                  // the channel carried boundary rows
    int rr = 0, n_claims = 0, n_trace = 0;
    auto live = [&](int i) { return pc[i] <= pio[i]; };

    while (n_live > 0) {
        int ic = rr;
        while (!live(ic)) ic = (ic + 1 == B) ? 0 : ic + 1;
        int best = pick_io(req, pc, pio, n_ctx, opts->io_key);
        int64_t fin_c = t_c + req[ic].a(pc[ic]);
        int64_t fin_io = t_io + req[best].b[pio[best]];
        cf_claim cl;
        if (fin_c <= fin_io) {
            cl = {0, ic, pc[ic]};
            t_c = fin_c;
            // a stage above layer 0 recomputes from boundary rows that cross the host link
            t_io += req[ic].c_io[pc[ic]];
            boundary_moved |= req[ic].c_io[pc[ic]] > 0;
            ++n_c;
            ++pc[ic];
            if (!live(ic)) --n_live;
            rr = (ic + 1 == B) ? 0 : ic + 1;
        } else {
            cl = {1, best, pio[best]};
            t_io = fin_io;
            ++n_io;
            --pio[best];
            if (!live(best)) --n_live;
        }
        if (n_trace < trace_cap) trace[n_trace++] = cl;
        ++n_claims;
    }
    for (int i = 0; i < B; ++i) {
        out[i].mode = req[i].mode;
        if (req[i].mode == CF_TOKEN_WISE) {
            int64_t k = (int64_t)pc[i] * opts->chunk_tokens;
            out[i].k_tokens = (int32_t)(k < n_ctx[i] ? k : n_ctx[i]);
            out[i].layer_cut = opts->n_layers;
        } else {
            out[i].k_tokens = n_ctx[i];
            out[i].layer_cut = pc[i];
        }
    }
    if (n_c == 0) t_c = 0;     // an engine that claimed nothing never started
    if (n_io == 0 && !boundary_moved) t_io = 0;
    if (stats) {
        stats->t_comp = t_c;
        stats->t_io = t_io;
        stats->makespan = t_c > t_io ? t_c : t_io;
        stats->n_claims = n_claims;
        stats->n_trace = n_trace;
    }
    return CF_OK;
}

extern "C" int cf_plan_eval(const cf_cost_model* cost, const cf_plan_opts* opts, int32_t B,
                            const int32_t* n_ctx, const cf_split* splits, int64_t* t_comp,
                            int64_t* t_io) {
    int rc = check(cost, opts, B, n_ctx, "cf_plan_eval");
    if (rc) return rc;
    if ((B > 0 && !splits) || !t_comp || !t_io)
        return cf::fail(CF_ERR_INVALID_ARG, "cf_plan_eval: null argument");
    int64_t tc = 0, tio = 0;
    bool any_c = false, any_io = false;
    for (int i = 0; i < B; ++i) {
        const cf_split& s = splits[i];
        if (s.k_tokens < 0 || s.k_tokens > n_ctx[i] || s.layer_cut < 0 ||
            s.layer_cut > opts->n_layers || (s.mode != CF_TOKEN_WISE && s.mode != CF_LAYER_WISE))
            return cf::fail(CF_ERR_INVALID_PLAN, "cf_plan_eval: split %d out of range", i);
        Units u = make_units(*cost, *opts, n_ctx[i], s.mode);
        int n_comp = s.mode == CF_TOKEN_WISE
                         ? (int)cf::ceil_div(s.k_tokens, opts->chunk_tokens)
                         : s.layer_cut;
        if (n_comp > u.m()) n_comp = u.m();
        tc += u.a_prefix[n_comp];
        for (int v = n_comp; v < u.m(); ++v) tio += u.b[v];
        for (int v = 0; v < n_comp; ++v) {
            tio += u.c_io[v];
            any_io |= u.c_io[v] > 0;
        }
        any_c |= n_comp > 0;
        any_io |= n_comp < u.m();
    }
    *t_comp = any_c ? tc + cost->s_c : 0;
    *t_io = any_io ? tio + cost->s_io : 0;
    return CF_OK;
}

extern "C" int cf_derive_l_delta(const cf_cost_model* cost, const cf_plan_opts* opts,
                                 int32_t n_max, int32_t* l_delta) {
    int32_t dummy = 0;
    int rc = check(cost, opts, 1, &dummy, "cf_derive_l_delta");
    if (rc) return rc;
    if (!l_delta || n_max < 0) return cf::fail(CF_ERR_INVALID_ARG, "cf_derive_l_delta: bad argument");
    cf_plan_opts o = *opts;
    o.l_delta = 0;
    int64_t c = opts->chunk_tokens;
    for (int64_t n = c; n <= n_max; n += c) {
        int32_t nn = (int32_t)n;
        cf_split s;
        cf_plan_stats st_tok, st_lay;
        o.force_mode = CF_TOKEN_WISE;
        cf_restore_plan(cost, &o, 1, &nn, &s, &st_tok, nullptr, 0);
        o.force_mode = CF_LAYER_WISE;
        cf_restore_plan(cost, &o, 1, &nn, &s, &st_lay, nullptr, 0);
        if (st_tok.makespan <= st_lay.makespan) {
            *l_delta = nn;
            return CF_OK;
        }
    }
    *l_delta = (int32_t)(n_max + c);
    return CF_OK;
}

// Compute-clock cost of the new-turn prefill of a batch (the recompute cost formula applied to
// rows n_ctx[i] .. n_ctx[i]+n_new[i]-1 through n_layers layers).
extern "C" int cf_prefill_cost(const cf_cost_model* cost, int32_t n_layers, int32_t B,
                               const int32_t* n_ctx, const int32_t* n_new, int64_t* out_ps) {
    if (!cost || !out_ps || n_layers < 0 || B < 0 || (B > 0 && (!n_ctx || !n_new)))
        return cf::fail(CF_ERR_INVALID_ARG, "cf_prefill_cost: bad argument");
    int64_t total = 0;
    for (int i = 0; i < B; ++i) {
        if (n_ctx[i] < 0 || n_new[i] < 0)
            return cf::fail(CF_ERR_INVALID_ARG, "cf_prefill_cost: request %d has a negative length", i);
        if (n_new[i] > 0) total += layer_pass_cost(*cost, n_layers, n_new[i], n_ctx[i]);
    }
    *out_ps = total;
    return CF_OK;
}

// Closed-loop correction of the cost model from one executed batch: the compute-side
// coefficients are scaled by measured/predicted compute time, the I/O-side ones by
// measured/predicted I/O time (each clamped to [1/4, 4] per update).  This is how the
// scheduler adapts to what calibration in isolation cannot see: the two engines slow each
// other down when they run together (Sec. 3.3: priorities follow evolving resource
// availability).  Integer arithmetic, round to nearest.
extern "C" int cf_cost_feedback(cf_cost_model* cost, int64_t pred_comp, int64_t meas_comp,
                                int64_t pred_io, int64_t meas_io) {
    if (!cost || pred_comp < 0 || meas_comp < 0 || pred_io < 0 || meas_io < 0)
        return cf::fail(CF_ERR_INVALID_ARG, "cf_cost_feedback: bad argument");
    auto scale = [](int64_t v, int64_t num, int64_t den) -> int64_t {
        if (num > 4 * den) { num = 4; den = 1; }
        if (4 * num < den) { num = 1; den = 4; }
        __int128 r = ((__int128)v * num + den / 2) / den;
        return (int64_t)r;
    };
    if (pred_comp > 0 && meas_comp > 0) {
        cost->f_c = scale(cost->f_c, meas_comp, pred_comp);
        cost->alpha = std::max<int64_t>(1, scale(cost->alpha, meas_comp, pred_comp));
        cost->beta = scale(cost->beta, meas_comp, pred_comp);
        cost->s_c = scale(cost->s_c, meas_comp, pred_comp);
    }
    if (pred_io > 0 && meas_io > 0) {
        cost->f_io = scale(cost->f_io, meas_io, pred_io);
        cost->gamma = std::max<int64_t>(1, scale(cost->gamma, meas_io, pred_io));
        cost->s_io = scale(cost->s_io, meas_io, pred_io);
    }
    return CF_OK;
}

// ---------------------------------------------------------------- planning policy
// cf_plan_batch: Algorithm 1 with the terms a serving loop has to add around it, and the check
// against the two extremes; cf_plan_feedback: the closed loop.  Integer arithmetic throughout
// (an oracle twin reproduces every number bit for bit).

namespace {

int64_t scale_permille(int64_t v, int64_t permille) {          // round to nearest
    return (int64_t)(((__int128)v * permille + 500) / 1000);
}

// v * num / den with the ratio clamped to [4/5, 5/4]: how far one batch may move an overlap factor
int64_t ratio_step(int64_t v, int64_t num, int64_t den) {
    if (4 * num > 5 * den) { num = 5; den = 4; }
    if (5 * num < 4 * den) { num = 4; den = 5; }
    return (int64_t)(((__int128)v * num + den / 2) / den);
}

}  // namespace

extern "C" int cf_plan_batch(const cf_cost_model* cost, const cf_overlap_model* overlap,
                             const cf_model_desc* desc, const cf_batch_plan_opts* bo, int32_t B,
                             const int32_t* n_ctx, const int32_t* n_new, cf_split* out,
                             cf_batch_plan* info) {
    if (!cost || !overlap || !desc || !bo || B < 0 || (B > 0 && (!n_ctx || !out)))
        return cf::fail(CF_ERR_INVALID_ARG, "cf_plan_batch: null argument or negative batch");
    if (desc->n_layers <= 0 || desc->d_model <= 0 || desc->n_q_heads <= 0 || desc->n_kv_heads <= 0 ||
        desc->head_dim <= 0 || desc->d_ffn <= 0 || (desc->dtype != CF_F32 && desc->dtype != CF_BF16))
        return cf::fail(CF_ERR_INVALID_ARG, "cf_plan_batch: model descriptor has a non-positive field or bad dtype");
    if (overlap->comp_permille < 500 || overlap->comp_permille > 8000 || overlap->io_permille < 500 ||
        overlap->io_permille > 8000)
        return cf::fail(CF_ERR_INVALID_ARG, "cf_plan_batch: overlap factors must lie in [500, 8000] permille");
    if (bo->stage_layers < 0 || bo->stage_layers > desc->n_layers)
        return cf::fail(CF_ERR_INVALID_ARG, "cf_plan_batch: stage_layers %d not in [0, %d]", bo->stage_layers,
                        desc->n_layers);
    const int L = bo->stage_layers > 0 ? bo->stage_layers : desc->n_layers;
    // 1. the K/V projection's share of a layer's linear FLOPs
    const int64_t d = desc->d_model, hd = desc->head_dim;
    const int64_t qkv = 2 * d * (desc->n_q_heads + 2 * (int64_t)desc->n_kv_heads) * hd;
    const int64_t lin = qkv + 2 * (int64_t)desc->n_q_heads * hd * d + 6 * d * (int64_t)desc->d_ffn;
    cf_plan_opts po;
    po.chunk_tokens = bo->chunk_tokens;
    po.l_delta = bo->l_delta;
    po.n_layers = L;
    po.kv_bytes_per_token_layer = (int32_t)(2 * (int64_t)desc->n_kv_heads * hd * (int64_t)cf::elem_bytes(desc->dtype));
    po.force_mode = bo->force_mode;
    po.io_key = bo->io_key;
    po.kv_only_permille = (int32_t)((1000 * qkv + lin / 2) / lin);
    po.boundary_bytes_per_token = (bo->stage_layers > 0 && bo->stage_first_layer > 0) ? (int32_t)(4 * d) : 0;
    if (bo->stage_first_layer < 0 || bo->stage_first_layer + L > desc->n_layers)
        return cf::fail(CF_ERR_INVALID_ARG, "cf_plan_batch: stage [%d, %d) outside the model's %d layers",
                        bo->stage_first_layer, bo->stage_first_layer + L, desc->n_layers);
    int rc = check(cost, &po, B, n_ctx, "cf_plan_batch");
    if (rc) return rc;
    // a stage pays its share of the per-pass start-up and has no new turn of its own
    cf_cost_model base = *cost;
    if (bo->stage_layers > 0) base.s_c = (int64_t)(((__int128)cost->s_c * L) / desc->n_layers);
    // 2. the new turn
    int64_t prefill = 0;
    if (n_new && bo->stage_layers == 0)
        for (int i = 0; i < B; ++i) {
            if (n_new[i] < 0) return cf::fail(CF_ERR_INVALID_ARG, "cf_plan_batch: n_new[%d] < 0", i);
            if (n_new[i] > 0) prefill += layer_pass_cost(base, L, n_new[i], n_ctx[i]);
        }
    const bool piped = bo->pipelined_join != 0;
    // Times of a candidate x from its start-up s_c_x, its new-turn cost pre_x, the compute
    // clock `comp` at the end of its claims (start-up included; 0 = claimed nothing) and its
    // channel time t_io.  The new turn as a pass of its own costs nt = s_c_x + pre_x.
    //   pipelined join : the new turn rides on the compute clock, which Algorithm 1 was started
    //                    at s_c_x + pre_x for; one layer of it is left when the last load lands
    //   sequential join: the new turn is a pass after both engines are done
    struct Times { int64_t t_comp, ttft; };
    auto times_of = [&](int64_t s_c_x, int64_t pre_x, int64_t comp, int64_t t_io) {
        const int64_t nt = pre_x > 0 ? s_c_x + pre_x : 0;
        Times t;
        if (piped) {
            t.t_comp = comp > 0 ? comp : nt;
            t.ttft = std::max(t.t_comp, t_io + pre_x / L);
        } else {
            t.t_comp = comp;
            t.ttft = std::max(comp, t_io) + nt;
        }
        return t;
    };
    // 3. the hybrid under contention
    cf_cost_model hy = base;
    hy.f_c = scale_permille(base.f_c, overlap->comp_permille);
    hy.alpha = std::max<int64_t>(base.alpha > 0 ? 1 : 0, scale_permille(base.alpha, overlap->comp_permille));
    hy.beta = scale_permille(base.beta, overlap->comp_permille);
    hy.s_c = scale_permille(base.s_c, overlap->comp_permille);
    hy.f_io = scale_permille(base.f_io, overlap->io_permille);
    hy.gamma = std::max<int64_t>(base.gamma > 0 ? 1 : 0, scale_permille(base.gamma, overlap->io_permille));
    hy.s_io = scale_permille(base.s_io, overlap->io_permille);
    const int64_t prefill_hy = scale_permille(prefill, overlap->comp_permille);
    cf_cost_model hy_plan = hy;
    if (piped) hy_plan.s_c += prefill_hy;
    std::vector<cf_split> sp_h(std::max(B, 1));
    cf_plan_stats st_h;
    rc = cf_restore_plan(&hy_plan, &po, B, n_ctx, sp_h.data(), &st_h, nullptr, 0);
    if (rc) return rc;
    bool recomputes = false, loads = false;
    for (int i = 0; i < B; ++i) {
        if (sp_h[i].k_tokens > 0 && sp_h[i].layer_cut > 0) recomputes = true;
        if (n_ctx[i] > 0 && (sp_h[i].k_tokens < n_ctx[i] || sp_h[i].layer_cut < L)) loads = true;
    }
    const Times th = times_of(hy.s_c, prefill_hy, st_h.t_comp, st_h.t_io);
    // 4. the extremes, each engine alone
    std::vector<cf_split> sp_l(std::max(B, 1)), sp_r(std::max(B, 1));
    for (int i = 0; i < B; ++i) {
        const int mode = mode_of(po, n_ctx[i]);
        sp_l[i] = mode == CF_TOKEN_WISE ? cf_split{mode, 0, L} : cf_split{mode, n_ctx[i], 0};
        sp_r[i] = cf_split{mode, n_ctx[i], L};
    }
    int64_t l_c = 0, l_io = 0, r_c = 0, r_io = 0;
    rc = cf_plan_eval(&base, &po, B, n_ctx, sp_l.data(), &l_c, &l_io);
    if (rc) return rc;
    rc = cf_plan_eval(&base, &po, B, n_ctx, sp_r.data(), &r_c, &r_io);
    if (rc) return rc;
    const Times tl = times_of(base.s_c, prefill, 0, l_io);
    const Times tr = times_of(base.s_c, prefill, r_c > 0 ? r_c + (piped ? prefill : 0) : 0, r_io);   // boundary rows, if any
    const int64_t ttft_h = th.ttft, ttft_l = tl.ttft, ttft_r = tr.ttft;
    // 5. / 6. the best candidate
    int kind = CF_PLAN_HYBRID;
    if (!recomputes) kind = CF_PLAN_ALL_LOAD;
    else if (!loads) kind = CF_PLAN_ALL_RECOMPUTE;
    int64_t best = kind == CF_PLAN_HYBRID ? ttft_h : (kind == CF_PLAN_ALL_LOAD ? ttft_l : ttft_r);
    if (ttft_l < best) { kind = CF_PLAN_ALL_LOAD; best = ttft_l; }
    if (ttft_r < best) { kind = CF_PLAN_ALL_RECOMPUTE; best = ttft_r; }
    const std::vector<cf_split>& chosen = kind == CF_PLAN_HYBRID ? sp_h : (kind == CF_PLAN_ALL_LOAD ? sp_l : sp_r);
    for (int i = 0; i < B; ++i) out[i] = chosen[i];
    if (info) {
        info->kind = kind;
        info->kv_only_permille = po.kv_only_permille;
        info->pipelined_join = piped ? 1 : 0;
        info->reserved = 0;
        info->prefill_ps = prefill;
        const Times& tc = kind == CF_PLAN_HYBRID ? th : (kind == CF_PLAN_ALL_LOAD ? tl : tr);
        info->t_comp = tc.t_comp;
        info->t_io = kind == CF_PLAN_HYBRID ? st_h.t_io : (kind == CF_PLAN_ALL_LOAD ? l_io : r_io);
        info->ttft = best;
        info->ttft_hybrid = ttft_h;
        info->ttft_all_load = ttft_l;
        info->ttft_all_recompute = ttft_r;
    }
    return CF_OK;
}

extern "C" int cf_plan_feedback(cf_cost_model* cost, cf_overlap_model* overlap, const cf_batch_plan* info,
                                int64_t meas_compute_ps, int64_t meas_copy_ps, int64_t meas_total_ps,
                                int64_t meas_wait_ps) {
    if (!cost || !overlap || !info || meas_compute_ps < 0 || meas_copy_ps < 0 || meas_total_ps < 0 || meas_wait_ps < 0)
        return cf::fail(CF_ERR_INVALID_ARG, "cf_plan_feedback: bad argument");
    if (info->kind < CF_PLAN_HYBRID || info->kind > CF_PLAN_ALL_RECOMPUTE)
        return cf::fail(CF_ERR_INVALID_ARG, "cf_plan_feedback: unknown plan kind %d", info->kind);
    // the compute stream's end: with the pipelined join, the call's end when that came well
    // after the copy stream's
    // after the copy stream's, less the time it stood waiting for loads
    const int64_t meas_end = (info->pipelined_join && (__int128)meas_total_ps * 100 > (__int128)meas_copy_ps * 102)
                                 ? meas_total_ps : meas_compute_ps;
    const int64_t meas_comp = std::max<int64_t>(0, meas_end - meas_wait_ps);
    if (info->kind == CF_PLAN_HYBRID) {
        if (info->t_comp > 0 && meas_comp > 0)
            overlap->comp_permille = (int32_t)std::min<int64_t>(
                8000, std::max<int64_t>(500, ratio_step(overlap->comp_permille, meas_comp, info->t_comp)));
        if (info->t_io > 0 && meas_copy_ps > 0)
            overlap->io_permille = (int32_t)std::min<int64_t>(
                8000, std::max<int64_t>(500, ratio_step(overlap->io_permille, meas_copy_ps, info->t_io)));
        return CF_OK;
    }
    // An extreme ran one engine alone: its ratio corrects that engine's own coefficients, and it
    // teaches nothing about contention -- what was learned about that ages: the factors move a
    // quarter of the way back to 1000, so that a bad sample cannot rule the hybrid out for good
    // (while an extreme is chosen the factors are not measured at all).
    auto relax = [](int32_t pm) { return pm >= 1000 ? pm - (pm - 1000) / 4 : pm + (1000 - pm) / 4; };
    overlap->comp_permille = relax(overlap->comp_permille);
    overlap->io_permille = relax(overlap->io_permille);
    if (info->kind == CF_PLAN_ALL_LOAD)
        return cf_cost_feedback(cost, 0, 0, info->t_io, meas_copy_ps);
    return cf_cost_feedback(cost, info->t_comp, meas_comp, 0, 0);
}

// ---------------------------------------------------------------- run-time scheduling
// The same two-pointer rule driven by actual progress instead of simulated clocks (Sec. 3.3,
// the progressive chunk-level update): an executor asks these two functions whenever one of
// its engines runs dry.  Costs come from the cost model, corrected by the ratios
// measured/predicted the executor has observed so far in the call (in permille).  Each engine
// takes a unit only if that does not push the end of the whole restoration out: with the
// other engine's time-to-finish T_other (everything unclaimed counted on its side), a unit of
// own cost x is taken iff (own busy time + x) <= T_other.

namespace {

struct DynState {
    std::vector<Units> req;
    int32_t scale_c, scale_io;
    int64_t sc(int64_t v) const { return (int64_t)(((__int128)v * scale_c) / 1000); }
    int64_t sio(int64_t v) const { return (int64_t)(((__int128)v * scale_io) / 1000); }
};

int dyn_setup(const char* who, const cf_cost_model* cost, const cf_plan_opts* opts, int32_t B,
              const int32_t* n_ctx, const int32_t* p_comp, const int32_t* p_io, int64_t t0, int64_t t1,
              int32_t scale_c, int32_t scale_io, DynState* st) {
    int rc = check(cost, opts, B, n_ctx, who);
    if (rc) return rc;
    if (B > 0 && (!p_comp || !p_io)) return cf::fail(CF_ERR_INVALID_ARG, "%s: null pointer array", who);
    if (t0 < 0 || t1 < 0 || scale_c <= 0 || scale_io <= 0)
        return cf::fail(CF_ERR_INVALID_ARG, "%s: times must be >= 0, scales > 0", who);
    st->req.resize(B);
    for (int i = 0; i < B; ++i) st->req[i] = make_units(*cost, *opts, n_ctx[i], mode_of(*opts, n_ctx[i]));
    st->scale_c = scale_c;
    st->scale_io = scale_io;
    return check_pointers(st->req, p_comp, p_io, who);
}

}  // namespace

extern "C" int cf_dynamic_io_pick(const cf_cost_model* cost, const cf_plan_opts* opts, int32_t B,
                                  const int32_t* n_ctx, const int32_t* p_comp, const int32_t* p_io,
                                  const uint8_t* compute_closed, int64_t io_backlog_ps,
                                  int64_t compute_busy_ps, int32_t scale_c_permille,
                                  int32_t scale_io_permille, int32_t* pick) {
    DynState st;
    int rc = dyn_setup("cf_dynamic_io_pick", cost, opts, B, n_ctx, p_comp, p_io, io_backlog_ps,
                       compute_busy_ps, scale_c_permille, scale_io_permille, &st);
    if (rc) return rc;
    if (!pick) return cf::fail(CF_ERR_INVALID_ARG, "cf_dynamic_io_pick: null pick");
    std::vector<int> pc(p_comp, p_comp + B), pio(p_io, p_io + B);
    int best = pick_io(st.req, pc, pio, n_ctx, opts->io_key);
    *pick = best;
    if (best < 0) return CF_OK;
    // units of a request the compute engine has closed are the channel's in any case
    if (compute_closed && compute_closed[best]) return CF_OK;
    // C: when the compute engine would be done if the channel took nothing more
    int64_t Crem = compute_busy_ps;
    for (int i = 0; i < B; ++i) {
        if (compute_closed && compute_closed[i]) continue;
        for (int u = pc[i]; u <= pio[i]; ++u) Crem += st.sc(st.req[i].a(u));
    }
    // the candidate: the far-end unit of `best`; layer-wise requests move together, so the
    // same layer of every open layer-wise request comes with it
    int64_t b = 0;
    if (st.req[best].mode == CF_LAYER_WISE) {
        for (int i = 0; i < B; ++i)
            if (pc[i] <= pio[i] && st.req[i].mode == CF_LAYER_WISE) b += st.sio(st.req[i].b[pio[i]]);
    } else {
        b = st.sio(st.req[best].b[pio[best]]);
    }
    if (io_backlog_ps + b > Crem) *pick = -1;      // the compute engine gets there sooner
    return CF_OK;
}

extern "C" int cf_dynamic_claim(const cf_cost_model* cost, const cf_plan_opts* opts, int32_t B,
                                const int32_t* n_ctx, const int32_t* p_comp, const int32_t* p_io,
                                const uint8_t* compute_closed, int64_t io_backlog_ps,
                                int64_t step_fixed_ps, int64_t compute_later_ps, int64_t step_cap_ps,
                                int32_t order,
                                int32_t scale_c_permille, int32_t scale_io_permille, int32_t max_units,
                                int32_t io_alone_permille, int32_t* take, int64_t* step_ps) {
    DynState st;
    int rc = dyn_setup("cf_dynamic_claim", cost, opts, B, n_ctx, p_comp, p_io, io_backlog_ps, step_fixed_ps,
                       scale_c_permille, scale_io_permille, &st);
    if (rc) return rc;
    if (B > 0 && !take) return cf::fail(CF_ERR_INVALID_ARG, "cf_dynamic_claim: null take");
    if (step_cap_ps < 0 || compute_later_ps < 0 || (order != CF_ORDER_CHEAPEST && order != CF_ORDER_SHORTEST) ||
        max_units < 0 || io_alone_permille < 0)
        return cf::fail(CF_ERR_INVALID_ARG, "cf_dynamic_claim: bad step cap, later work, order, unit limit or scale");
    const std::vector<Units>& req = st.req;

    // R: when the I/O channel would be done if the compute engine took nothing more
    int64_t R = io_backlog_ps;
    for (int i = 0; i < B; ++i)
        for (int u = p_comp[i]; u <= p_io[i]; ++u) R += st.sio(req[i].b[u]);

    // candidates: the next unit of every open token-wise request (behind the units the pass
    // already holds of it), and the next layer of all open layer-wise requests together (they
    // move through the layers as one packed batch; a step runs one layer of them)
    std::vector<int> group;
    int64_t grp_full = 0, grp_kv = 0;    // what the group's layer costs to run in full / up to its K/V write
    int64_t a_next = 0;
    bool has_next = true;
    std::vector<char> cand(B, 0);        // open token-wise requests
    for (int i = 0; i < B; ++i) {
        take[i] = 0;
        if (p_comp[i] > p_io[i] || (compute_closed && compute_closed[i])) continue;
        if (req[i].mode == CF_TOKEN_WISE) { cand[i] = 1; continue; }
        group.push_back(i);
        int64_t full = layer_pass_cost(*cost, 1, n_ctx[i], 0);
        grp_full += st.sc(full);
        grp_kv += st.sc(opts->kv_only_permille > 0 ? kv_only_cost(*cost, opts->kv_only_permille, n_ctx[i]) : full);
        if (p_comp[i] + 1 <= p_io[i]) a_next += st.sc(req[i].a(p_comp[i] + 1));
        else has_next = false;
    }
    // CHEAPEST: least recomputation per unit of I/O time saved first (a1/b1 < a2/b2);
    // SHORTEST: least recomputation still ahead first, so that requests finish one after the
    // other and their new turns can start while the channel works on the long ones; then by index
    struct Item { int first; bool group; int64_t a, b, rem; };
    auto before = [order](const Item& x, const Item& y) {
        if (order == CF_ORDER_SHORTEST) {
            if (x.rem != y.rem) return x.rem < y.rem;
        } else {
            __int128 l = (__int128)x.a * y.b, r = (__int128)y.a * x.b;
            if (l != r) return l < r;
        }
        return x.first < y.first;
    };
    // One pass of the rule.  The best-ranked candidate is taken if the pass, with it -- and with
    // compute_later_ps of work the compute engine has to do afterwards in any case -- still ends
    // no later than the channel would need for everything the pass so far leaves to it (the
    // pass starts out with step_fixed_ps of work it carries in any case); otherwise its request
    // is out.  cap: the pass stops growing once it is this long (0: never; it always gets its
    // first unit); limit: most units of one request (0: no limit); group_depth: how many layers
    // of the layer-wise group the pass may take.
    struct Pass { int64_t A, Bs; int g_taken; };
    auto greedy = [&](int64_t cap, int limit, int group_depth, int32_t* tk) {
        std::vector<int> front(p_comp, p_comp + B);
        std::vector<char> out(B, 0);
        std::vector<int32_t> n_taken(B, 0);
        Pass ps{step_fixed_ps, 0, 0};
        bool g_open = !group.empty();
        while (true) {
            if (cap > 0 && ps.A >= cap && ps.A > step_fixed_ps) break;
            bool have = false;
            Item best{};
            for (int i = 0; i < B; ++i) {
                if (!cand[i] || out[i] || front[i] > p_io[i] || (limit > 0 && n_taken[i] >= limit)) continue;
                Item it{i, false, st.sc(req[i].a(front[i])), st.sio(req[i].b[front[i]]),
                        req[i].a_prefix[p_io[i] + 1] - req[i].a_prefix[front[i]]};
                if (!have || before(it, best)) { best = it; have = true; }
            }
            bool g_cand = g_open && ps.g_taken < group_depth;
            if (g_cand)
                for (int i : group) g_cand = g_cand && p_comp[i] + ps.g_taken <= p_io[i];
            if (g_cand) {
                Item it{group[0], true, 0, 0, 0};
                for (int i : group) {
                    const int u = p_comp[i] + ps.g_taken;
                    it.a += st.sc(req[i].a(u));
                    it.b += st.sio(req[i].b[u]);
                    it.rem += req[i].a_prefix[p_io[i] + 1] - req[i].a_prefix[u];
                }
                if (!have || before(it, best)) { best = it; have = true; }
            }
            if (!have) break;
            if (ps.A + best.a + compute_later_ps <= R - ps.Bs) {
                ps.A += best.a;
                ps.Bs += best.b;
                if (best.group) ++ps.g_taken;
                else { ++n_taken[best.first]; ++front[best.first]; }
            } else if (best.group) {
                g_open = false;
            } else {
                out[best.first] = 1;
            }
        }
        if (tk) for (int i = 0; i < B; ++i) tk[i] = n_taken[i];
        return ps;
    };
    // contention: scale_io prices the channel beside a recomputing engine, io_alone the channel
    // on its own.  Nothing is taken unless recomputing pays for the slowdown it causes, judged
    // on everything the engine would take from this state (a capped step is the first of
    // several: what counts is where the engine ends up, not what one step holds).
    if (io_alone_permille > 0) {
        const Pass all = greedy(0, 0, INT32_MAX, nullptr);
        if (all.A > step_fixed_ps || all.g_taken > 0) {
            int64_t R_alone = io_backlog_ps;
            for (int i = 0; i < B; ++i)
                for (int u = p_comp[i]; u <= p_io[i]; ++u)
                    R_alone += (int64_t)(((__int128)req[i].b[u] * io_alone_permille) / 1000);
            if (std::max(all.A + compute_later_ps, R - all.Bs) >= std::max(step_fixed_ps + compute_later_ps, R_alone)) {
                if (step_ps) *step_ps = step_fixed_ps;
                return CF_OK;
            }
        }
    }
    const Pass step = greedy(step_cap_ps, max_units, 1, take);
    int64_t A = step.A;
    const int64_t Bs = step.Bs;
    const bool grp_taken = step.g_taken > 0;
    int64_t grp_a = 0;
    for (int i : group) grp_a += st.sc(req[i].a(p_comp[i]));
    if (grp_taken) {
        // 1: go through the whole layer (the next one looks worth taking too); 2: stop after
        // the K/V write, this is the group's last recomputed layer
        bool more = has_next && A + a_next + compute_later_ps <= R - Bs;
        for (int i : group) take[i] = more ? 1 : 2;
        // unit prices charge a layer's attention and MLP to the NEXT layer's unit; the step
        // itself runs this layer in full (1) or up to its K/V write (2)
        A += (more ? grp_full : grp_kv) - grp_a;
    }
    if (step_ps) *step_ps = A;
    return CF_OK;
}
