/*
 * cacheflow.h -- C ABI of the batched hybrid KV-cache restoration library for
 * AMD MI355X (gfx950).
 *
 * Problem (Sec. 3 of the CacheFlow paper): a batch of requests arrives, each
 * with a cached prefix of N_c tokens whose KV cache sits in external storage
 * (here: pinned host memory).  Restore every request's KV cache into GPU
 * memory as fast as possible by recomputing part of it on the GPU while the
 * rest is loaded over the host link, then run the new-turn prompt over the
 * restored cache to emit the first token (TTFT = restoration + that prefill).
 *
 * A restoration split for request i is (mode, k_tokens, layer_cut): cells
 * (token t < k_tokens, layer l < layer_cut) are recomputed; every other cell
 * of the request is loaded.  Token-wise mode (Sec. 3.1) yields layer_cut = L
 * and k_tokens a multiple of the chunk size; layer-wise mode yields
 * k_tokens = n_ctx and layer_cut = the cut-over layer.
 *
 * Conventions
 *  - Every call returns an int status: CF_OK (0) or a negative cf_status.
 *    No exception or abort crosses this boundary.  cf_last_error() returns a
 *    thread-local human-readable message for the last failure.
 *  - "host" pointers are ordinary CPU pointers; "device" pointers are HIP
 *    device memory on the current device.  The library never frees caller
 *    memory.  Objects it creates (cf_cache, cf_ctx) are destroyed by their
 *    *_destroy call.
 *  - Nothing here is thread-safe per object; use one object per thread.
 *
 * Matrix layout: every weight matrix is output-major, W[out][in], contiguous,
 * so y = x W^T.  Element type is the model dtype (float or bf16); norm gains
 * are always float.
 *
 * KV page layout (device pool and host blocks share it).  A page holds
 * page_tokens = 16 consecutive tokens of ONE layer of one request:
 *     K part: [kv_head][slot 0..15][head_dim]
 *     V part: [kv_head][head_dim][slot 0..15]      (V is stored transposed so
 *                                                   P*V reads 16-byte vectors)
 * K part first, then V part; page_bytes = 2*Hkv*16*hd*sizeof(elem).
 * Device pool : pool[layer][page_id]            (layer stride = n_pages pages)
 * Host block  : host_kv[layer][page 0..ceil(n_ctx/16)-1]  (layer-major, so a
 *               token suffix of one layer and a whole layer are contiguous).
 *               Slots past n_ctx in the last page are ignored.
 */
#ifndef CACHEFLOW_H
#define CACHEFLOW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CF_PAGE_TOKENS 16

enum cf_status {
    CF_OK = 0,
    CF_ERR_INVALID_ARG = -1,     /* null pointer, negative size, bad enum          */
    CF_ERR_INVALID_PLAN = -2,    /* split outside [0,n_ctx] x [0,L]                */
    CF_ERR_OUT_OF_PAGES = -3,    /* page pool exhausted                            */
    CF_ERR_HIP = -4,             /* a HIP call failed; see cf_last_error()         */
    CF_ERR_UNKNOWN_REQUEST = -5, /* req_id not allocated / already allocated       */
    CF_ERR_WORKSPACE = -6,       /* workspace too small / batch exceeds ctx limits */
    CF_ERR_UNSUPPORTED = -7      /* shape outside what the kernels were built for  */
};

enum cf_dtype { CF_F32 = 0, CF_BF16 = 1 };
enum cf_mode { CF_TOKEN_WISE = 0, CF_LAYER_WISE = 1 };
enum cf_io_key {
    CF_KEY_REMAINING_COST = 0,   /* Sec. 3.3: largest remaining recomputation cost */
    CF_KEY_REMAINING_CELLS = 1,  /* Sec. 3.3: "longest length to restore"           */
    CF_KEY_MARGINAL = 2          /* abstract: highest recompute saved per I/O time  */
};

const char* cf_status_str(int status);
const char* cf_last_error(void);

/* ------------------------------------------------------------------ planner
 * Batch-aware two-pointer scheduler, Algorithm 1 / Sec. 3.3, over an integer
 * cost model.  Pure host code: no GPU, no context.                          */

/* All picoseconds.  One layer of recompute over t tokens that start at
 * position p0 costs  f_c + alpha*t + beta*ceil(pairs/1024)  with
 * pairs = t*p0 + t*(t+1)/2 causal (query,key) pairs (Sec. 3.1: superlinear
 * T_comp with fixed overheads).  Loading one unit of `bytes` bytes costs
 * f_io + ceil(bytes*gamma / 2^20)  (Sec. 3.1: T_io linear, bandwidth-bound).
 * s_c / s_io are one-time start-up costs: the clock of an engine that takes
 * any unit at all starts there (recompute is batched over all requests, so
 * its launch-bound floor is paid once per batch, not once per chunk).       */
typedef struct cf_cost_model {
    int64_t f_c, alpha, beta, f_io, gamma, s_c, s_io;
} cf_cost_model;

typedef struct cf_plan_opts {
    int32_t chunk_tokens;             /* C (Sec. 3.1), > 0                           */
    int32_t l_delta;                  /* token-wise iff n_ctx >= l_delta (Alg. 1)    */
    int32_t n_layers;                 /* L                                           */
    int32_t kv_bytes_per_token_layer; /* 2*Hkv*hd*sizeof(elem)                       */
    int32_t force_mode;               /* -1 use l_delta; else a cf_mode for all      */
    int32_t io_key;                   /* cf_io_key                                   */
    int32_t kv_only_permille;         /* 0: every recomputed layer is priced in full.
                                         > 0: the executor stops a request's LAST
                                         recomputed layer after its K/V write, so
                                         that layer costs f_c + alpha*t*permille/1000
                                         (rounded up), no attention term: the top
                                         layer of a token-wise chunk, the first
                                         claimed layer of a layer-wise request (each
                                         further claim completes the layer below and
                                         adds a K/V-only one).  Set it to 1000 x the
                                         K/V-projection share of a layer's linear
                                         FLOPs                                       */
    int32_t boundary_bytes_per_token; /* 0: recompute starts from token ids.  > 0: a
                                         pipeline stage above layer 0 (Sec. 3.2)
                                         recomputes from cached stage-input hidden
                                         states, which cross the same host link as the
                                         KV: every recompute claim also costs the I/O
                                         channel ceil(tokens * this * gamma / 2^20) --
                                         the tokens of a token-wise chunk; all tokens of
                                         a layer-wise request at its first claimed
                                         layer, nothing after that.  float32 rows:
                                         4 * d_model                                  */
} cf_plan_opts;

typedef struct cf_split {
    int32_t mode;       /* cf_mode the planner used (informational for execution) */
    int32_t k_tokens;   /* tokens [0,k_tokens) are recomputed ...                  */
    int32_t layer_cut;  /* ... in layers [0,layer_cut); all other cells are loaded */
} cf_split;

typedef struct cf_claim {
    int32_t engine;     /* 0 = compute, 1 = I/O */
    int32_t request;
    int32_t unit;       /* chunk index (token-wise) or layer index (layer-wise)   */
} cf_claim;

typedef struct cf_plan_stats {
    int64_t t_comp, t_io, makespan;   /* predicted busy time of each engine, ps */
    int32_t n_claims;                 /* units scheduled = sum of unit counts   */
    int32_t n_trace;                  /* claims written to `trace`              */
} cf_plan_stats;

/* Plan a batch.  n_ctx: host int32[B] (each >= 0).  out_splits: host
 * cf_split[B].  trace (may be NULL): host cf_claim[trace_cap], receives the
 * claims in scheduling order (truncated at trace_cap).  stats may be NULL.
 * Errors: CF_ERR_INVALID_ARG on null/negative/zero chunk or layers.         */
int cf_restore_plan(const cf_cost_model* cost, const cf_plan_opts* opts, int32_t B,
                    const int32_t* n_ctx, cf_split* out_splits, cf_plan_stats* stats,
                    cf_claim* trace, int32_t trace_cap);

/* (t_comp, t_io) in ps of a given split vector under the cost model, with the
 * same unit accounting as the planner (k_tokens rounded up to whole chunks in
 * token-wise mode; with boundary_bytes_per_token set, t_io includes the
 * boundary rows of what is recomputed, also when nothing is loaded).  splits:
 * host cf_split[B] whose `mode` fields are used.                            */
int cf_plan_eval(const cf_cost_model* cost, const cf_plan_opts* opts, int32_t B,
                 const int32_t* n_ctx, const cf_split* splits, int64_t* t_comp,
                 int64_t* t_io);

/* Closed-loop correction after an executed batch (Sec. 3.3: scheduling adapts to
 * evolving resource availability): scales f_c, alpha, beta, s_c by
 * meas_comp/pred_comp and f_io, gamma, s_io by meas_io/pred_io, each ratio
 * clamped to [1/4, 4], rounding to nearest (alpha, gamma stay >= 1).  pred_* are
 * cf_plan_stats.t_comp / t_io of the plan that ran, meas_* the compute / copy
 * stream times of cf_timing, all in picoseconds; a side with pred or meas == 0
 * is left unchanged.  Pure host integer arithmetic.                          */
int cf_cost_feedback(cf_cost_model* cost, int64_t pred_comp, int64_t meas_comp, int64_t pred_io,
                     int64_t meas_io);

/* Compute-clock cost (ps) of the new-turn prefill of a batch: request i runs
 * n_new[i] tokens from position n_ctx[i] through n_layers layers, priced with
 * the recompute formula above (Sec. 3: TTFT = restoration + this prefill).
 * With the pipelined join that work shares the compute stream with the
 * recompute, so a caller adds the result to cf_cost_model.s_c before
 * cf_restore_plan; the planner itself schedules restoration only.  Pure host. */
int cf_prefill_cost(const cf_cost_model* cost, int32_t n_layers, int32_t B, const int32_t* n_ctx,
                    const int32_t* n_new, int64_t* out_ps);

struct cf_model_desc;

/* ------------------------------------------------------- planning policy
 * cf_restore_plan is Algorithm 1 and nothing else.  What a serving loop needs
 * around it -- the new turn's prefill on the compute clock, the K/V-only
 * price of a request's last recomputed layer, the slow-down the two engines
 * cause each other (Sec. 3.3: contention on shared resources), and the check
 * that the hybrid actually beats the two extremes of Sec. 4.1 (recompute
 * everything / load everything) -- is cf_plan_batch; cf_plan_feedback closes
 * the loop after the batch has run.  Pure host integer code.                */

/* Contention between the engines: while both run, every compute cost counts
 * comp_permille / 1000 of its isolated value and every load cost io_permille
 * / 1000 (1000 = no interference; rounded to nearest per coefficient).      */
typedef struct cf_overlap_model {
    int32_t comp_permille, io_permille;
} cf_overlap_model;

typedef struct cf_batch_plan_opts {
    int32_t chunk_tokens;      /* C (Sec. 3.1), > 0                                  */
    int32_t l_delta;           /* token-wise iff n_ctx >= l_delta (Alg. 1)           */
    int32_t force_mode;        /* -1 use l_delta; else a cf_mode for all             */
    int32_t io_key;            /* cf_io_key                                          */
    int32_t pipelined_join;    /* nonzero: the new-turn rows ride along with the
                                  recompute pass (cf_ctx_set_pipelined_join), so their
                                  cost starts the compute clock and only one layer of
                                  it is left when the last load lands; zero: the new
                                  turn runs after both engines are done               */
    int32_t stage_layers;      /* 0: the whole model; else the number of layers of the
                                  pipeline stage that is planned (cf_ctx_set_stage)   */
    int32_t stage_first_layer; /* first layer of that stage; above 0 the stage recomputes
                                  from boundary activations (float32 rows of d_model),
                                  whose transfer is charged to the I/O channel
                                  (cf_plan_opts.boundary_bytes_per_token)             */
} cf_batch_plan_opts;

enum cf_plan_kind { CF_PLAN_HYBRID = 0, CF_PLAN_ALL_LOAD = 1, CF_PLAN_ALL_RECOMPUTE = 2 };

typedef struct cf_batch_plan {
    int32_t kind;              /* cf_plan_kind of the splits returned                 */
    int32_t kv_only_permille;  /* K/V projection's share of a layer's linear FLOPs    */
    int32_t pipelined_join;    /* copied from the options (cf_plan_feedback reads it)  */
    int32_t reserved;
    int64_t prefill_ps;        /* isolated cost of the new-turn prefill               */
    int64_t t_comp, t_io;      /* predicted busy time of each engine under the plan
                                  returned (contention applied iff kind == hybrid;
                                  t_comp includes the prefill with the pipelined join) */
    int64_t ttft;              /* predicted time to the first token of the plan       */
    int64_t ttft_hybrid, ttft_all_load, ttft_all_recompute;   /* the three candidates */
} cf_batch_plan;

/* Plan a batch for cf_restore_batch.  n_new: host int32[B] or NULL (no new
 * turn).  Steps, all in integers:
 *  1. kv_only_permille = round(1000 * 2d(Hq+2Hkv)hd / linear FLOPs of a layer);
 *  2. prefill = sum_i cost of n_new[i] tokens from position n_ctx[i] through
 *     all layers (the recompute formula);
 *  3. hybrid candidate: Algorithm 1 under the cost model with the compute
 *     coefficients (f_c, alpha, beta, s_c, and the prefill) scaled by
 *     comp_permille and the load coefficients (f_io, gamma, s_io) by
 *     io_permille; with the pipelined join its compute clock starts at the
 *     scaled s_c + prefill;
 *  4. the extremes under the unscaled model: all-load (every unit loaded) and
 *     all-recompute (every unit recomputed);
 *  5. times of a candidate with start-up s, new-turn cost p, compute clock c
 *     at the end of its claims (0: none) and channel time t_io, nt = s + p
 *     (0 if p = 0) being the new turn as a pass of its own:
 *       pipelined join : t_comp = c (claims on top of s + p) or nt;
 *                        ttft = max(t_comp, t_io + p / L) -- one layer of the
 *                        new turn is left when the last load lands;
 *       sequential join: t_comp = c; ttft = max(c, t_io) + nt;
 *  6. the candidate with the smallest ttft is returned (ties: hybrid, then
 *     all-load); a hybrid that recomputes nothing or loads nothing is one of
 *     the extremes and is reported as such.
 * out_splits: host cf_split[B]; info may be NULL.                           */
int cf_plan_batch(const cf_cost_model* cost, const cf_overlap_model* overlap,
                  const struct cf_model_desc* desc, const cf_batch_plan_opts* opts, int32_t B,
                  const int32_t* n_ctx, const int32_t* n_new, cf_split* out_splits,
                  cf_batch_plan* info);

/* Closed loop after the batch has run (Sec. 3.3: scheduling follows evolving
 * resource availability).  meas_*_ps are cf_timing.compute_ms / copy_ms /
 * total_ms / compute_wait_ms of the call in picoseconds; the time the compute
 * stream waited for loads is taken off its measurement (it would otherwise
 * read as slow compute, move work to the channel and make the wait longer).  The compute measurement is
 * meas_compute_ps, except under the pipelined join when the call ended more
 * than 2 % after the copy stream did (the compute stream was the last to
 * finish, new turn included): then it is meas_total_ps.  A hybrid ran both
 * engines side by side, so its ratios measured / predicted correct the overlap
 * model (one call moves a factor by 5/4 or 4/5 at most: the first hybrid
 * after a cold start can measure far off on both engines at once; the factors
 * stay in [500, 8000]); an extreme ran one engine alone, so its ratio corrects
 * that engine's coefficients of the cost model (as cf_cost_feedback does), and
 * the overlap factors move a quarter of the way back to 1000: an extreme
 * teaches nothing about contention, nothing measures the factors while one is
 * chosen, and a bad sample must not rule the hybrid out for good.           */
int cf_plan_feedback(cf_cost_model* cost, cf_overlap_model* overlap, const cf_batch_plan* info,
                     int64_t meas_compute_ps, int64_t meas_copy_ps, int64_t meas_total_ps,
                     int64_t meas_wait_ps);

/* L_delta = min{N : T_token(N) <= T_layer(N)} (Sec. 3.1, adaptive strategy)
 * searched on multiples of chunk_tokens up to n_max; n_max + C if none.     */
int cf_derive_l_delta(const cf_cost_model* cost, const cf_plan_opts* opts, int32_t n_max,
                      int32_t* l_delta);

/* ------------------------------------------------- run-time scheduling steps
 * The two decisions of Alg. 1 taken against actual progress instead of
 * simulated clocks (Sec. 3.3: after each chunk the scheduler updates the
 * remaining cost of every request and re-ranks).  cf_restore_dynamic calls
 * them whenever one of its engines runs dry; they are pure host integer code.
 * State of request i: p_comp[i] = its next unit for the compute engine
 * (units below it are recomputed or being recomputed), p_io[i] = its next unit
 * for the I/O channel (units above it are loaded or being loaded); the request
 * is live while p_comp[i] <= p_io[i].  Units and their costs are those of
 * cf_restore_plan (chunks of C tokens, or layers).  p_comp in [0, units],
 * p_io in [-1, units-1], else CF_ERR_INVALID_ARG.
 *   compute_closed (host uint8[B], may be NULL = none): nonzero = the compute
 *                   engine can take no further unit of request i (a
 *                   layer-wise batch that has run its last layer K/V-only)
 *   io_backlog_ps : predicted time the I/O channel still needs for units it
 *                   has already claimed
 *   compute_busy_ps : predicted time left of the compute step that is running
 *   scale_*_permille : measured / predicted time of the compute steps and of
 *                   the loads seen so far in this call (1000 = as modelled);
 *                   every unit cost is multiplied by its scale (rounded down)
 * Both follow one rule: an engine takes a unit only if its own finish time
 * with it is no later than the time the OTHER engine would need for
 * everything still unclaimed -- taking it then cannot delay the end.
 *
 * cf_dynamic_io_pick: the live request whose far-end unit the channel would
 * load next has the largest key `opts->io_key` (default: recomputation still
 * ahead of it; ties to the longer context, then the lower index).  Its load
 * cost b (layer-wise: summed over all live layer-wise requests, which are
 * loaded layer by layer together) passes iff
 *   io_backlog + b <= compute_busy + sum of a over the unclaimed units of
 *                     requests that are not closed,
 * or if the request is closed.  *pick = that request, or -1 if none is live
 * or the unit is better left to the compute engine for now.                  */
int cf_dynamic_io_pick(const cf_cost_model* cost, const cf_plan_opts* opts, int32_t B,
                       const int32_t* n_ctx, const int32_t* p_comp, const int32_t* p_io,
                       const uint8_t* compute_closed, int64_t io_backlog_ps,
                       int64_t compute_busy_ps, int32_t scale_c_permille,
                       int32_t scale_io_permille, int32_t* pick);

enum cf_claim_order {
    CF_ORDER_CHEAPEST = 0,   /* least recompute cost per load cost saved (a/b) first   */
    CF_ORDER_SHORTEST = 1    /* least recomputation still ahead of the request first  */
};

/* cf_dynamic_claim: which units of the live, not closed requests the compute
 * engine takes for its next step (one step = those units run together,
 * layer-major).  With R = io_backlog + sum of the load costs b of all unclaimed
 * units (when the channel would be done on its own), the candidates are the
 * next unit of every open token-wise request -- the unit behind those the step
 * already holds of it, while it holds fewer than max_units of that request
 * (0: no limit) -- and ALL open layer-wise requests as ONE candidate, once per
 * step (they advance through the layers as a packed batch, one layer per
 * step; a = sum a_i, b = sum b_i).  Ranked by `order` (cf_claim_order; ties to
 * the lower index), the best candidate is taken if
 *        A + a + compute_later_ps <= R - Bs
 * (A, Bs: recompute and load cost of what the step already holds; A starts at
 * step_fixed_ps, the predicted cost of work the step carries in any case, such
 * as the new-turn prefill of requests that are already restored;
 * compute_later_ps is work the compute engine must do after this step whatever
 * it takes now, such as the new-turn prefill of the other requests); a request
 * whose candidate fails is out for this step.  This repeats until no candidate
 * is left or the step has reached step_cap_ps, if that is > 0 (a step always
 * gets a first unit).
 * Contention: scale_io_permille prices the channel while the compute engine
 * recomputes beside it, io_alone_permille (> 0) the channel when the compute
 * engine takes nothing.  What was chosen is given back (all take[i] = 0,
 * *step_ps = step_fixed_ps) unless it pays for the slowdown it causes:
 *   max(A + compute_later_ps, R - Bs)
 *        < max(step_fixed_ps + compute_later_ps, R at the scale io_alone_permille).
 * io_alone_permille = 0 skips the test.
 *   take[i] (host int32[B]) : token-wise: number of consecutive units taken,
 *                   from p_comp[i] on; layer-wise: 0 not taken, 1 taken, 2 taken
 *                   as the group's last layer -- the same test fails for the
 *                   group's following layer (or there is none), so the
 *                   executor stops this one after its K/V write
 *   step_ps (may be NULL)   : predicted duration of the step: step_fixed_ps +
 *                   the units taken, the layer-wise ones at what the step
 *                   really runs (the whole layer for 1, its K/V projection
 *                   for 2; unit prices charge a layer's attention and MLP to
 *                   the following unit)                                      */
int cf_dynamic_claim(const cf_cost_model* cost, const cf_plan_opts* opts, int32_t B,
                     const int32_t* n_ctx, const int32_t* p_comp, const int32_t* p_io,
                     const uint8_t* compute_closed, int64_t io_backlog_ps, int64_t step_fixed_ps,
                     int64_t compute_later_ps, int64_t step_cap_ps, int32_t order,
                     int32_t scale_c_permille, int32_t scale_io_permille, int32_t max_units,
                     int32_t io_alone_permille, int32_t* take, int64_t* step_ps);

/* --------------------------------------------------------------- page table
 * Paged KV cache bookkeeping (the serving substrate of Sec. 4.1).  Policy is
 * part of the contract: an allocation takes the ceil(n/16) lowest-numbered
 * free pages in ascending order.  Host-only object; `pool` is a device
 * pointer that is stored, never dereferenced by these calls (may be NULL for
 * host-only use).                                                           */
typedef struct cf_cache cf_cache;

/* n_pages = pool_bytes / (n_layers * page_bytes).                           */
int cf_cache_create(void* pool, size_t pool_bytes, int32_t n_layers, int32_t n_kv_heads,
                    int32_t head_dim, int32_t dtype, cf_cache** out);
void cf_cache_destroy(cf_cache* cache);
int cf_cache_n_pages(const cf_cache* cache);
int cf_cache_n_free(const cf_cache* cache);
size_t cf_cache_page_bytes(const cf_cache* cache);
/* Reserve pages for n_tokens (context + new tokens) of request req_id.
 * CF_ERR_UNKNOWN_REQUEST if req_id is live, CF_ERR_OUT_OF_PAGES if short.   */
int cf_cache_alloc(cf_cache* cache, uint64_t req_id, int32_t n_tokens);
int cf_cache_free(cf_cache* cache, uint64_t req_id);
/* Copy the request's page ids to out[0..cap); *n_pages receives the count
 * (even when cap is too small, in which case nothing is written past cap).  */
int cf_cache_page_table(const cf_cache* cache, uint64_t req_id, int32_t* out, int32_t cap,
                        int32_t* n_pages);

/* Bytes of one request's host KV block for n_ctx tokens.                    */
size_t cf_host_kv_bytes(int32_t n_layers, int32_t n_kv_heads, int32_t head_dim, int32_t dtype,
                        int32_t n_ctx);

/* ----------------------------------------------------------------- executor */
typedef struct cf_model_desc {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t dtype;                 /* cf_dtype of weights, activations fed to GEMMs, KV */
    float rope_base;               /* rotate-half RoPE, theta_j = base^(-2j/hd)         */
    float rms_eps;
} cf_model_desc;

typedef struct cf_layer_weights {  /* device pointers, borrowed for the ctx lifetime */
    const float* attn_norm;        /* [d]                                  */
    const void* wqkv;              /* [(Hq+2Hkv)*hd, d]: Q heads, K heads, V heads */
    const void* wo;                /* [d, Hq*hd]                           */
    const float* mlp_norm;         /* [d]                                  */
    const void* w_gate;            /* [ffn, d]                             */
    const void* w_up;              /* [ffn, d]                             */
    const void* w_down;            /* [d, ffn]                             */
} cf_layer_weights;

typedef struct cf_weights {
    const void* embed;             /* device [vocab, d]                    */
    const void* lm_head;           /* device [vocab, d]                    */
    const float* final_norm;       /* device [d]                           */
    const cf_layer_weights* layers;/* HOST array of n_layers entries (copied) */
} cf_weights;

typedef struct cf_ctx_opts {
    int32_t max_batch;             /* most requests per cf_restore_batch           */
    int32_t max_tokens;            /* most packed tokens in one forward phase:
                                      max(sum k_i, sum n_new) over calls           */
    int32_t max_positions;         /* RoPE table length: max n_ctx + n_new         */
    int32_t chunk_rows;            /* token rows per kernel pass (0 = default)     */
    int64_t staging_bytes;         /* host->device staging ring (0 = default)      */
} cf_ctx_opts;

typedef struct cf_ctx cf_ctx;

/* Device workspace the context needs; the caller allocates it (e.g. with
 * torch) and passes it to cf_ctx_create.                                    */
int cf_workspace_bytes(const cf_model_desc* desc, const cf_ctx_opts* opts, size_t* bytes);

/* compute_stream / copy_stream: hipStream_t handles (as void*), default
 * priority, distinct for overlap.  workspace: device memory of at least
 * cf_workspace_bytes, 256-byte aligned, owned by the caller and borrowed
 * until cf_ctx_destroy.  Creates one more stream and its events, allocates
 * small pinned host buffers and uploads the RoPE table; no device allocation. */
int cf_ctx_create(const cf_model_desc* desc, const cf_weights* weights, const cf_ctx_opts* opts,
                  void* workspace, size_t workspace_bytes, void* compute_stream,
                  void* copy_stream, cf_ctx** out);
void cf_ctx_destroy(cf_ctx* ctx);

typedef struct cf_request {
    uint64_t req_id;               /* must be allocated in the cache with
                                      >= n_ctx + n_new tokens                      */
    const int32_t* ctx_tokens;     /* host int32[n_ctx]; only [0,k_tokens) is read */
    int32_t n_ctx;
    int32_t n_new;
    const void* host_kv;           /* host block (layout above); pinned, device-mapped
                                      memory (hipHostMalloc) selects the direct load
                                      path, pageable memory the staged one; may be
                                      NULL iff the split loads nothing             */
    const int32_t* new_tokens;     /* host int32[n_new]                            */
    const float* boundary_h;       /* host float[n_ctx][d_model] (pinned for speed):
                                      the hidden states entering the stage's first
                                      layer (Sec. 3.2, boundary activations); rows
                                      [0,k_tokens) are read.  Needed iff the context
                                      restores a stage that starts above layer 0
                                      (cf_ctx_set_stage) and the split recomputes;
                                      NULL otherwise                               */
} cf_request;

typedef struct cf_timing {
    float restore_ms;     /* call start -> both streams done with restoration    */
    float compute_ms;     /* call start -> end of the last recomputed layer on the
                             compute stream (pipelined join: the new-turn rows of
                             the layers up to there included)                    */
    float copy_ms;        /* call start -> last loaded cell in place (copy stream) */
    float suffix_ms;      /* total_ms - restore_ms: what the new-turn prefill and
                             the logits add after restoration                    */
    float total_ms;       /* call start -> logits ready (batch TTFT)             */
    float compute_wait_ms;/* of compute_ms, time the compute stream stood still
                             waiting for loaded KV (pipelined join: the new-turn
                             attention of a layer waits for that layer's loads;
                             waits above the last recomputed layer lie after
                             compute_ms and are not counted); a compute stream
                             that ends late because it WAITED is not slow         */
    double recompute_flops; /* algorithmic: linear layers + causal pairs needed  */
    double suffix_flops;
    int64_t loaded_bytes; /* KV bytes that crossed the host link                 */
    int64_t recomputed_cells; /* (token, layer) cells recomputed                  */
    int64_t loaded_cells;
} cf_timing;

/* Restore the batch under the given splits, then prefill each request's new
 * tokens over its restored cache and write first-token logits.
 *   reqs, splits : host arrays of B entries; any split with 0<=k<=n_ctx and
 *                  0<=cut<=L is accepted (planner's, forced, all-recompute,
 *                  all-load).
 *   logits_out   : DEVICE float[B][vocab], or NULL to skip the new-token phase
 *                  (n_new may then be 0).
 *   timing       : host, may be NULL.
 * Blocking: returns after logits are ready and both streams are idle.
 * Recompute runs on the compute stream, layer-major over the whole batch;
 * loads run on the copy stream (pinned host -> pages by a load kernel, or
 * host -> staging -> page scatter; see cf_ctx_set_load_path).
 * max(sum k_i + sum n_new) must not exceed the context's max_tokens.         */
int cf_restore_batch(cf_ctx* ctx, cf_cache* cache, int32_t B, const cf_request* reqs,
                     const cf_split* splits, float* logits_out, cf_timing* timing);

typedef struct cf_dynamic_stats {
    int32_t compute_steps;      /* steps the compute engine ran (new-turn ones too) */
    int32_t compute_units;      /* units it claimed (chunks, or request-layers)    */
    int32_t io_units;           /* loads the channel claimed (each one launch or a
                                   group of transfers), the planned tail's layers
                                   included                                        */
    int32_t scale_c_permille;   /* measured / predicted at the end of the call:
                                   compute engine,                                 */
    int32_t scale_io_permille;  /* channel beside a recomputing compute engine,    */
    int32_t scale_io_alone_permille;   /* channel on its own                       */
    int32_t planned_tail;       /* 1: the call ended with the planned tail (see below) */
    int32_t last_step_merged;   /* 1: the last recompute step carried the planned
                                   tail and every outstanding new turn itself      */
    double compute_gap_ms;      /* compute stream idle between steps (host decides
                                   the next step only when the last one is done)   */
} cf_dynamic_stats;

typedef struct cf_dynamic_opts {
    int64_t step_cap_ps;        /* a compute step stops taking units once its predicted
                                   duration reaches this (0: no cap); shorter steps decide
                                   later and finish requests one after the other, longer
                                   ones run larger GEMMs                              */
    int32_t order;              /* cf_claim_order of the compute engine's candidates  */
    int32_t units_per_request;  /* most consecutive units of one token-wise request a
                                   step may take (0: no limit; 1: a step holds one chunk
                                   of each request it takes)                          */
    int32_t overlap_comp_permille;   /* cf_overlap_model of the machine (cf_calibrate_overlap,
                                   cf_plan_feedback).  If either is > 0 the context's ratios */
    int32_t overlap_io_permille;     /* measured / predicted restart in this call: the two
                                   engines' side-by-side ratios from these factors (0 reads
                                   as 1000), the channel's own from 1000.  Both 0: the ratios
                                   carry on from the context's previous call (a new context
                                   starts at 1000).  Pass them with a new or changed cost
                                   model, leave them 0 while the same one stays in use.   */
} cf_dynamic_opts;

/* Restore a batch WITHOUT a precomputed split: the two engines claim units at
 * run time (Sec. 3.3, progressive chunk-level scheduling).  The I/O channel
 * keeps one unit in flight plus as many more as it takes to have about 2 ms
 * of predicted work queued (at most 4), each picked by cf_dynamic_io_pick when
 * a slot frees up; the compute engine asks cf_dynamic_claim each time its
 * previous step has completed (HIP events, polled by the calling thread) and
 * runs the units it gets as one packed step: the claimed chunks of token-wise
 * requests through all layers, and the next layer of the layer-wise requests,
 * whose hidden states stay in the workspace from step to step.  A request
 * whose cache is complete (pointers crossed, its loads landed) has its
 * new-turn rows prefilled in the very next step, beside whatever that step
 * recomputes.  Once the compute engine, idle, declines every unit that is
 * left, the rest of the schedule is known and is laid out like a planned
 * restore (the planned tail): the channel loads all unclaimed cells layer by
 * layer from the bottom, and the new turn of every request not yet prefilled
 * runs beside those loads, its attention in layer l waiting for layer l only.
 * The logits follow when the last request is through.
 *   cost, opts : the cost model seeds the predictions; the ratios measured /
 *                predicted are tracked inside the call -- the compute engine's,
 *                the channel's while a recompute step runs beside it, and the
 *                channel's on its own -- and carried over to the context's
 *                next call (see cf_dynamic_opts).  opts->chunk_tokens
 *                must be a multiple of 16 (page size); modes by
 *                opts->force_mode / l_delta as in cf_restore_plan.
 *   reqs       : as for cf_restore_batch; every request with n_ctx > 0 needs
 *                ctx_tokens and pinned, device-mapped host_kv (the direct
 *                load path is the only one used here).
 *   splits_out : host cf_split[B], the split that resulted (token-wise:
 *                k = chunks recomputed x C, cut = L; layer-wise: k = n_ctx,
 *                cut = layers recomputed); the restored cache and the logits
 *                are those of cf_restore_batch under these splits up to the
 *                order of floating-point summation (chunks are recomputed
 *                one step at a time, over the pages of the chunks before).
 *   dyn        : may be NULL = {0, CF_ORDER_CHEAPEST, 0, 0, 0}.
 *   logits_out, timing : as for cf_restore_batch.  stats may be NULL.
 * The context must cover the whole model (no cf_ctx_set_stage restriction).
 * Rows: (tokens of all layer-wise requests) + (token-wise requests x C) +
 * sum n_new must fit max_tokens.  timing->compute_ms marks the end of the last
 * step that recomputed anything.  Blocking.                                   */
int cf_restore_dynamic(cf_ctx* ctx, cf_cache* cache, int32_t B, const cf_request* reqs,
                       const cf_cost_model* cost, const cf_plan_opts* opts,
                       const cf_dynamic_opts* dyn, float* logits_out, cf_split* splits_out,
                       cf_timing* timing, cf_dynamic_stats* stats);

/* Copy a request's first n_ctx tokens of KV from its pages to a host block
 * of cf_host_kv_bytes(n_ctx) bytes in the host layout (whole pages; the
 * eviction direction of Sec. 3's external storage, and how host KV is
 * manufactured for the large configurations).  Blocking.  If the block is
 * pinned, device-mapped memory a store kernel writes it over the host link in
 * one launch; otherwise (or with load path 1) pages are gathered into the
 * staging buffer and copied out layer by layer.  Same bytes either way
 * (slots past n_ctx in the last page are written as zero).                  */
int cf_offload(cf_ctx* ctx, cf_cache* cache, uint64_t req_id, int32_t n_ctx, void* host_kv);

/* cf_offload for callers that cannot allocate device memory (code under HIP
 * graph capture set-up, tight serving loops, harnesses that forbid hipMalloc):
 * the same result as cf_offload's staged path -- whole pages in the host
 * layout, slots past n_ctx in the last page zero -- but the device scratch it
 * needs (the request's page table, one job record, one 16 MiB staging slot)
 * lives in a static device array of the library (16 MiB + 64 KiB, held on every
 * GPU the library runs on until the process ends) instead of the context's
 * workspace.  The call allocates nothing, on the device or through the HIP
 * runtime: it uses the context's compute stream and pinned metadata buffer,
 * and host_kv must be PINNED host memory (hipHostMalloc; a copy into pageable
 * memory would go through buffers the runtime allocates), else
 * CF_ERR_INVALID_ARG.  Limits: n_ctx <= cf_offload_static_max_tokens()
 * (16320 pages = 261120 tokens) and page_bytes <= 16 MiB, else
 * CF_ERR_WORKSPACE.  Blocking.  Every call on a GPU shares that GPU's array,
 * which keeps the previous call's contents (each call overwrites what it
 * reads back, nothing needs to start at zero): calls that overlap on one GPU,
 * from any thread or context, race.                                          */
int cf_offload_static(cf_ctx* ctx, cf_cache* cache, uint64_t req_id, int32_t n_ctx, void* host_kv);
size_t cf_offload_static_max_tokens(void);

/* Time a large pinned host->device copy on the copy stream: the bandwidth
 * roofline of the load path.  host_buf pinned, dev_buf device, both >= bytes. */
int cf_measure_h2d(cf_ctx* ctx, const void* host_buf, void* dev_buf, size_t bytes, int32_t reps,
                   double* gb_per_s);

/* Fit the integer cost model on this GPU (Sec. 3.1: T_comp and T_io come from
 * profiling): times recompute passes of three sizes and two host->device loads
 * through cf_restore_batch on scratch pages of `cache` (needs free pages for
 * min(8192, ctx limits) tokens; request ids 0xCA11B000.. are used and freed)
 * with the pinned scratch block `host_buf` (>= cf_host_kv_bytes of that many
 * tokens; contents irrelevant), solves for the coefficients and rounds them
 * to integer picoseconds.  A hardware measurement: not reproducible bit for
 * bit, so plans are only comparable given the same table.                  */
int cf_calibrate(cf_ctx* ctx, cf_cache* cache, void* host_buf, size_t host_bytes,
                 cf_cost_model* out);

/* First estimate of the overlap model (Sec. 3.3, contention): one batch in
 * which one scratch request is recomputed in full while another is loaded in
 * full, both of min(8192, ctx limits) tokens, timed against what `cost` (from
 * cf_calibrate on the same context) predicts for each alone.  The load is
 * short beside the recompute, so the compute factor is a rough figure;
 * cf_plan_feedback refines both from real batches.  Needs free pages for twice
 * that many tokens; host_buf as for cf_calibrate.                            */
int cf_calibrate_overlap(cf_ctx* ctx, cf_cache* cache, void* host_buf, size_t host_bytes,
                         const cf_cost_model* cost, cf_overlap_model* out);

/* Per-kernel timing inside cf_restore_batch, from HIP event pairs recorded
 * around each selected launch on the stream it is launched on.             */
enum cf_kernel {
    CF_K_GEMM_QKV = 0, CF_K_GEMM_OPROJ = 1, CF_K_GEMM_GATE_UP = 2, CF_K_GEMM_DOWN = 3,
    CF_K_GEMM_LM_HEAD = 4, CF_K_ATTENTION = 5, CF_K_RMSNORM = 6, CF_K_ROPE_WRITE = 7,
    CF_K_EMBED = 8, CF_K_PAGE_SCATTER = 9, CF_K_H2D_COPY = 10, CF_N_KERNELS = 11
};
typedef struct cf_kernel_stat {
    int32_t kernel;      /* cf_kernel                                              */
    int32_t launches;
    double total_ms;     /* sum of event-pair durations                            */
    double work;         /* algorithmic FLOPs (GEMMs: 2MNK, attention: 4*Hq*hd per
                            causal pair) or bytes (other kernels: bytes they must
                            move; copies: bytes over the link)                      */
} cf_kernel_stat;
/* kernel_mask: bit i selects cf_kernel i; 0 turns profiling off (default). */
int cf_ctx_profile(cf_ctx* ctx, uint32_t kernel_mask);
/* out: host cf_kernel_stat[CF_N_KERNELS], totals since the last reset.     */
int cf_ctx_profile_read(cf_ctx* ctx, cf_kernel_stat* out, int32_t reset);

/* Final hidden state (residual stream after the last layer, before the final
 * norm) of each request's last new token, as left by the most recent
 * cf_restore_batch that produced logits for B requests.  out: host
 * float[B][d_model].  For parity checks of the final norm and LM head at
 * sizes where the CPU cannot run the whole context.                         */
int cf_read_final_hidden(cf_ctx* ctx, int32_t B, float* out_host);

/* Join mode.  on != 0 (default): pipelined join -- the new-turn rows are packed
 * with the recompute rows into one layer-major pass, loads are issued layer by
 * layer from the bottom, and only the attention of the new-turn rows of layer l
 * waits for layer l's loads, so the first-token prefill overlaps restoration.
 * on == 0: sequential join -- recompute || load (top layer first), then wait
 * for both, then the new-turn prefill.  Results are identical.               */
int cf_ctx_set_pipelined_join(cf_ctx* ctx, int32_t on);

/* Load path (the I/O side of Sec. 3.1's two pointers).  path 0 (default):
 * automatic -- for pinned, device-mapped host blocks the direct path, in which
 * runs of whole pages whose pool slots are consecutive and that are at least
 * 4 MiB long go as single DMA transfers straight into the pool (no kernel, no
 * compute unit taken from the GEMMs running beside the loads) and everything
 * else -- scattered or short runs, partly loaded pages -- through the load
 * kernel; the staged path for other host memory.  path 2: direct -- a load
 * kernel of n_workgroups resident workgroups (0 keeps the current value,
 * default 8, at most 1024) reads the host block over the host link and writes
 * the KV pages itself, one launch per layer; cf_restore_batch then fails with
 * CF_ERR_INVALID_ARG for a host block that is not device-mapped.  path 1:
 * staged -- DMA transfers into the workspace's staging slots followed by a
 * scatter kernel (works for any host memory; pageable memory is slow).
 * Results are identical.                                                    */
int cf_ctx_set_load_path(cf_ctx* ctx, int32_t path, int32_t n_workgroups);

/* Stage restriction (Sec. 3.2, Eq. 2: with S pipeline stages every stage
 * restores its own layers independently, from the hidden states it cached at
 * its input).  After cf_ctx_set_stage(ctx, b, e), 0 <= b < e <= n_layers,
 * cf_restore_batch touches only layers [b, e): a split's layer_cut is counted
 * from b (0..e-b), recompute of tokens [0,k) starts from cf_request.boundary_h
 * instead of the token embeddings when b > 0, loads cover the stage's layers
 * of the host block (which keeps the full-model layout), and logits_out must
 * be NULL unless the stage is the whole model.  Plan a stage with
 * cf_plan_opts.n_layers = e - b.  Default: the whole model.                  */
int cf_ctx_set_stage(cf_ctx* ctx, int32_t layer_begin, int32_t layer_end);

/* One-shot capture of boundary activations: during the NEXT cf_restore_batch,
 * when the compute stream reaches `layer` (model numbering), the residual
 * stream of the packed rows active in that layer is copied to dev_out, a
 * DEVICE float[cap_rows][d_model].  Packed row order: recompute rows of the
 * requests in order of descending layer cut (call order among equals), then
 * the new-turn rows when logits are produced.  This is how a stage's
 * cf_request.boundary_h is manufactured from a full prefill.  The call fails
 * with CF_ERR_WORKSPACE if more than cap_rows rows are active.               */
int cf_ctx_capture_boundary(cf_ctx* ctx, int32_t layer, float* dev_out, int64_t cap_rows);

/* One-shot sampling of the residual stream for teacher-forced parity checks
 * at sizes where the CPU cannot run the whole context (the scale plan's
 * per-layer check: a layer's K/V cells, its attention half and its MLP half
 * are recomputed on the CPU from the hidden state the GPU fed them, so errors
 * do not accumulate over depth).  During the NEXT cf_restore_batch, for every
 * layer l of the context's stage (l = 0 .. L-1, counted from the stage's
 * first layer) the residual stream of the listed packed rows is copied
 *   to dev_out[2l][j][0..d_model)    as it enters the layer, and
 *   to dev_out[2l+1][j][0..d_model)  as it enters the layer's MLP half (input
 *                                    plus the projected attention output);
 * what leaves the last layer goes to dev_out[2L][j].  A listed row leaves a
 * slot untouched where it is not active: a recompute row at or above its
 * layer cut has no entry, and in its last recomputed layer, which stops after
 * the K/V write, neither an MLP input nor (for l = L-1) a final state; only
 * new-turn rows have all 2L+1 slots.
 *   packed_rows : host int32[n_rows] (copied), packed row order as for
 *                 cf_ctx_capture_boundary; n_rows <= 4096; 0 cancels
 *   dev_out     : DEVICE float[2L+1][n_rows][d_model]
 * With the sequential join only the recompute phase is sampled.             */
int cf_ctx_capture_rows(cf_ctx* ctx, const int32_t* packed_rows, int32_t n_rows, float* dev_out);

/* Emulation of a slower storage tier or link (the bandwidth ablation of the
 * paper's evaluation): with gb_per_s > 0 the copy stream of cf_restore_batch
 * is held after every transfer unit until the bytes moved so far would have
 * crossed a link of that rate (a one-lane wait kernel on the constant-rate
 * device clock; bounded spin).  0 (default) switches it off.  cf_calibrate run
 * afterwards measures the throttled link; cf_measure_h2d always measures the
 * real one.  Results are unaffected.                                        */
int cf_ctx_set_link_throttle(cf_ctx* ctx, double gb_per_s);

/* Kernel selection for a context: simple_only != 0 routes every step through
 * the plain float-FMA kernels (the float32 path); 0 (default) uses the MFMA
 * kernels wherever they support the shape.  For kernel-vs-kernel GPU tests. */
int cf_ctx_set_kernel_set(cf_ctx* ctx, int32_t simple_only);

/* Test hook for the error path: the nth_check-th status check that
 * cf_restore_batch makes AFTER it has started to enqueue work (1 = the first)
 * reports a failure as if the HIP call had returned an error; the call then
 * has to wait for all three streams before it returns CF_ERR_HIP, because the
 * work already enqueued reads caller memory.  One shot: cleared by the next
 * cf_restore_batch whether it fires or not.  0 switches it off.  Nothing on
 * the GPU is made to fail.                                                  */
int cf_ctx_inject_failure(cf_ctx* ctx, int32_t nth_check);

/* Test hook: force the block tile of every MFMA GEMM the library launches from
 * now on, wherever the shape allows it (0 = the library's own choice, the
 * default; 256 / 128 / 64 = that tile; 257 = 256 with the quartered tail).
 * Process-wide.  The tile never changes a result bit; the hook exists so that
 * small end-to-end tests can run on the tile the full-size runs take.
 * cf_op_gemm sets and clears it for its own launches.                       */
int cf_debug_force_gemm_tile(int32_t tile);

/* One GEMM of the recompute path, exposed for parity tests and roofline
 * measurement: acc[M,N] = A[M,K] * W[N,K]^T with A, W (and W2) device arrays
 * in the context's model dtype, float accumulation, then the epilogue
 *   epi 0: Cf = acc          epi 1: Cf += acc           (Cf device float[M,N])
 *   epi 2: Dt = (dtype)acc   epi 3: Dt = (dtype)(silu(acc) * (A*W2^T))
 *                                                        (Dt device dtype[M,N])
 * (the QKV / O-proj and down-proj / - / gate-up steps of a layer).
 * impl 0 = what cf_restore_batch would pick, 1 = plain FMA kernel, 2 = MFMA
 * kernel with its own tile choice, 3 / 4 / 5 = MFMA kernel forced to 256x256 /
 * 128x128 / 64x64 block tiles (epi 3 has no 64x64 tile and takes 128x128;
 * CF_ERR_UNSUPPORTED if MFMA does not take the shape), 6 = 256x256 tiles
 * whose last partial round of tiles is covered by 128x128 tiles in the same
 * launch wherever the tile count allows it (what impl 0 picks for large
 * problems; the plain 256x256 launch otherwise).  Runs `reps`
 * times on the compute stream, blocks, and returns the mean time per run
 * from HIP events in *avg_ms (may be NULL).                                 */
int cf_op_gemm(cf_ctx* ctx, const void* A, const void* W, const void* W2, float* Cf, void* Dt,
               int32_t M, int32_t N, int32_t K, int32_t epi, int32_t impl, int32_t reps,
               float* avg_ms);

#ifdef __cplusplus
}
#endif
#endif /* CACHEFLOW_H */
