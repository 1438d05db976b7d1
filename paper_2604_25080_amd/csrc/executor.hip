// Executor of batched hybrid KV-cache restoration (Sec. 3.1-3.3): for every
// request the cells (token < k, layer < cut) are recomputed on the compute
// stream, layer-major over the whole batch, while all other cells are copied
// from pinned host memory and scattered into the same pages on the copy
// stream; after the join the new-turn tokens are prefilled over the restored
// pages and the first-token logits are produced (TTFT = restoration + that
// prefill).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <climits>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <deque>
#include <functional>
#include <thread>
#include <vector>

#include "cf_common.h"
#include "kernels.h"

namespace cf {

#define CF_HIP(call)                                                                     \
    do {                                                                                 \
        hipError_t e_ = (call);                                                          \
        if (e_ != hipSuccess)                                                            \
            return cf::fail(CF_ERR_HIP, "%s:%d %s -> %s", __FILE__, __LINE__, #call,     \
                            hipGetErrorString(e_));                                      \
    } while (0)

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

constexpr int PAGE_MOVE_SPLIT = 4;       // blocks per page in the page mover
constexpr int N_STAGING_SLOTS = 2;

struct Carve {
    size_t rope, h, dl, a, qkv, q, o, act, a_last, h_last, attn_part, staging, meta, total;
    size_t staging_bytes, meta_bytes;
    int chunk_rows;
    size_t pace;
};

static int carve_workspace(const cf_model_desc& m, const cf_ctx_opts& o, Carve* c) {
    if (m.n_layers <= 0 || m.d_model <= 0 || m.n_q_heads <= 0 || m.n_kv_heads <= 0 ||
        m.head_dim <= 0 || m.d_ffn <= 0 || m.vocab <= 0 || (m.dtype != CF_F32 && m.dtype != CF_BF16))
        return fail(CF_ERR_INVALID_ARG, "model descriptor has a non-positive field or bad dtype");
    if (m.n_q_heads % m.n_kv_heads != 0 || (m.head_dim != 64 && m.head_dim != 128) ||
        m.d_model % 8 != 0 || m.d_model > 8192 || m.d_ffn % 8 != 0)
        return fail(CF_ERR_UNSUPPORTED,
                    "need Hq %% Hkv == 0, head_dim in {64,128}, d_model %% 8 == 0 and <= 8192, "
                    "d_ffn %% 8 == 0");
    if (o.max_batch <= 0 || o.max_tokens <= 0 || o.max_positions <= 0 || o.chunk_rows < 0 ||
        o.staging_bytes < 0)
        return fail(CF_ERR_INVALID_ARG, "context options must be positive");
    size_t es = elem_bytes(m.dtype);
    int chunk = o.chunk_rows > 0 ? o.chunk_rows : 16384;
    chunk = (int)align_up((size_t)std::min(chunk, std::max(o.max_tokens, 1)), 256);
    size_t pb = page_bytes(m.n_kv_heads, m.head_dim, m.dtype);
    size_t stg = o.staging_bytes > 0 ? (size_t)o.staging_bytes : ((size_t)128 << 20);
    stg = std::max(stg / N_STAGING_SLOTS / pb, (size_t)1) * pb * N_STAGING_SLOTS;
    size_t qcols = (size_t)(m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
    size_t pages_per_req = (size_t)o.max_positions / CF_PAGE_TOKENS + 2;
    size_t meta = (size_t)2 * 12 * o.max_tokens                       // ids, positions, slots
                  + (size_t)4 * o.max_batch * pages_per_req            // page tables
                  + (size_t)(sizeof(AttnWork) + sizeof(AttnCombine)) *
                        (2 * ((size_t)o.max_tokens / ATTN_BLOCK_ROWS) + 4 * (size_t)o.max_batch +
                         4 * ((size_t)o.max_tokens / chunk + 2) + 2 * ATTN_MAX_PART_BLOCKS)
                  + (size_t)sizeof(PageJob) * ((size_t)o.max_batch * m.n_layers * 2 + 4096)
                  // run-time scheduling: one job per (chunk of >= 256 tokens, layer) of every request
                  + (size_t)sizeof(PageJob) * (size_t)o.max_batch * ((size_t)o.max_positions / 256 + 2) * m.n_layers +
                  (size_t)8 * o.max_batch + (1 << 16);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes, 256); return at; };
    c->rope = take((size_t)o.max_positions * (m.head_dim / 2) * sizeof(float2));
    c->h = take((size_t)o.max_tokens * m.d_model * 4);
    c->dl = take((size_t)o.max_tokens * m.d_model * 4);
    c->a = take((size_t)chunk * m.d_model * es);
    c->qkv = take((size_t)chunk * qcols * 4);
    c->q = take((size_t)chunk * m.n_q_heads * m.head_dim * es);
    c->o = take((size_t)chunk * m.n_q_heads * m.head_dim * es);
    c->act = take((size_t)chunk * m.d_ffn * es);
    c->a_last = take((size_t)o.max_batch * m.d_model * es);
    c->h_last = take((size_t)o.max_batch * m.d_model * 4);
    c->attn_part = take(attn_part_bytes(m.head_dim));
    c->staging = take(stg);
    c->meta = take(meta);
    c->pace = take(256);
    c->total = off;
    c->staging_bytes = stg;
    c->meta_bytes = meta;
    c->chunk_rows = chunk;
    return CF_OK;
}

}  // namespace cf

using namespace cf;

static int static_scratch_of_current_device(char** out);

struct cf_ctx {
    cf_model_desc m;
    cf_ctx_opts opts;
    cf_weights w;
    std::vector<cf_layer_weights> layers;
    hipStream_t cs = nullptr, ps = nullptr, ss = nullptr;  // compute, copy, scatter
    bool own_ss = false;
    char* ws = nullptr;
    Carve cv;
    char* meta_host = nullptr;
    hipEvent_t ev_start = nullptr, ev_meta = nullptr, ev_comp = nullptr, ev_copy = nullptr,
               ev_end = nullptr, ev_scat = nullptr, ev_t0 = nullptr, ev_t1 = nullptr, ev_q2 = nullptr;
    hipEvent_t ev_filled[N_STAGING_SLOTS] = {}, ev_free[N_STAGING_SLOTS] = {};
    bool simple_only = false;
    bool pipelined = true;            // new-turn rows ride along with the recompute pass
    int load_path = 0;                // 0 auto, 1 staged DMA + scatter, 2 direct load kernel
    int load_wgs = 8;                 // resident workgroups of the direct load kernel
    int stage_begin = 0, stage_end = 0;   // layers this context restores (one pipeline stage)
    int capture_layer = -1;               // next call: copy the rows entering this layer ...
    float* capture_out = nullptr;         // ... to this device array [rows][d]
    int64_t capture_cap_rows = 0;
    std::vector<int32_t> caprows;         // next call: packed rows whose residual stream is sampled ...
    float* caprows_out = nullptr;         // ... at every layer entry, to this device array [L+1][n][d]
    const int32_t* caprows_dev = nullptr; // the row list in the call's device metadata
    int inject_fail_at = 0;           // > 0: that status check of the next call's enqueue part fails
    double throttle_gbs = 0;          // > 0: the copy stream is paced to this many GB/s
    double wall_hz = 1e8;             // rate of the device's constant wall clock
    std::vector<hipEvent_t> ev_layer; // copy stream: loaded KV of layer l is in place
    std::vector<hipEvent_t> ev_wait;  // compute stream: before / after its wait for layer l's loads (2 per layer)
    std::vector<char> waited;         // layers whose wait was recorded in the current call
    std::vector<hipEvent_t> dyn_events;   // run-time scheduler: loads in flight + the compute step
    // run-time scheduler: ratios measured / predicted carried from call to call -- the compute
    // engine's, the channel's beside a recomputing engine, the channel's on its own
    int dyn_scale_c = 1000, dyn_scale_io = 1000, dyn_scale_io_alone = 1000;
    int dma_queues = 2;                   // streams a layer's DMA transfers are spread over (1 or 2)
    int n_last = 0;                   // requests whose final hidden row the last call left in h_last

    // per-kernel-class timing (cf_ctx_profile): event pairs around selected launches
    struct ProfRec { int cls; double work; hipEvent_t e0, e1; };
    uint32_t prof_mask = 0;
    std::vector<ProfRec> prof_recs;
    std::vector<hipEvent_t> prof_pool;
    cf_kernel_stat prof_acc[CF_N_KERNELS] = {};
    bool prof_on(int cls) const { return (prof_mask >> cls) & 1u; }
    hipEvent_t prof_event() {
        hipEvent_t e = nullptr;
        if (!prof_pool.empty()) { e = prof_pool.back(); prof_pool.pop_back(); }
        else if (hipEventCreate(&e) != hipSuccess) e = nullptr;
        return e;
    }
    void prof_begin(int cls, double work, hipStream_t st) {
        if (!prof_on(cls)) return;
        ProfRec r{cls, work, prof_event(), prof_event()};
        if (!r.e0 || !r.e1) return;
        (void)hipEventRecord(r.e0, st);
        prof_recs.push_back(r);
    }
    void prof_end(int cls, hipStream_t st) {
        if (!prof_on(cls) || prof_recs.empty()) return;
        (void)hipEventRecord(prof_recs.back().e1, st);
    }
    void prof_collect() {     // after the streams are idle
        for (ProfRec& r : prof_recs) {
            float ms = 0;
            if (hipEventElapsedTime(&ms, r.e0, r.e1) == hipSuccess) {
                prof_acc[r.cls].launches += 1;
                prof_acc[r.cls].total_ms += ms;
                prof_acc[r.cls].work += r.work;
            }
            prof_pool.push_back(r.e0);
            prof_pool.push_back(r.e1);
        }
        prof_recs.clear();
    }

    float* h() { return (float*)(ws + cv.h); }
    float* dl() { return (float*)(ws + cv.dl); }   // pending residual update of each row
    void* a() { return ws + cv.a; }
    float* qkv() { return (float*)(ws + cv.qkv); }
    void* q() { return ws + cv.q; }
    void* o() { return ws + cv.o; }
    void* act() { return ws + cv.act; }
    void* a_last() { return ws + cv.a_last; }
    float* h_last() { return (float*)(ws + cv.h_last); }   // final hidden row of each request's last new token
    float* attn_part() { return (float*)(ws + cv.attn_part); }
    float2* rope() { return (float2*)(ws + cv.rope); }
    char* staging() { return ws + cv.staging; }
    char* meta_dev() { return ws + cv.meta; }
    void* pace_dev() { return ws + cv.pace; }
};

extern "C" int cf_workspace_bytes(const cf_model_desc* desc, const cf_ctx_opts* opts, size_t* bytes) {
    if (!desc || !opts || !bytes) return fail(CF_ERR_INVALID_ARG, "cf_workspace_bytes: null argument");
    Carve c;
    int rc = carve_workspace(*desc, *opts, &c);
    if (rc) return rc;
    *bytes = c.total;
    return CF_OK;
}

extern "C" int cf_ctx_create(const cf_model_desc* desc, const cf_weights* weights,
                             const cf_ctx_opts* opts, void* workspace, size_t workspace_bytes,
                             void* compute_stream, void* copy_stream, cf_ctx** out) {
    if (!desc || !weights || !opts || !workspace || !out || !weights->layers || !weights->embed ||
        !weights->lm_head || !weights->final_norm)
        return fail(CF_ERR_INVALID_ARG, "cf_ctx_create: null argument");
    Carve cv;
    int rc = carve_workspace(*desc, *opts, &cv);
    if (rc) return rc;
    if (workspace_bytes < cv.total)
        return fail(CF_ERR_WORKSPACE, "cf_ctx_create: workspace %zu < needed %zu", workspace_bytes,
                    cv.total);
    if (((uintptr_t)workspace & 255) != 0)
        return fail(CF_ERR_INVALID_ARG, "cf_ctx_create: workspace must be 256-byte aligned");
    for (int l = 0; l < desc->n_layers; ++l) {
        const cf_layer_weights& lw = weights->layers[l];
        if (!lw.attn_norm || !lw.wqkv || !lw.wo || !lw.mlp_norm || !lw.w_gate || !lw.w_up || !lw.w_down)
            return fail(CF_ERR_INVALID_ARG, "cf_ctx_create: layer %d has a null weight", l);
    }
    cf_ctx* c = new cf_ctx;
    c->m = *desc;
    c->opts = *opts;
    c->w = *weights;
    c->layers.assign(weights->layers, weights->layers + desc->n_layers);
    c->w.layers = c->layers.data();
    c->cs = (hipStream_t)compute_stream;
    c->ps = (hipStream_t)copy_stream;
    c->ws = (char*)workspace;
    c->cv = cv;
    c->stage_begin = 0;
    c->stage_end = desc->n_layers;
    c->simple_only = false;
    auto bail = [&](int code) { cf_ctx_destroy(c); return code; };
#define CF_HIP_CTX(call)                                                                      \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return bail(fail(CF_ERR_HIP, "%s:%d %s -> %s", __FILE__, __LINE__, #call,         \
                             hipGetErrorString(e_)));                                         \
    } while (0)
    {
        // set-up of cf_offload_static on this device: resolve the static scratch array's address
        char* sc = nullptr;
        int rs = static_scratch_of_current_device(&sc);
        if (rs) return bail(rs);
    }
    CF_HIP_CTX(hipStreamCreateWithFlags(&c->ss, hipStreamNonBlocking));
    c->own_ss = true;
    CF_HIP_CTX(hipHostMalloc((void**)&c->meta_host, cv.meta_bytes, hipHostMallocDefault));
    hipEvent_t* evs[] = {&c->ev_start, &c->ev_meta, &c->ev_comp, &c->ev_copy, &c->ev_end,
                         &c->ev_scat, &c->ev_t0, &c->ev_t1, &c->ev_q2};
    for (hipEvent_t* e : evs) CF_HIP_CTX(hipEventCreate(e));
    for (int i = 0; i < N_STAGING_SLOTS; ++i) {
        CF_HIP_CTX(hipEventCreateWithFlags(&c->ev_filled[i], hipEventDisableTiming));
        CF_HIP_CTX(hipEventCreateWithFlags(&c->ev_free[i], hipEventDisableTiming));
    }
    c->ev_layer.assign(desc->n_layers, nullptr);
    for (int l = 0; l < desc->n_layers; ++l)
        CF_HIP_CTX(hipEventCreateWithFlags(&c->ev_layer[l], hipEventDisableTiming));
    c->ev_wait.assign(2 * (size_t)desc->n_layers, nullptr);
    for (hipEvent_t& e : c->ev_wait) CF_HIP_CTX(hipEventCreate(&e));
    c->waited.assign(desc->n_layers, 0);
    // RoPE table: angles formed in double, rounded once to float.
    {
        int half = desc->head_dim / 2;
        std::vector<float2> tab((size_t)opts->max_positions * half);
        std::vector<double> theta(half);
        for (int j = 0; j < half; ++j)
            theta[j] = std::pow((double)desc->rope_base, -2.0 * j / (double)desc->head_dim);
        for (int p = 0; p < opts->max_positions; ++p)
            for (int j = 0; j < half; ++j) {
                double ang = (double)p * theta[j];
                tab[(size_t)p * half + j] = make_float2((float)std::cos(ang), (float)std::sin(ang));
            }
        CF_HIP_CTX(hipMemcpy(c->rope(), tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice));
    }
#undef CF_HIP_CTX
    *out = c;
    return CF_OK;
}

extern "C" void cf_ctx_destroy(cf_ctx* c) {
    if (!c) return;
    hipEvent_t evs[] = {c->ev_start, c->ev_meta, c->ev_comp, c->ev_copy, c->ev_end,
                        c->ev_scat, c->ev_t0, c->ev_t1, c->ev_q2};
    for (hipEvent_t e : evs)
        if (e) (void)hipEventDestroy(e);
    for (int i = 0; i < N_STAGING_SLOTS; ++i) {
        if (c->ev_filled[i]) (void)hipEventDestroy(c->ev_filled[i]);
        if (c->ev_free[i]) (void)hipEventDestroy(c->ev_free[i]);
    }
    for (hipEvent_t e : c->ev_layer)
        if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->ev_wait)
        if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->dyn_events)
        if (e) (void)hipEventDestroy(e);
    for (auto& r : c->prof_recs) { c->prof_pool.push_back(r.e0); c->prof_pool.push_back(r.e1); }
    for (hipEvent_t e : c->prof_pool) (void)hipEventDestroy(e);
    if (c->meta_host) (void)hipHostFree(c->meta_host);
    if (c->own_ss && c->ss) (void)hipStreamDestroy(c->ss);
    delete c;
}

extern "C" int cf_ctx_set_pipelined_join(cf_ctx* ctx, int32_t on) {
    if (!ctx) return fail(CF_ERR_INVALID_ARG, "cf_ctx_set_pipelined_join: null ctx");
    ctx->pipelined = on != 0;
    return CF_OK;
}

extern "C" int cf_ctx_set_load_path(cf_ctx* ctx, int32_t path, int32_t n_workgroups) {
    if (!ctx) return fail(CF_ERR_INVALID_ARG, "cf_ctx_set_load_path: null ctx");
    if (path < 0 || path > 2) return fail(CF_ERR_INVALID_ARG, "cf_ctx_set_load_path: path %d not in 0..2", path);
    if (n_workgroups < 0 || n_workgroups > 1024)
        return fail(CF_ERR_INVALID_ARG, "cf_ctx_set_load_path: n_workgroups %d not in 0..1024", n_workgroups);
    ctx->load_path = path;
    if (n_workgroups > 0) ctx->load_wgs = n_workgroups;
    return CF_OK;
}

extern "C" int cf_ctx_set_stage(cf_ctx* ctx, int32_t layer_begin, int32_t layer_end) {
    if (!ctx) return fail(CF_ERR_INVALID_ARG, "cf_ctx_set_stage: null ctx");
    if (layer_begin < 0 || layer_begin >= layer_end || layer_end > ctx->m.n_layers)
        return fail(CF_ERR_INVALID_ARG, "cf_ctx_set_stage: need 0 <= begin < end <= %d, got [%d, %d)",
                    ctx->m.n_layers, layer_begin, layer_end);
    ctx->stage_begin = layer_begin;
    ctx->stage_end = layer_end;
    return CF_OK;
}

extern "C" int cf_ctx_capture_boundary(cf_ctx* ctx, int32_t layer, float* dev_out, int64_t cap_rows) {
    if (!ctx) return fail(CF_ERR_INVALID_ARG, "cf_ctx_capture_boundary: null ctx");
    if (layer < 0 || layer >= ctx->m.n_layers || !dev_out || cap_rows <= 0)
        return fail(CF_ERR_INVALID_ARG, "cf_ctx_capture_boundary: bad layer or buffer");
    ctx->capture_layer = layer;
    ctx->capture_out = dev_out;
    ctx->capture_cap_rows = cap_rows;
    return CF_OK;
}

extern "C" int cf_ctx_capture_rows(cf_ctx* ctx, const int32_t* packed_rows, int32_t n_rows, float* dev_out) {
    if (!ctx) return fail(CF_ERR_INVALID_ARG, "cf_ctx_capture_rows: null ctx");
    if (n_rows < 0 || n_rows > 4096 || (n_rows > 0 && (!packed_rows || !dev_out)))
        return fail(CF_ERR_INVALID_ARG, "cf_ctx_capture_rows: need 0 <= n_rows <= 4096 and non-null arrays");
    if (ctx->m.d_model % 4 != 0) return fail(CF_ERR_UNSUPPORTED, "cf_ctx_capture_rows: d_model %% 4 != 0");
    ctx->caprows.assign(packed_rows, packed_rows + n_rows);
    ctx->caprows_out = n_rows > 0 ? dev_out : nullptr;
    return CF_OK;
}

extern "C" int cf_ctx_set_link_throttle(cf_ctx* ctx, double gb_per_s) {
    if (!ctx) return fail(CF_ERR_INVALID_ARG, "cf_ctx_set_link_throttle: null ctx");
    if (!(gb_per_s >= 0) || gb_per_s > 1e6)
        return fail(CF_ERR_INVALID_ARG, "cf_ctx_set_link_throttle: rate must be in [0, 1e6] GB/s");
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess && khz > 0)
        ctx->wall_hz = 1e3 * khz;
    else
        (void)hipGetLastError();
    ctx->throttle_gbs = gb_per_s;
    return CF_OK;
}

extern "C" int cf_ctx_set_kernel_set(cf_ctx* ctx, int32_t simple_only) {
    if (!ctx) return fail(CF_ERR_INVALID_ARG, "cf_ctx_set_kernel_set: null ctx");
    ctx->simple_only = simple_only != 0;
    return CF_OK;
}

extern "C" int cf_ctx_inject_failure(cf_ctx* ctx, int32_t nth_check) {
    if (!ctx) return fail(CF_ERR_INVALID_ARG, "cf_ctx_inject_failure: null ctx");
    if (nth_check < 0) return fail(CF_ERR_INVALID_ARG, "cf_ctx_inject_failure: nth_check must be >= 0");
    ctx->inject_fail_at = nth_check;
    return CF_OK;
}

namespace {

// ---------------------------------------------------------------- host metadata
struct Segment {        // rows of one request inside a packed phase
    int req;            // index into the call's request array
    int row0, n_rows;   // packed rows
    int pos0;           // absolute position of the first row
    int layers;         // rows are active in layers [0, layers)
    bool is_new;        // new-turn rows: they read loaded KV and go through every layer fully
};

struct ChunkInfo {
    int r0, r1;         // packed row range
    int work_off, n_work;
    int grp_off, n_grp; // combine groups of the items whose key range was split
    int r_mid;                   // rows [r0, r_mid) are recompute rows, [r_mid, r1) new-turn rows
    int n_work_rec, n_grp_rec;   // leading items / groups that belong to recompute rows
};

struct Phase {
    int T = 0;
    std::vector<Segment> segs;          // packed order; `layers` non-increasing
    std::vector<const float*> seg_boundary;   // per segment: host hidden states of its rows, or null
    std::vector<ChunkInfo> chunks;
    std::vector<AttnWork> work;
    std::vector<AttnCombine> groups;
    // device offsets (bytes into meta)
    size_t off_ids = 0, off_pos = 0, off_slot = 0, off_work = 0, off_grp = 0;
    int rows_active(int layer) const {
        int t = 0;
        for (const Segment& s : segs)
            if (s.layers > layer) t = s.row0 + s.n_rows;
        return t;
    }
    // packed order: recompute rows (layer cut non-increasing), then new-turn rows
    int rec_rows() const {
        int t = 0;
        for (const Segment& s : segs)
            if (!s.is_new) t = s.row0 + s.n_rows;
        return t;
    }
    // recompute rows active in `layer` (a prefix), and those that go on past its K/V write
    // because they have a further layer to feed (a prefix as well)
    int rec_active(int layer, int ahead) const {
        int t = 0;
        for (const Segment& s : segs)
            if (!s.is_new && s.layers > layer + ahead) t = s.row0 + s.n_rows;
        return t;
    }
};

struct MetaWriter {
    char* host;
    size_t cap, off = 0;
    bool overflow = false;
    size_t put(const void* src, size_t bytes) {
        size_t at = off;
        size_t end = (off + bytes + 15) / 16 * 16;
        if (end > cap) { overflow = true; return 0; }
        if (bytes) std::memcpy(host + at, src, bytes);
        off = end;
        return at;
    }
};

// Cut a phase into row chunks and the chunks into attention work items of up to 128 query
// rows.  When a chunk has too few items to fill the GPU (few new tokens over long contexts)
// and `n_q_heads_split` > 0, the key range of an item is split into slices that run as
// separate workgroups and are merged afterwards.
void build_chunks(Phase& ph, int chunk_rows, const std::vector<int>& pt_off, int n_q_heads_split,
                  int heads_per_block) {
    for (int r0 = 0; r0 < ph.T; r0 += chunk_rows) {
        ChunkInfo ci;
        ci.r0 = r0;
        ci.r1 = std::min(ph.T, r0 + chunk_rows);
        ci.work_off = (int)ph.work.size();
        ci.grp_off = (int)ph.groups.size();
        std::vector<AttnWork> items;
        int n_items_rec = 0, n_rec_attending = 0;
        ci.r_mid = std::min(std::max(ph.rec_rows(), ci.r0), ci.r1);
        for (const Segment& s : ph.segs) {
            int a = std::max(s.row0, ci.r0), b = std::min(s.row0 + s.n_rows, ci.r1);
            for (int r = a; r < b; r += ATTN_BLOCK_ROWS) {
                AttnWork w;
                w.row0 = r - ci.r0;                       // relative to the chunk buffer
                w.n_rows = std::min(ATTN_BLOCK_ROWS, b - r);
                w.pos0 = s.pos0 + (r - s.row0);
                w.pt_off = pt_off[s.req];
                w.tile_begin = 0;
                w.tile_end = (w.pos0 + w.n_rows + ATTN_KEY_TILE - 1) / ATTN_KEY_TILE;
                w.part = -1;
                w.pad = 0;
                items.push_back(w);
                if (!s.is_new) {
                    n_items_rec = (int)items.size();      // recompute segments come first
                    if (s.layers >= 2) ++n_rec_attending; // a request cut after layer 1 never attends
                }
            }
        }
        // The recompute items and the new-turn items of a layer are separate launches, so each
        // group gets its own split factor: the one that brings its workgroup count to about 1024.
        // workgroups that fit the chip at once: 2 per CU of 4 wavefronts, or 1 per CU of 8
        const int64_t resident = heads_per_block == 2 ? 256 : 512;
        auto factor_for = [&](int n_items) {
            if (n_q_heads_split <= 0 || n_items <= 0) return 1;
            int64_t blocks = (int64_t)n_items * (n_q_heads_split / heads_per_block);
            return blocks < resident ? (int)((2 * resident + blocks - 1) / blocks) : 1;
        };
        const int factor_rec = factor_for(n_rec_attending);
        const int factor_new = factor_for((int)items.size() - n_items_rec);
        int next_part = 0, item_idx = 0;
        ci.n_work_rec = ci.n_grp_rec = 0;
        for (const AttnWork& w : items) {
            const int factor = item_idx < n_items_rec ? factor_rec : factor_new;
            if (item_idx++ == n_items_rec) {       // everything before this came from recompute rows
                ci.n_work_rec = (int)ph.work.size() - ci.work_off;
                ci.n_grp_rec = (int)ph.groups.size() - ci.grp_off;
                next_part = 0;                     // the partial buffers are free again by then
            }
            int full_tiles = w.pos0 / ATTN_KEY_TILE;          // tiles every row sees completely
            int n_split = std::min(factor, std::max(1, full_tiles / 16));
            if (n_split > 1 && (int64_t)(next_part + n_split) * n_q_heads_split > ATTN_MAX_PART_BLOCKS)
                n_split = 1;
            if (n_split <= 1) {
                ph.work.push_back(w);
                continue;
            }
            AttnCombine gcomb{w.row0, w.n_rows, next_part, n_split};
            int begin = 0;
            for (int j = 0; j < n_split; ++j) {
                AttnWork p = w;
                p.tile_begin = begin;
                p.tile_end = (j + 1 == n_split) ? w.tile_end
                                                : std::min((int)((int64_t)(j + 1) * w.tile_end / n_split), full_tiles);
                p.part = next_part++;
                begin = p.tile_end;
                ph.work.push_back(p);
            }
            ph.groups.push_back(gcomb);
        }
        ci.n_work = (int)ph.work.size() - ci.work_off;
        ci.n_grp = (int)ph.groups.size() - ci.grp_off;
        if (n_items_rec == (int)items.size()) { ci.n_work_rec = ci.n_work; ci.n_grp_rec = ci.n_grp; }
        // The kernel walks a launch's list backwards.  New-turn items (one launch per layer, contexts
        // of very different lengths) are listed lightest first so that the launch starts with its
        // longest items; recompute items stay in row order: a layer launches a prefix of them.
        std::stable_sort(ph.work.begin() + ci.work_off + ci.n_work_rec, ph.work.end(),
                         [](const AttnWork& a, const AttnWork& b) {
                             return a.tile_end - a.tile_begin < b.tile_end - b.tile_begin;
                         });
        ph.chunks.push_back(ci);
    }
}

void gemm(cf_ctx* c, int cls, const void* A, const void* W, const void* W2, float* Cf, void* Dt,
          int M, int N, int K, int epi) {
    c->prof_begin(cls, 2.0 * M * (double)N * K * (epi == EPI_SILU_MUL ? 2 : 1), c->cs);
    if (!c->simple_only && gemm_mfma_supported(c->m.dtype, M, N, K, epi))
        launch_gemm_mfma(c->cs, A, W, W2, Cf, Dt, M, N, K, epi);
    else
        launch_gemm_simple(c->cs, c->m.dtype, A, W, W2, Cf, Dt, M, N, K, epi);
    c->prof_end(cls, c->cs);
}

// Run layers [l_begin, n_layers_max) of one packed phase on the compute stream; the phase's
// rows sit at rows row_base.. of the residual buffers.  l_begin > 0 resumes a phase whose
// earlier layers ran in a previous call with the same row_base (its hidden states are still
// in the workspace), so nothing is embedded.  `between_layers` (may be null) is called before
// every layer is enqueued; a negative result aborts.
//
// The residual stream h stays float.  O-proj and down-proj store their result into the
// float buffer dl (plain stores out of the GEMM), and the next RMSNorm folds it in
// (h += dl) while it reads the row anyway.  Recompute rows in their LAST active layer stop
// after the K/V write: nothing downstream reads their attention or MLP output.  New-turn
// rows (packed after the recompute rows) go through every layer fully.
//
// `layer_ready` (may be null): per layer, the event after which the loaded KV of that layer is
// in place (null entry = nothing is loaded for it); the attention of the new-turn rows of a
// layer waits for it, everything else of the layer does not.  `ev_rec_done` is recorded after
// the last layer in which a recompute row is active.
// Layers are counted from the context's stage: layer l here is layer stage_begin + l of the model.
// A stage above layer 0 has no embedding to start from: its rows start from the boundary
// activations the caller holds for them (copied into h ahead of the first layer).
int run_phase(cf_ctx* c, cf_cache* cache, const Phase& ph, int n_layers_max,
              const hipEvent_t* layer_ready, hipEvent_t ev_rec_done, int l_begin = 0, int row_base = 0,
              const std::function<int()>* between_layers = nullptr) {
    const int layer0 = c->stage_begin;
    const cf_model_desc& m = c->m;
    int last_rec_layer = -1;
    for (const Segment& sg : ph.segs)
        if (!sg.is_new) last_rec_layer = std::max(last_rec_layer, sg.layers - 1);
    if (last_rec_layer < 0 && ev_rec_done) CF_HIP(hipEventRecord(ev_rec_done, c->cs));
    if (ph.T <= 0) return CF_OK;
    size_t es = elem_bytes(m.dtype);
    char* md = c->meta_dev();
    const int32_t* d_ids = (const int32_t*)(md + ph.off_ids);
    const int32_t* d_pos = (const int32_t*)(md + ph.off_pos);
    const int32_t* d_slot = (const int32_t*)(md + ph.off_slot);
    const AttnWork* d_work = (const AttnWork*)(md + ph.off_work);
    const AttnCombine* d_grp = (const AttnCombine*)(md + ph.off_grp);
    const int32_t* d_pt = (const int32_t*)md;      // page tables sit at offset 0
    KvGeom g;
    g.n_kv_heads = m.n_kv_heads;
    g.head_dim = m.head_dim;
    g.page_elems = (int64_t)(cache->page_bytes / es);
    g.layer_stride = g.page_elems * cache->n_pages;
    const int qcols = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
    const int nq = m.n_q_heads * m.head_dim;
    const int d = m.d_model;
    bool mfma_attn = !c->simple_only &&
                     attention_mfma_supported(m.dtype, m.head_dim, m.n_q_heads, m.n_kv_heads);
    const bool any_new = ph.rec_rows() < ph.T;

    float* const h_rows = c->h() + (size_t)row_base * d;
    float* const dl_rows = c->dl() + (size_t)row_base * d;
    if (l_begin > 0) {
        // resumed phase: hidden states are in place
    } else if (layer0 == 0) {
        c->prof_begin(CF_K_EMBED, (double)ph.T * d * (es + 4), c->cs);
        launch_embed(c->cs, m.dtype, c->w.embed, d_ids, h_rows, ph.T, d);
        c->prof_end(CF_K_EMBED, c->cs);
    } else {
        for (size_t si = 0; si < ph.segs.size(); ++si) {
            const Segment& sg = ph.segs[si];
            if (sg.n_rows <= 0) continue;
            // Pinned, device-mapped rows are read over the link by a copy kernel: a DMA copy on
            // this stream can queue behind the load streams' long transfers on a shared engine.
            hipPointerAttribute_t at;
            void* dp = nullptr;
            if (hipPointerGetAttributes(&at, ph.seg_boundary[si]) == hipSuccess && at.type == hipMemoryTypeHost &&
                hipHostGetDevicePointer(&dp, const_cast<float*>(ph.seg_boundary[si]), 0) == hipSuccess && dp) {
                launch_residual_rows(c->cs, h_rows + (size_t)sg.row0 * d, (const float*)dp, nullptr, sg.n_rows, d);
            } else {
                (void)hipGetLastError();
                CF_HIP(hipMemcpyAsync(h_rows + (size_t)sg.row0 * d, ph.seg_boundary[si],
                                      (size_t)sg.n_rows * d * sizeof(float), hipMemcpyHostToDevice, c->cs));
            }
        }
    }
    for (int l = l_begin; l < n_layers_max; ++l) {
        if (between_layers && (*between_layers)() < 0)
            return fail(CF_ERR_HIP, "the copy stream failed while a compute step was being enqueued");
        const int Ta_rec = ph.rec_active(l, 0);    // recompute rows that need K/V in this layer
        const int Tn_rec = ph.rec_active(l, 1);    // ... and go on through the layer
        if (Ta_rec <= 0 && !any_new) break;
        const cf_layer_weights& lw = c->layers[layer0 + l];
        char* pool_layer = (char*)cache->pool + (size_t)(layer0 + l) * g.layer_stride * es;
        if (c->caprows_out && c->caprows_dev && row_base == 0)
            launch_residual_gather(c->cs, c->caprows_out + (size_t)(2 * l) * c->caprows.size() * d, h_rows,
                                   l > 0 ? dl_rows : nullptr, c->caprows_dev, (int)c->caprows.size(), d,
                                   0, Ta_rec, ph.rec_rows(), ph.T);
        if (c->capture_out && c->capture_layer == layer0 + l) {
            // boundary activations: the residual stream of the rows entering this layer
            int rows = any_new ? ph.T : Ta_rec;
            if (rows > c->capture_cap_rows)
                return fail(CF_ERR_WORKSPACE, "cf_restore_batch: boundary capture needs %d rows, buffer holds %lld",
                            rows, (long long)c->capture_cap_rows);
            launch_residual_rows(c->cs, c->capture_out, h_rows, l > 0 ? dl_rows : nullptr, rows, d);
            c->capture_out = nullptr;          // one shot
            c->capture_layer = -1;
        }
        for (const ChunkInfo& ci : ph.chunks) {
            // the chunk's rows: recompute rows [r0, r_mid) then new-turn rows [r_mid, r1)
            int rec_end = std::min(ci.r_mid, Ta_rec), rec_cont = std::min(ci.r_mid, Tn_rec);
            bool has_rec = rec_end > ci.r0, has_new = ci.r1 > ci.r_mid;
            if (!has_rec && !has_new) continue;
            // row ranges of this chunk in this layer: {x, y (rows needing K/V), ycont (rows going on)}
            int ranges[2][3], n_ranges = 0;
            if (has_rec && has_new && rec_cont == ci.r_mid) {
                ranges[n_ranges][0] = ci.r0; ranges[n_ranges][1] = ci.r1; ranges[n_ranges][2] = ci.r1; ++n_ranges;
            } else {
                if (has_rec) { ranges[n_ranges][0] = ci.r0; ranges[n_ranges][1] = rec_end; ranges[n_ranges][2] = std::max(rec_cont, ci.r0); ++n_ranges; }
                if (has_new) { ranges[n_ranges][0] = ci.r_mid; ranges[n_ranges][1] = ci.r1; ranges[n_ranges][2] = ci.r1; ++n_ranges; }
            }
            for (int ri = 0; ri < n_ranges; ++ri) {
                const int x = ranges[ri][0], y = ranges[ri][1], ycont = ranges[ri][2];
                const int Tc = y - x, Tr = ycont - x, xo = x - ci.r0;   // xo: row offset inside the chunk buffers
                float* h = h_rows + (size_t)x * d;
                float* dl = dl_rows + (size_t)x * d;
                char* a_buf = (char*)c->a() + (size_t)xo * d * es;
                float* qkv_buf = c->qkv() + (size_t)xo * qcols;
                char* q_buf = (char*)c->q() + (size_t)xo * nq * es;
                char* o_buf = (char*)c->o() + (size_t)xo * nq * es;
                char* act_buf = (char*)c->act() + (size_t)xo * m.d_ffn * es;
                c->prof_begin(CF_K_RMSNORM, (double)Tc * d * (4 + es), c->cs);
                launch_rmsnorm(c->cs, m.dtype, h, l > 0 ? dl : nullptr, lw.attn_norm, a_buf, Tc, d, m.rms_eps, nullptr);
                c->prof_end(CF_K_RMSNORM, c->cs);
                if (!c->simple_only && gemm_mfma_qkv_rope_supported(m.dtype, Tc, qcols, d, m.head_dim)) {
                    // RoPE and the page write happen on the accumulators of the QKV projection
                    const RopeEpilogue re{d_pos + x, d_slot + x, c->rope(), pool_layer, m.n_q_heads, g};
                    c->prof_begin(CF_K_GEMM_QKV, 2.0 * Tc * (double)qcols * d, c->cs);
                    launch_gemm_mfma_qkv_rope(c->cs, a_buf, lw.wqkv, q_buf, Tc, qcols, d, re);
                    c->prof_end(CF_K_GEMM_QKV, c->cs);
                } else {
                    gemm(c, CF_K_GEMM_QKV, a_buf, lw.wqkv, nullptr, qkv_buf, nullptr, Tc, qcols, d, EPI_STORE_F32);
                    c->prof_begin(CF_K_ROPE_WRITE, (double)Tc * qcols * (4 + es), c->cs);
                    launch_rope_write(c->cs, m.dtype, qkv_buf, d_pos + x, d_slot + x, c->rope(), q_buf, pool_layer,
                                      Tc, m.n_q_heads, g);
                    c->prof_end(CF_K_ROPE_WRITE, c->cs);
                }
                if (Tr <= 0) continue;
                // attention work items (row0 is relative to the chunk): recompute items lead, new-turn
                // items trail.  Recompute rows run first; the new-turn rows also read this layer's
                // loaded KV and therefore wait for the copy stream to have delivered it.
                bool with_rec = x < ci.r_mid, with_new = ycont > ci.r_mid;
                int rec_items = 0, rec_groups = 0;
                if (with_rec) {
                    int lim = std::min(ycont, ci.r_mid);
                    for (int i = 0; i < ci.n_work_rec; ++i)
                        if (ph.work[ci.work_off + i].row0 + ci.r0 < lim) rec_items = i + 1;
                    for (int i = 0; i < ci.n_grp_rec; ++i)
                        if (ph.groups[ci.grp_off + i].row0 + ci.r0 < lim) rec_groups = i + 1;
                }
                for (int part = 0; part < 2; ++part) {
                    int w0, w1, g0, g1;
                    if (part == 0) { if (!with_rec) continue; w0 = 0; w1 = rec_items; g0 = 0; g1 = rec_groups; }
                    else { if (!with_new) continue; w0 = ci.n_work_rec; w1 = ci.n_work; g0 = ci.n_grp_rec; g1 = ci.n_grp; }
                    if (w1 <= w0) continue;
                    if (part == 1 && layer_ready && layer_ready[l]) {
                        // the stall of the compute stream on the copy stream is timed (first wait
                        // of a layer: later chunks of the layer find the event complete)
                        const bool timed = !c->waited[l];
                        if (timed) CF_HIP(hipEventRecord(c->ev_wait[2 * l], c->cs));
                        CF_HIP(hipStreamWaitEvent(c->cs, layer_ready[l], 0));
                        if (timed) {
                            CF_HIP(hipEventRecord(c->ev_wait[2 * l + 1], c->cs));
                            c->waited[l] = 1;
                        }
                    }
                    if (c->prof_on(CF_K_ATTENTION)) {
                        double pairs = 0;
                        for (int i = w0; i < w1; ++i) {
                            const AttnWork& aw = ph.work[ci.work_off + i];
                            if (aw.part >= 0 && aw.tile_begin > 0) continue;   // count a split item once
                            pairs += (double)aw.n_rows * aw.pos0 + (double)aw.n_rows * (aw.n_rows + 1) / 2;
                        }
                        c->prof_begin(CF_K_ATTENTION, pairs * 4.0 * m.n_q_heads * m.head_dim, c->cs);
                    }
                    if (mfma_attn)
                        launch_attention_mfma(c->cs, c->q(), c->o(), c->attn_part(), pool_layer,
                                              d_work + ci.work_off + w0, w1 - w0, d_grp + ci.grp_off + g0,
                                              g1 - g0, d_pt, m.n_q_heads, g);
                    else
                        launch_attention_simple(c->cs, m.dtype, c->q(), c->o(), pool_layer,
                                                d_work + ci.work_off + w0, w1 - w0, d_pt, m.n_q_heads, g);
                    c->prof_end(CF_K_ATTENTION, c->cs);
                }
                gemm(c, CF_K_GEMM_OPROJ, o_buf, lw.wo, nullptr, dl, nullptr, Tr, d, nq, EPI_STORE_F32);
                if (c->caprows_out && c->caprows_dev && row_base == 0)     // the stream entering the MLP half
                    launch_residual_gather(c->cs, c->caprows_out + (size_t)(2 * l + 1) * c->caprows.size() * d,
                                           h_rows, dl_rows, c->caprows_dev, (int)c->caprows.size(), d, x, x + Tr, 0, 0);
                c->prof_begin(CF_K_RMSNORM, (double)Tr * d * (12 + es), c->cs);
                launch_rmsnorm(c->cs, m.dtype, h, dl, lw.mlp_norm, a_buf, Tr, d, m.rms_eps, nullptr);
                c->prof_end(CF_K_RMSNORM, c->cs);
                gemm(c, CF_K_GEMM_GATE_UP, a_buf, lw.w_gate, lw.w_up, nullptr, act_buf, Tr, m.d_ffn, d, EPI_SILU_MUL);
                gemm(c, CF_K_GEMM_DOWN, act_buf, lw.w_down, nullptr, dl, nullptr, Tr, d, m.d_ffn, EPI_STORE_F32);
            }
        }
        if (l == last_rec_layer && ev_rec_done) CF_HIP(hipEventRecord(ev_rec_done, c->cs));
    }
    if (c->caprows_out && c->caprows_dev && row_base == 0 && any_new && l_begin < n_layers_max)
        // what leaves the last layer: only the new-turn rows ran it to the end
        launch_residual_gather(c->cs, c->caprows_out + (size_t)(2 * n_layers_max) * c->caprows.size() * d, h_rows,
                               dl_rows, c->caprows_dev, (int)c->caprows.size(), d, 0, 0, ph.rec_rows(), ph.T);
    c->caprows_dev = nullptr;         // the first phase of a call is the one that is sampled
    return CF_OK;
}

double linear_flops_per_token_layer(const cf_model_desc& m) {
    double qcols = (double)(m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
    return 2.0 * m.d_model * qcols + 2.0 * m.n_q_heads * m.head_dim * (double)m.d_model +
           6.0 * m.d_model * (double)m.d_ffn;
}

// index of the first request whose id already occurred earlier in the batch, or -1
int first_repeated_id(const cf_request* reqs, int B) {
    std::vector<uint64_t> ids(B);
    for (int i = 0; i < B; ++i) ids[i] = reqs[i].req_id;
    std::vector<uint64_t> sorted(ids);
    std::sort(sorted.begin(), sorted.end());
    auto it = std::adjacent_find(sorted.begin(), sorted.end());
    if (it == sorted.end()) return -1;
    int seen = 0;
    for (int i = 0; i < B; ++i)
        if (ids[i] == *it && seen++ == 1) return i;
    return -1;
}

struct CopyOp {
    size_t dst_off;      // into staging
    const char* src;
    size_t bytes;
};

struct LayerLoad {            // direct path: the loads of one layer -- DMA transfers, then one load-kernel launch
    int layer, job_first, n_jobs, n_vblocks;
    size_t bytes;             // all of the layer's loaded bytes (both kinds)
    int dma_first, n_dma;
};
struct DmaOp {                // a run of whole pages that is contiguous in the pool: one transfer, no kernel
    char* dst;
    const char* src;
    size_t bytes;
};
constexpr size_t DMA_MIN_BYTES = (size_t)4 << 20;   // shorter transfers do not reach link speed

// A layer's DMA transfers, alternating between the copy stream and the library's own stream: a
// transfer has a few microseconds of set-up during which the link idles, and two queues let one
// transfer's set-up hide under the other's data.  The second queue may not run ahead into the
// next layer (the layers must complete in order: the new turn's attention waits for them one by
// one), so it first waits for the end of the previous layer's loads on the copy stream
// (`ev_prev`, recorded by end_layer_dma below), and the copy stream waits for the second queue
// before it goes on.  One queue when `two` is false (a paced link: the pacing kernel must see
// every byte in order).
int issue_layer_dma(hipStream_t ps, hipStream_t ss, hipEvent_t ev_prev, hipEvent_t ev_join, bool two,
                    bool& prev_recorded, const DmaOp* ops, int n) {
    two = two && n > 1;
    if (two && prev_recorded && hipStreamWaitEvent(ss, ev_prev, 0) != hipSuccess) return -1;
    for (int k = 0; k < n; ++k)
        if (hipMemcpyAsync(ops[k].dst, ops[k].src, ops[k].bytes, hipMemcpyHostToDevice,
                           (two && (k & 1)) ? ss : ps) != hipSuccess)
            return -1;
    if (two && (hipEventRecord(ev_join, ss) != hipSuccess || hipStreamWaitEvent(ps, ev_join, 0) != hipSuccess))
        return -1;
    return 0;
}
// after everything of the layer is on the copy stream
int end_layer_dma(hipStream_t ps, hipEvent_t ev_prev, bool& prev_recorded) {
    if (hipEventRecord(ev_prev, ps) != hipSuccess) return -1;
    prev_recorded = true;
    return 0;
}

// The load of tokens [lo, hi) of one request in one layer, split by engine.  Whole pages whose
// pool slots are consecutive (the usual case: the allocator hands out the lowest free ids in
// order) go as ONE DMA transfer straight into the pool -- no kernel, no compute unit taken from
// the GEMMs running beside the loads -- when `use_dma` and the transfer is long enough to reach
// link speed.  A first page that is only partly loaded (unaligned split), a last page whose tail
// slots are not part of the range, and short or scattered runs go through the load kernel, which
// writes slot by slot.  host_dev_layer / host_layer: page 0 of this layer in the request's host
// block, as the device and as the host address it; pool_layer: page 0 of the layer in the pool.
void split_load_run(std::vector<PageJob>& jobs, std::vector<DmaOp>& dma, LayerLoad& ll, const int32_t* pt_i,
                    int pt_off_i, const char* host_dev_layer, const char* host_layer, char* pool_layer,
                    size_t pb, int model_layer, int lo, int hi, bool use_dma) {
    const int j = lo / CF_PAGE_TOKENS, j1 = (int)ceil_div(hi, CF_PAGE_TOKENS);
    auto kernel_job = [&](int ja, int jb) {      // pages [ja, jb) through the load kernel
        if (jb <= ja) return;
        PageJob job;
        job.staging_off = (int64_t)(uintptr_t)(host_dev_layer + (size_t)ja * pb);
        job.layer = model_layer;
        job.pt_off = pt_off_i;
        job.page_first = ja;
        job.n_pages = jb - ja;
        job.tok_first = std::max(lo, ja * CF_PAGE_TOKENS);
        job.tok_end = std::min(hi, jb * CF_PAGE_TOKENS);
        job.block_first = ll.n_vblocks;
        job.pad = 0;
        jobs.push_back(job);
        ++ll.n_jobs;
        ll.n_vblocks += (int)ceil_div((int64_t)(jb - ja) * (int64_t)(pb / 16), PAGE_LOAD_UNIT_VECS);
    };
    int ja = j, jb = j1, kfirst = j;              // [kfirst, .) accumulates kernel pages
    if (use_dma) {
        if (lo % CF_PAGE_TOKENS != 0) ++ja;
        if (hi % CF_PAGE_TOKENS != 0) --jb;
        for (int p0 = ja; p0 < jb;) {
            int p1 = p0 + 1;
            while (p1 < jb && pt_i[p1] == pt_i[p1 - 1] + 1) ++p1;
            const size_t seg = (size_t)(p1 - p0) * pb;
            if (seg >= DMA_MIN_BYTES) {
                kernel_job(kfirst, p0);
                kfirst = p1;
                dma.push_back(DmaOp{pool_layer + (size_t)pt_i[p0] * pb, host_layer + (size_t)p0 * pb, seg});
                ++ll.n_dma;
            }
            p0 = p1;
        }
    }
    kernel_job(kfirst, j1);
    ll.bytes += (size_t)(j1 - j) * pb;
}
struct SlotPlan {
    int slot;
    int op_first, n_ops;
    int job_first, n_jobs, n_blocks;
};

}  // namespace

extern "C" int cf_restore_batch(cf_ctx* c, cf_cache* cache, int32_t B, const cf_request* reqs,
                                const cf_split* splits, float* logits_out, cf_timing* timing) {
    if (!c || !cache || B < 0 || (B > 0 && (!reqs || !splits)))
        return fail(CF_ERR_INVALID_ARG, "cf_restore_batch: null argument");
    const cf_model_desc& m = c->m;
    if (cache->n_layers != m.n_layers || cache->n_kv_heads != m.n_kv_heads ||
        cache->head_dim != m.head_dim || cache->dtype != m.dtype || !cache->pool)
        return fail(CF_ERR_INVALID_ARG, "cf_restore_batch: cache geometry does not match the model");
    if (B > c->opts.max_batch)
        return fail(CF_ERR_WORKSPACE, "cf_restore_batch: batch %d > max_batch %d", B, c->opts.max_batch);
    if (timing) std::memset(timing, 0, sizeof(*timing));
    if (B == 0) return CF_OK;
    size_t es = elem_bytes(m.dtype);
    // the context's stage: layers [Lb, Lb + L) of the model; layer indices below are relative to Lb
    const int Lb = c->stage_begin, L = c->stage_end - c->stage_begin;
    if (logits_out && L != m.n_layers)
        return fail(CF_ERR_INVALID_ARG, "cf_restore_batch: logits need the whole model, the context is "
                    "restricted to layers [%d, %d)", c->stage_begin, c->stage_end);

    // ---- validate requests and splits on the host before anything is enqueued
    std::vector<int> pt_off(B), n_pages_req(B);
    std::vector<const int32_t*> pt(B);
    int64_t sum_rec = 0, sum_new = 0;
    int total_pt = 0;
    for (int i = 0; i < B; ++i) {
        const cf_request& r = reqs[i];
        const cf_split& s = splits[i];
        if (r.n_ctx < 0 || r.n_new < 0 || (r.n_new > 0 && !r.new_tokens))
            return fail(CF_ERR_INVALID_ARG, "cf_restore_batch: request %d has bad sizes", i);
        if (s.k_tokens < 0 || s.k_tokens > r.n_ctx || s.layer_cut < 0 || s.layer_cut > L)
            return fail(CF_ERR_INVALID_PLAN, "cf_restore_batch: split %d = (k %d, cut %d) outside [0,%d]x[0,%d]",
                        i, s.k_tokens, s.layer_cut, r.n_ctx, L);
        int np = 0;
        pt[i] = cache->table_of(r.req_id, &np);
        if (!cache->has(r.req_id))
            return fail(CF_ERR_UNKNOWN_REQUEST, "cf_restore_batch: request id %llu has no pages",
                        (unsigned long long)r.req_id);
        if ((int64_t)np * CF_PAGE_TOKENS < (int64_t)r.n_ctx + (logits_out ? r.n_new : 0))
            return fail(CF_ERR_OUT_OF_PAGES, "cf_restore_batch: request %d holds %d pages, needs %d tokens",
                        i, np, r.n_ctx + r.n_new);
        if (r.n_ctx + r.n_new > c->opts.max_positions)
            return fail(CF_ERR_WORKSPACE, "cf_restore_batch: request %d exceeds max_positions", i);
        bool recomputes = s.k_tokens > 0 && s.layer_cut > 0;
        bool loads = (s.k_tokens < r.n_ctx) || (s.layer_cut < L && r.n_ctx > 0);
        if (recomputes && !r.ctx_tokens)
            return fail(CF_ERR_INVALID_ARG, "cf_restore_batch: request %d recomputes but has no tokens", i);
        if (recomputes && Lb > 0 && !r.boundary_h)
            return fail(CF_ERR_INVALID_ARG, "cf_restore_batch: request %d recomputes in a stage that starts at "
                        "layer %d but has no boundary activations", i, Lb);
        if (loads && !r.host_kv)
            return fail(CF_ERR_INVALID_ARG, "cf_restore_batch: request %d loads but has no host KV", i);
        if (recomputes) {
            sum_rec += s.k_tokens;
            for (int t = 0; t < s.k_tokens; ++t)
                if ((uint32_t)r.ctx_tokens[t] >= (uint32_t)m.vocab)
                    return fail(CF_ERR_INVALID_ARG, "cf_restore_batch: request %d token %d out of vocab", i, t);
        }
        if (logits_out) {
            if (r.n_new <= 0)
                return fail(CF_ERR_INVALID_ARG, "cf_restore_batch: request %d needs n_new > 0 for logits", i);
            sum_new += r.n_new;
            for (int t = 0; t < r.n_new; ++t)
                if ((uint32_t)r.new_tokens[t] >= (uint32_t)m.vocab)
                    return fail(CF_ERR_INVALID_ARG, "cf_restore_batch: request %d new token %d out of vocab", i, t);
        }
        pt_off[i] = total_pt;
        n_pages_req[i] = np;
        total_pt += np;
    }
    if (int dup = first_repeated_id(reqs, B); dup >= 0)
        return fail(CF_ERR_INVALID_ARG, "cf_restore_batch: request %d repeats the id %llu of an earlier request "
                    "of the batch (two segments would write the same pages)", dup,
                    (unsigned long long)reqs[dup].req_id);
    if (sum_rec > c->opts.max_tokens || sum_new > c->opts.max_tokens)
        return fail(CF_ERR_WORKSPACE, "cf_restore_batch: %lld recompute / %lld new tokens > max_tokens %d",
                    (long long)sum_rec, (long long)sum_new, c->opts.max_tokens);

    // ---- metadata: page tables first (offset 0), then per-phase arrays, then jobs
    MetaWriter mw{c->meta_host, c->cv.meta_bytes};
    {
        std::vector<int32_t> all_pt(std::max(total_pt, 1));
        for (int i = 0; i < B; ++i)
            if (n_pages_req[i]) std::memcpy(&all_pt[pt_off[i]], pt[i], (size_t)n_pages_req[i] * 4);
        mw.put(all_pt.data(), all_pt.size() * 4);
    }
    auto slot_of = [&](int i, int t) { return pt[i][t / CF_PAGE_TOKENS] * CF_PAGE_TOKENS + t % CF_PAGE_TOKENS; };

    // key ranges are split only for the MFMA attention kernel (the plain one walks them whole)
    int split_heads = (!c->simple_only && attention_mfma_supported(m.dtype, m.head_dim, m.n_q_heads, m.n_kv_heads))
                          ? m.n_q_heads : 0;
    // recompute phase: requests in order of descending layer cut so that the rows
    // active in layer l are a prefix of the packed array
    // Packed rows.  Pipelined join (default): ONE phase holds the recompute rows followed by the
    // new-turn rows, so the new-turn prefill of layer l runs right behind the recompute of layer
    // l (same GEMM launches when the rows are adjacent) and only its attention waits for the
    // loaded KV of that layer.  Sequential join: a recompute phase, then a new-token phase.
    Phase rec, suf;
    std::vector<int32_t> last_rows;
    const bool merged = c->pipelined && logits_out != nullptr;
    auto add_segment = [&](Phase& ph, std::vector<int32_t>& ids, std::vector<int32_t>& pos,
                           std::vector<int32_t>& slot, int i, const int32_t* toks, int n_rows, int pos0,
                           int layers, bool is_new) {
        Segment sg{i, ph.T, n_rows, pos0, layers, is_new};
        ph.seg_boundary.push_back(is_new ? nullptr : reqs[i].boundary_h);
        for (int t = 0; t < n_rows; ++t) {
            ids.push_back(toks[t]);
            pos.push_back(pos0 + t);
            slot.push_back(slot_of(i, pos0 + t));
        }
        ph.T += n_rows;
        ph.segs.push_back(sg);
    };
    auto finish_phase = [&](Phase& ph, std::vector<int32_t>& ids, std::vector<int32_t>& pos,
                            std::vector<int32_t>& slot) {
        build_chunks(ph, c->cv.chunk_rows, pt_off, split_heads,
                     split_heads ? attention_mfma_heads_per_block(m.n_q_heads, m.n_kv_heads) : 1);
        ph.off_ids = mw.put(ids.data(), ids.size() * 4);
        ph.off_pos = mw.put(pos.data(), pos.size() * 4);
        ph.off_slot = mw.put(slot.data(), slot.size() * 4);
        ph.off_work = mw.put(ph.work.data(), ph.work.size() * sizeof(AttnWork));
        ph.off_grp = mw.put(ph.groups.data(), ph.groups.size() * sizeof(AttnCombine));
    };
    {
        std::vector<int> order;
        for (int i = 0; i < B; ++i)
            if (splits[i].k_tokens > 0 && splits[i].layer_cut > 0) order.push_back(i);
        std::stable_sort(order.begin(), order.end(),
                         [&](int a, int b) { return splits[a].layer_cut > splits[b].layer_cut; });
        std::vector<int32_t> ids, pos, slot;
        if (merged && sum_rec + sum_new > c->opts.max_tokens)
            return fail(CF_ERR_WORKSPACE, "cf_restore_batch: %lld recompute + %lld new rows > max_tokens %d",
                        (long long)sum_rec, (long long)sum_new, c->opts.max_tokens);
        for (int i : order)
            add_segment(rec, ids, pos, slot, i, reqs[i].ctx_tokens, splits[i].k_tokens, 0,
                        splits[i].layer_cut, false);
        if (merged)
            for (int i = 0; i < B; ++i) {
                add_segment(rec, ids, pos, slot, i, reqs[i].new_tokens, reqs[i].n_new, reqs[i].n_ctx, L, true);
                last_rows.push_back(rec.T - 1);
            }
        finish_phase(rec, ids, pos, slot);
    }
    if (logits_out && !merged) {
        std::vector<int32_t> ids, pos, slot;
        for (int i = 0; i < B; ++i) {
            add_segment(suf, ids, pos, slot, i, reqs[i].new_tokens, reqs[i].n_new, reqs[i].n_ctx, L, true);
            last_rows.push_back(suf.T - 1);
        }
        finish_phase(suf, ids, pos, slot);
    }
    if (c->capture_out && std::max(rec.T, suf.T) > c->capture_cap_rows)
        return fail(CF_ERR_WORKSPACE, "cf_restore_batch: boundary capture buffer holds %lld rows, the call packs %d",
                    (long long)c->capture_cap_rows, std::max(rec.T, suf.T));
    size_t off_last = mw.put(last_rows.data(), last_rows.size() * 4);
    c->n_last = 0;
    const size_t off_caprows = c->caprows_out ? mw.put(c->caprows.data(), c->caprows.size() * 4) : 0;

    // Load path.  Direct: a load kernel reads the pinned host block over the link and writes the
    // pages itself (needs device-mapped host memory).  Staged: DMA into staging slots, then a
    // scatter kernel.  Auto takes the direct path when every host block is device-mapped.
    std::vector<const char*> host_dev(B, nullptr);
    bool direct = c->load_path != 1;
    for (int i = 0; i < B && direct; ++i) {
        if (!reqs[i].host_kv) continue;
        hipPointerAttribute_t at;
        hipError_t e = hipPointerGetAttributes(&at, reqs[i].host_kv);
        if (e != hipSuccess) { (void)hipGetLastError(); direct = false; break; }
        void* dp = nullptr;
        if (at.type != hipMemoryTypeHost ||
            hipHostGetDevicePointer(&dp, const_cast<void*>(reqs[i].host_kv), 0) != hipSuccess || !dp) {
            (void)hipGetLastError();
            direct = false;
            break;
        }
        host_dev[i] = (const char*)dp;
    }
    if (!direct && c->load_path == 2)
        return fail(CF_ERR_INVALID_ARG, "cf_restore_batch: the direct load path needs pinned, device-mapped host KV");
    // copy plan: runs of pages per (request, layer); staged path: packed into staging slots;
    // direct path: one launch per layer
    std::vector<CopyOp> ops;
    std::vector<PageJob> jobs;
    std::vector<SlotPlan> slots;
    std::vector<LayerLoad> layer_loads;
    std::vector<DmaOp> dma_ops;
    int64_t loaded_bytes = 0, loaded_cells = 0, rec_cells = 0;
    std::vector<int> layer_last_slot(L, -1);   // slot (in issue order) holding a layer's last job
    {
        size_t pb = cache->page_bytes;
        size_t slot_cap = c->cv.staging_bytes / N_STAGING_SLOTS;
        SlotPlan cur{0, 0, 0, 0, 0, 0};
        size_t fill = 0;
        auto flush = [&]() {
            if (cur.n_jobs == 0) return;
            slots.push_back(cur);
            int next = (cur.slot + 1) % N_STAGING_SLOTS;
            cur = SlotPlan{next, (int)ops.size(), 0, (int)jobs.size(), 0, 0};
            fill = 0;
        };
        std::vector<int> by_len(B);
        for (int i = 0; i < B; ++i) by_len[i] = i;
        std::stable_sort(by_len.begin(), by_len.end(),
                         [&](int a, int b) { return reqs[a].n_ctx > reqs[b].n_ctx; });
        // order of (request, layer) runs.  Pipelined join: layer by layer from the bottom, so
        // layer l's loads land while the forward pass is still below l.  Sequential join: from
        // the far end (Sec. 3.1, the I/O pointer walks down from the top layer) -- layer-major
        // for the direct path, per request (longest first) for the staged one.
        std::vector<std::pair<int, int>> runs;
        if (merged) {
            for (int l = 0; l < L; ++l)
                for (int i : by_len) runs.emplace_back(i, l);
        } else if (direct) {
            for (int l = L - 1; l >= 0; --l)
                for (int i : by_len) runs.emplace_back(i, l);
        } else {
            for (int i : by_len)
                for (int l = L - 1; l >= 0; --l) runs.emplace_back(i, l);
        }
        for (const auto& run : runs) {
            const int i = run.first, l = run.second;
            const cf_request& r = reqs[i];
            const cf_split& s = splits[i];
            int np_ctx = (int)ceil_div(r.n_ctx, CF_PAGE_TOKENS);
            int lo = (l < s.layer_cut) ? s.k_tokens : 0, hi = r.n_ctx;
            if (l < s.layer_cut) rec_cells += s.k_tokens;
            if (lo >= hi) continue;
            loaded_cells += hi - lo;
            int j = lo / CF_PAGE_TOKENS, j1 = np_ctx;
            if (direct) {
                // the load kernel indexes a run's 16-byte vectors in 32 bits
                if ((int64_t)(j1 - j) * (int64_t)(pb / 16) >= ((int64_t)1 << 31))
                    return fail(CF_ERR_WORKSPACE, "cf_restore_batch: request %d loads more than 32 GiB per layer", i);
                if (layer_loads.empty() || layer_loads.back().layer != l)
                    layer_loads.push_back(LayerLoad{l, (int)jobs.size(), 0, 0, 0, (int)dma_ops.size(), 0});
                LayerLoad& ll = layer_loads.back();
                split_load_run(jobs, dma_ops, ll, pt[i], pt_off[i], host_dev[i] + (size_t)(Lb + l) * np_ctx * pb,
                               (const char*)reqs[i].host_kv + (size_t)(Lb + l) * np_ctx * pb,
                               (char*)cache->pool + (size_t)(Lb + l) * cache->n_pages * pb, pb, Lb + l, lo, hi,
                               c->load_path == 0);
                loaded_bytes += (int64_t)(j1 - j) * pb;
                continue;
            }
            while (j < j1) {
                size_t room = (slot_cap - fill) / pb;
                if (room == 0) { flush(); continue; }
                int take = (int)std::min<size_t>(room, (size_t)(j1 - j));
                size_t dst = (size_t)cur.slot * slot_cap + fill;
                const char* src = (const char*)r.host_kv + ((size_t)(Lb + l) * np_ctx + j) * pb;
                size_t bytes = (size_t)take * pb;
                if (cur.n_ops > 0 && ops.back().src + ops.back().bytes == src &&
                    ops.back().dst_off + ops.back().bytes == dst)
                    ops.back().bytes += bytes;
                else { ops.push_back(CopyOp{dst, src, bytes}); ++cur.n_ops; }
                PageJob jb;
                jb.staging_off = (int64_t)dst;
                jb.layer = Lb + l;
                jb.pt_off = pt_off[i];
                jb.page_first = j;
                jb.n_pages = take;
                jb.tok_first = lo;
                jb.tok_end = hi;
                jb.block_first = cur.n_blocks;
                jb.pad = 0;
                jobs.push_back(jb);
                ++cur.n_jobs;
                cur.n_blocks += take * PAGE_MOVE_SPLIT;
                fill += bytes;
                loaded_bytes += bytes;
                j += take;
                layer_last_slot[l] = (int)slots.size();     // index the current slot will get
            }
        }
        flush();
    }
    // Direct path with DMA: what is left to the load kernel are the ragged ends of the runs (and
    // runs too short for a transfer).  A launch per layer would have each of them queue for
    // compute units behind the GEMM that happens to run (measured: 0.2 ms per layer for a few
    // hundred KB, 7 ms of a 175 ms copy stream), so when they are a small part of the bytes (1/64:
    // what goes first delays the first layer's loads) ONE launch moves them all before the first
    // transfer, while the GPU is still idle; the units of its jobs are then numbered through all
    // layers.  With more of the volume on the kernel (a fragmented pool, a short request whose
    // runs stay under the transfer size) the launches stay per layer: a layer's event must not
    // wait for all loads.  A paced link charges the bytes to their layers either way.
    int64_t kernel_bytes = 0;
    int upfront_units = 0;
    if (direct)
        for (const PageJob& jb : jobs) kernel_bytes += (int64_t)jb.n_pages * (int64_t)cache->page_bytes;
    const bool upfront = direct && !dma_ops.empty() && kernel_bytes > 0 && kernel_bytes * 64 <= loaded_bytes;
    if (upfront)
        for (LayerLoad& ll : layer_loads) {
            for (int k = 0; k < ll.n_jobs; ++k) jobs[ll.job_first + k].block_first += upfront_units;
            upfront_units += ll.n_vblocks;
        }
    size_t off_jobs = mw.put(jobs.data(), jobs.size() * sizeof(PageJob));
    if (mw.overflow)
        return fail(CF_ERR_WORKSPACE, "cf_restore_batch: batch metadata exceeds the context's limits");

    // From here on work is in flight on three streams that reads caller memory (token ids went
    // into the pinned metadata, but host KV blocks and boundary rows are read in place): every
    // failure first waits for the streams, so that the caller may free its buffers on return.
    int checks_done = 0;
    std::fill(c->waited.begin(), c->waited.end(), 0);
    auto bail = [&](int code) {
        (void)hipStreamSynchronize(c->cs);
        (void)hipStreamSynchronize(c->ps);
        (void)hipStreamSynchronize(c->ss);
        (void)hipGetLastError();
        c->prof_collect();
        c->capture_out = nullptr;
        c->capture_layer = -1;
        c->caprows_out = nullptr;
        c->caprows_dev = nullptr;
        c->inject_fail_at = 0;
        return code;
    };
#define CF_HIP_Q(call)                                                                        \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (c->inject_fail_at > 0 && ++checks_done == c->inject_fail_at) e_ = hipErrorUnknown; \
        if (e_ != hipSuccess)                                                                 \
            return bail(cf::fail(CF_ERR_HIP, "%s:%d %s -> %s", __FILE__, __LINE__, #call,     \
                                 hipGetErrorString(e_)));                                     \
    } while (0)
    // ---- enqueue
    char* md = c->meta_dev();
    CF_HIP_Q(hipEventRecord(c->ev_start, c->cs));
    CF_HIP_Q(hipMemcpyAsync(md, c->meta_host, mw.off, hipMemcpyHostToDevice, c->cs));
    CF_HIP_Q(hipEventRecord(c->ev_meta, c->cs));
    CF_HIP_Q(hipStreamWaitEvent(c->ps, c->ev_meta, 0));
    CF_HIP_Q(hipStreamWaitEvent(c->ss, c->ev_meta, 0));

    KvGeom g;
    g.n_kv_heads = m.n_kv_heads;
    g.head_dim = m.head_dim;
    g.page_elems = (int64_t)(cache->page_bytes / es);
    g.layer_stride = g.page_elems * cache->n_pages;

    // copy stream, direct path: one load-kernel launch per layer, host memory -> pages.
    // With a link throttle set, a wait kernel holds the stream after every unit until the bytes
    // moved so far would have crossed a link of that rate.
    double paced_bytes = 0;
    auto pace = [&](double bytes) {
        if (c->throttle_gbs <= 0) return;
        paced_bytes += bytes;
        launch_pace_wait(c->ps, c->pace_dev(),
                         (unsigned long long)(paced_bytes / (c->throttle_gbs * 1e9) * c->wall_hz));
    };
    if (c->throttle_gbs > 0) launch_pace_mark(c->ps, c->pace_dev());
    std::vector<char> layer_loaded(L, 0);
    std::vector<int> load_of_layer(L, -1);
    for (size_t k = 0; k < layer_loads.size(); ++k) {
        load_of_layer[layer_loads[k].layer] = (int)k;
        layer_loaded[layer_loads[k].layer] = 1;
    }
    size_t loads_enqueued = 0;
    bool q2_recorded = false;
    if (upfront)
        launch_page_load(c->ps, m.dtype, cache->pool, (const PageJob*)(md + off_jobs), (int)jobs.size(),
                         upfront_units, c->load_wgs, (const int32_t*)md, g);
    auto enqueue_load = [&](const LayerLoad& ll) -> int {
        c->prof_begin(CF_K_H2D_COPY, (double)ll.bytes, c->ps);
        if (issue_layer_dma(c->ps, c->ss, c->ev_q2, c->ev_scat, c->dma_queues > 1 && c->throttle_gbs <= 0,
                            q2_recorded, dma_ops.data() + ll.dma_first, ll.n_dma) < 0)
            return -1;
        if (!upfront)
            launch_page_load(c->ps, m.dtype, cache->pool, (const PageJob*)(md + off_jobs) + ll.job_first,
                             ll.n_jobs, ll.n_vblocks, c->load_wgs, (const int32_t*)md, g);
        pace((double)ll.bytes);
        c->prof_end(CF_K_H2D_COPY, c->ps);
        if (merged && hipEventRecord(c->ev_layer[ll.layer], c->ps) != hipSuccess) return -1;
        return end_layer_dma(c->ps, c->ev_q2, q2_recorded);
    };
    // Sequential join: everything is enqueued here, from the top layer down.  Pipelined join: the
    // loads of layer l are enqueued just before the compute stream's layer l (see below), so that
    // the host, which issues a transfer per (request, layer), never holds the compute stream back;
    // the copy stream still runs far ahead of it (enqueuing a layer takes microseconds, executing
    // it milliseconds).
    if (!merged)
        for (; loads_enqueued < layer_loads.size(); ++loads_enqueued)
            if (enqueue_load(layer_loads[loads_enqueued]) < 0)
                return bail(fail(CF_ERR_HIP, "cf_restore_batch: enqueuing a load failed"));
    // copy stream, staged path: fill a staging slot by DMA, then the scatter stream places its pages
    bool slot_used[N_STAGING_SLOTS] = {};
    int slot_idx = 0;
    for (const SlotPlan& sp : slots) {
        if (slot_used[sp.slot]) CF_HIP_Q(hipStreamWaitEvent(c->ps, c->ev_free[sp.slot], 0));
        double slot_bytes = 0;
        for (int k = 0; k < sp.n_ops; ++k) slot_bytes += (double)ops[sp.op_first + k].bytes;
        c->prof_begin(CF_K_H2D_COPY, slot_bytes, c->ps);
        for (int k = 0; k < sp.n_ops; ++k) {
            const CopyOp& op = ops[sp.op_first + k];
            CF_HIP_Q(hipMemcpyAsync(c->staging() + op.dst_off, op.src, op.bytes, hipMemcpyHostToDevice, c->ps));
        }
        pace(slot_bytes);
        c->prof_end(CF_K_H2D_COPY, c->ps);
        CF_HIP_Q(hipEventRecord(c->ev_filled[sp.slot], c->ps));
        CF_HIP_Q(hipStreamWaitEvent(c->ss, c->ev_filled[sp.slot], 0));
        c->prof_begin(CF_K_PAGE_SCATTER, 2.0 * slot_bytes, c->ss);
        launch_page_move(c->ss, m.dtype, c->staging(), cache->pool,
                         (const PageJob*)(md + off_jobs) + sp.job_first, sp.n_jobs, sp.n_blocks,
                         (const int32_t*)md, g, true);
        c->prof_end(CF_K_PAGE_SCATTER, c->ss);
        CF_HIP_Q(hipEventRecord(c->ev_free[sp.slot], c->ss));
        slot_used[sp.slot] = true;
        if (merged)
            for (int l = 0; l < L; ++l)
                if (layer_last_slot[l] == slot_idx) {
                    CF_HIP_Q(hipEventRecord(c->ev_layer[l], c->ss));
                    layer_loaded[l] = 1;
                }
        ++slot_idx;
    }
    // the end of the copy stream's work: after the scatter stream's last placement
    auto close_copy_stream = [&]() -> int {
        if (hipEventRecord(c->ev_scat, c->ss) != hipSuccess || hipStreamWaitEvent(c->ps, c->ev_scat, 0) != hipSuccess ||
            hipEventRecord(c->ev_copy, c->ps) != hipSuccess)
            return -1;
        return 0;
    };
    if (!merged && close_copy_stream() < 0)
        return bail(fail(CF_ERR_HIP, "cf_restore_batch: recording the end of the copy stream failed"));

    c->caprows_dev = c->caprows_out ? (const int32_t*)(md + off_caprows) : nullptr;
    // compute stream: layer-major over the batch
    int max_cut = 0;
    for (const Segment& sg : rec.segs) max_cut = std::max(max_cut, sg.layers);
    if (merged) {
        std::vector<hipEvent_t> ready(L, nullptr);
        for (int l = 0; l < L; ++l)
            if (layer_loaded[l]) ready[l] = c->ev_layer[l];
        // direct path: layer l's loads go onto the copy stream right before layer l's kernels go
        // onto the compute stream (the event of a layer is recorded before anything waits for it)
        int next_layer = 0;
        const std::function<int()> feed_copy_stream = [&]() -> int {
            const int l = next_layer++;
            if (l < L && load_of_layer[l] >= 0) {
                if (enqueue_load(layer_loads[load_of_layer[l]]) < 0) return -1;
                ++loads_enqueued;
            }
            return 0;
        };
        int rc2 = run_phase(c, cache, rec, L, ready.data(), c->ev_comp, 0, 0, &feed_copy_stream);
        if (rc2) return bail(rc2);
        while (next_layer < L)
            if (feed_copy_stream() < 0) return bail(fail(CF_ERR_HIP, "cf_restore_batch: enqueuing a load failed"));
        if (close_copy_stream() < 0)
            return bail(fail(CF_ERR_HIP, "cf_restore_batch: recording the end of the copy stream failed"));
        CF_HIP_Q(hipEventRecord(c->ev_t0, c->cs));
    } else {
        int rc2 = run_phase(c, cache, rec, max_cut, nullptr, c->ev_comp);
        if (rc2) return bail(rc2);
        // join, then the new-turn prefill
        CF_HIP_Q(hipStreamWaitEvent(c->cs, c->ev_copy, 0));
        CF_HIP_Q(hipEventRecord(c->ev_t0, c->cs));
        if (logits_out) {
            rc2 = run_phase(c, cache, suf, L, nullptr, nullptr);
            if (rc2) return bail(rc2);
        }
    }
    if (logits_out) {
        // first-token logits; the last layer's down-proj result is still pending in dl
        launch_rmsnorm(c->cs, m.dtype, c->h(), c->dl(), c->w.final_norm, c->a_last(), B, m.d_model,
                       m.rms_eps, (const int32_t*)(md + off_last));
        gemm(c, CF_K_GEMM_LM_HEAD, c->a_last(), c->w.lm_head, nullptr, logits_out, nullptr, B, m.vocab, m.d_model, EPI_STORE_F32);
        // the rows the head saw, kept for cf_read_final_hidden
        launch_residual_gather(c->cs, c->h_last(), c->h(), c->dl(), (const int32_t*)(md + off_last), B, m.d_model,
                               0, INT32_MAX, 0, 0);
        c->n_last = B;
    }
    CF_HIP_Q(hipStreamWaitEvent(c->cs, c->ev_copy, 0));
    CF_HIP_Q(hipEventRecord(c->ev_end, c->cs));
    CF_HIP_Q(hipGetLastError());
    CF_HIP_Q(hipStreamSynchronize(c->cs));
    CF_HIP_Q(hipStreamSynchronize(c->ps));
    CF_HIP_Q(hipStreamSynchronize(c->ss));
    c->prof_collect();

#undef CF_HIP_Q
    c->inject_fail_at = 0;
    c->caprows_out = nullptr;         // one shot
    c->caprows_dev = nullptr;
    float wait_ms = 0;
    int rec_layers = 0;               // layers in which context rows were still recomputed
    for (const Segment& sg : rec.segs)
        if (!sg.is_new) rec_layers = std::max(rec_layers, sg.layers);
    for (int l = 0; l < (int)c->waited.size(); ++l) {
        if (!c->waited[l]) continue;
        c->waited[l] = 0;
        // only the waits inside compute_ms count: those of the layers that still recomputed
        // (a layer-wise cut ends the recompute early; the new-turn rows of the layers above it
        // wait for their loads after the compute measurement has ended)
        if (l >= rec_layers) continue;
        float w = 0;
        if (hipEventElapsedTime(&w, c->ev_wait[2 * l], c->ev_wait[2 * l + 1]) == hipSuccess) wait_ms += w;
        else (void)hipGetLastError();
    }
    if (timing) {
        float t_comp = 0, t_copy = 0, t_join = 0, t_end = 0;
        CF_HIP(hipEventElapsedTime(&t_comp, c->ev_start, c->ev_comp));
        CF_HIP(hipEventElapsedTime(&t_copy, c->ev_start, c->ev_copy));
        CF_HIP(hipEventElapsedTime(&t_join, c->ev_start, c->ev_t0));
        CF_HIP(hipEventElapsedTime(&t_end, c->ev_start, c->ev_end));
        timing->compute_ms = t_comp;
        timing->copy_ms = t_copy;
        // restoration is complete when the last recomputed cell and the last loaded cell are in
        // place; with the pipelined join most of the new-turn prefill has already run by then
        timing->restore_ms = merged ? std::max(t_comp, t_copy) : std::max(t_join, std::max(t_comp, t_copy));
        timing->suffix_ms = t_end - timing->restore_ms;
        timing->total_ms = t_end;
        timing->compute_wait_ms = wait_ms;
        double lin = linear_flops_per_token_layer(m);
        double pair = 4.0 * m.n_q_heads * m.head_dim;
        double fr = 0, fs = 0;
        // the last recomputed layer of a request needs only its K/V projection
        double qkv_fl = 2.0 * m.d_model * (double)(m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
        for (const Segment& s : rec.segs) {
            if (s.is_new) continue;
            fr += (double)(s.layers - 1) * (s.n_rows * lin + pair * ((double)s.n_rows * (s.n_rows + 1) / 2)) +
                  s.n_rows * qkv_fl;
        }
        for (const Phase* ph : {&rec, &suf})
            for (const Segment& s : ph->segs) {
                if (!s.is_new) continue;
                fs += (double)L * (s.n_rows * lin + pair * ((double)s.n_rows * s.pos0 +
                                                            (double)s.n_rows * (s.n_rows + 1) / 2));
            }
        if (logits_out) fs += 2.0 * m.d_model * (double)m.vocab * B;
        timing->recompute_flops = fr;
        timing->suffix_flops = fs;
        timing->loaded_bytes = loaded_bytes;
        timing->recomputed_cells = rec_cells;
        timing->loaded_cells = loaded_cells;
    }
    return CF_OK;
}

// ------------------------------------------------------------------ run-time scheduling
// cf_restore_dynamic: the two engines claim units while the call runs (Sec. 3.3).  The calling
// thread is the scheduler: it polls completion events, keeps the copy stream a few units deep
// and gives the compute stream one step at a time.
namespace {

struct DynUnitLoad {          // one I/O unit: the jobs of its load-kernel launch, and whether DMA can move it
    int job_first, n_jobs, n_vblocks;
    size_t bytes;
    // token-wise units: pages [page_first, page_first + n_pages) of the request per layer;
    // dma_ok: whole pages with consecutive pool ids (one transfer per layer can carry them);
    // joins_prev: the pool id of its first page follows the last page of the unit before it
    int page_first = 0, n_pages = 0;
    bool dma_ok = false, joins_prev = false;
};

double now_ms() {
    using clk = std::chrono::steady_clock;
    return std::chrono::duration<double, std::milli>(clk::now().time_since_epoch()).count();
}

}  // namespace

extern "C" int cf_restore_dynamic(cf_ctx* c, cf_cache* cache, int32_t B, const cf_request* reqs,
                                  const cf_cost_model* cost, const cf_plan_opts* opts,
                                  const cf_dynamic_opts* dyn, float* logits_out, cf_split* splits_out,
                                  cf_timing* timing, cf_dynamic_stats* stats) {
    if (!c || !cache || !cost || !opts || B < 0 || (B > 0 && (!reqs || !splits_out)))
        return fail(CF_ERR_INVALID_ARG, "cf_restore_dynamic: null argument");
    const cf_model_desc& m = c->m;
    if (cache->n_layers != m.n_layers || cache->n_kv_heads != m.n_kv_heads ||
        cache->head_dim != m.head_dim || cache->dtype != m.dtype || !cache->pool)
        return fail(CF_ERR_INVALID_ARG, "cf_restore_dynamic: cache geometry does not match the model");
    if (c->stage_begin != 0 || c->stage_end != m.n_layers)
        return fail(CF_ERR_INVALID_ARG, "cf_restore_dynamic: the context must cover the whole model");
    if (B > c->opts.max_batch)
        return fail(CF_ERR_WORKSPACE, "cf_restore_dynamic: batch %d > max_batch %d", B, c->opts.max_batch);
    const int L = m.n_layers, C = opts->chunk_tokens;
    const size_t es = elem_bytes(m.dtype), pb = cache->page_bytes;
    const int64_t step_cap = dyn ? dyn->step_cap_ps : 0;
    const int32_t order = dyn ? dyn->order : CF_ORDER_CHEAPEST;
    const int32_t units_cap = dyn ? dyn->units_per_request : 0;
    if (dyn && (dyn->step_cap_ps < 0 || (order != CF_ORDER_CHEAPEST && order != CF_ORDER_SHORTEST) ||
                dyn->units_per_request < 0 || dyn->overlap_comp_permille < 0 || dyn->overlap_io_permille < 0))
        return fail(CF_ERR_INVALID_ARG, "cf_restore_dynamic: bad step cap, claim order, unit limit or overlap factor");
    if (dyn && (dyn->overlap_comp_permille > 0 || dyn->overlap_io_permille > 0)) {
        // the overlap model says how much slower each engine runs beside the other: the ratios
        // measured / predicted of the side-by-side case restart from there, the channel's own at 1
        c->dyn_scale_c = dyn->overlap_comp_permille > 0 ? dyn->overlap_comp_permille : 1000;
        c->dyn_scale_io = dyn->overlap_io_permille > 0 ? dyn->overlap_io_permille : 1000;
        c->dyn_scale_io_alone = 1000;
    }
    if (C <= 0 || C % CF_PAGE_TOKENS != 0)
        return fail(CF_ERR_INVALID_ARG, "cf_restore_dynamic: chunk_tokens must be a positive multiple of %d",
                    CF_PAGE_TOKENS);
    if (opts->n_layers != L || opts->kv_bytes_per_token_layer != (int32_t)(pb / CF_PAGE_TOKENS))
        return fail(CF_ERR_INVALID_ARG, "cf_restore_dynamic: plan options do not describe this model "
                    "(n_layers %d, KV bytes per token and layer %d)", opts->n_layers, opts->kv_bytes_per_token_layer);
    if (timing) std::memset(timing, 0, sizeof(*timing));
    if (stats) std::memset(stats, 0, sizeof(*stats));
    if (B == 0) return CF_OK;

    // ---- validate, page tables, modes and unit counts
    std::vector<int32_t> n_ctx(B), mode(B), n_units(B), p_comp(B, 0), p_io(B);
    std::vector<int> pt_off(B), n_pages_req(B);
    std::vector<const int32_t*> pt(B);
    std::vector<const char*> host_dev(B, nullptr);
    int total_pt = 0;
    int64_t sum_new = 0, rows_lw = 0, n_tw = 0;
    for (int i = 0; i < B; ++i) {
        const cf_request& r = reqs[i];
        if (r.n_ctx < 0 || r.n_new < 0 || (r.n_new > 0 && !r.new_tokens))
            return fail(CF_ERR_INVALID_ARG, "cf_restore_dynamic: request %d has bad sizes", i);
        int np = 0;
        pt[i] = cache->table_of(r.req_id, &np);
        if (!cache->has(r.req_id))
            return fail(CF_ERR_UNKNOWN_REQUEST, "cf_restore_dynamic: request id %llu has no pages",
                        (unsigned long long)r.req_id);
        if ((int64_t)np * CF_PAGE_TOKENS < (int64_t)r.n_ctx + (logits_out ? r.n_new : 0))
            return fail(CF_ERR_OUT_OF_PAGES, "cf_restore_dynamic: request %d holds %d pages, needs %d tokens",
                        i, np, r.n_ctx + r.n_new);
        if (r.n_ctx + r.n_new > c->opts.max_positions)
            return fail(CF_ERR_WORKSPACE, "cf_restore_dynamic: request %d exceeds max_positions", i);
        if (r.n_ctx > 0) {
            if (!r.ctx_tokens || !r.host_kv)
                return fail(CF_ERR_INVALID_ARG, "cf_restore_dynamic: request %d needs ctx_tokens and host_kv", i);
            for (int t = 0; t < r.n_ctx; ++t)
                if ((uint32_t)r.ctx_tokens[t] >= (uint32_t)m.vocab)
                    return fail(CF_ERR_INVALID_ARG, "cf_restore_dynamic: request %d token %d out of vocab", i, t);
            hipPointerAttribute_t at;
            void* dp = nullptr;
            if (hipPointerGetAttributes(&at, r.host_kv) != hipSuccess || at.type != hipMemoryTypeHost ||
                hipHostGetDevicePointer(&dp, const_cast<void*>(r.host_kv), 0) != hipSuccess || !dp) {
                (void)hipGetLastError();
                return fail(CF_ERR_INVALID_ARG, "cf_restore_dynamic: request %d: host KV must be pinned, "
                            "device-mapped memory", i);
            }
            host_dev[i] = (const char*)dp;
            int np_ctx = (int)ceil_div(r.n_ctx, CF_PAGE_TOKENS);
            if ((int64_t)np_ctx * (int64_t)(pb / 16) >= ((int64_t)1 << 31))
                return fail(CF_ERR_WORKSPACE, "cf_restore_dynamic: request %d holds more than 32 GiB per layer", i);
        }
        if (logits_out) {
            if (r.n_new <= 0)
                return fail(CF_ERR_INVALID_ARG, "cf_restore_dynamic: request %d needs n_new > 0 for logits", i);
            sum_new += r.n_new;
            for (int t = 0; t < r.n_new; ++t)
                if ((uint32_t)r.new_tokens[t] >= (uint32_t)m.vocab)
                    return fail(CF_ERR_INVALID_ARG, "cf_restore_dynamic: request %d new token %d out of vocab", i, t);
        }
        n_ctx[i] = r.n_ctx;
        mode[i] = (opts->force_mode == CF_TOKEN_WISE || opts->force_mode == CF_LAYER_WISE)
                      ? opts->force_mode : (r.n_ctx >= opts->l_delta ? CF_TOKEN_WISE : CF_LAYER_WISE);
        n_units[i] = r.n_ctx <= 0 ? 0 : (mode[i] == CF_TOKEN_WISE ? (int)ceil_div(r.n_ctx, C) : L);
        p_io[i] = n_units[i] - 1;
        if (r.n_ctx > 0 && mode[i] == CF_LAYER_WISE) rows_lw += r.n_ctx;
        if (r.n_ctx > 0 && mode[i] == CF_TOKEN_WISE) ++n_tw;
        pt_off[i] = total_pt;
        n_pages_req[i] = np;
        total_pt += np;
    }
    if (int dup = first_repeated_id(reqs, B); dup >= 0)
        return fail(CF_ERR_INVALID_ARG, "cf_restore_dynamic: request %d repeats the id %llu of an earlier request "
                    "of the batch", dup, (unsigned long long)reqs[dup].req_id);
    if (rows_lw + n_tw * C + sum_new > c->opts.max_tokens)
        return fail(CF_ERR_WORKSPACE, "cf_restore_dynamic: %lld layer-wise rows + %lld token-wise chunks of %d + "
                    "%lld new tokens exceed max_tokens %d", (long long)rows_lw, (long long)n_tw, C,
                    (long long)sum_new, c->opts.max_tokens);
    // argument check of the scheduling calls once, so that later calls cannot fail
    {
        int32_t pick = -1;
        int rc0 = cf_dynamic_io_pick(cost, opts, B, n_ctx.data(), p_comp.data(), p_io.data(), nullptr, 0, 0,
                                     1000, 1000, &pick);
        if (rc0) return rc0;
    }

    // ---- metadata written once: page tables, the jobs of every possible load unit, the packed
    // rows of the layer-wise group and of the new-turn rows.  What follows is rewritten per step.
    MetaWriter mw{c->meta_host, c->cv.meta_bytes};
    {
        std::vector<int32_t> all_pt(std::max(total_pt, 1));
        for (int i = 0; i < B; ++i)
            if (n_pages_req[i]) std::memcpy(&all_pt[pt_off[i]], pt[i], (size_t)n_pages_req[i] * 4);
        mw.put(all_pt.data(), all_pt.size() * 4);
    }
    auto slot_of = [&](int i, int t) { return pt[i][t / CF_PAGE_TOKENS] * CF_PAGE_TOKENS + t % CF_PAGE_TOKENS; };
    const int split_heads = (!c->simple_only && attention_mfma_supported(m.dtype, m.head_dim, m.n_q_heads, m.n_kv_heads))
                                ? m.n_q_heads : 0;
    const int hpb = split_heads ? attention_mfma_heads_per_block(m.n_q_heads, m.n_kv_heads) : 1;
    auto add_segment = [&](Phase& ph, std::vector<int32_t>& ids, std::vector<int32_t>& pos,
                           std::vector<int32_t>& slot, int i, const int32_t* toks, int n_rows, int pos0,
                           int layers, bool is_new) {
        ph.segs.push_back(Segment{i, ph.T, n_rows, pos0, layers, is_new});
        ph.seg_boundary.push_back(nullptr);
        for (int t = 0; t < n_rows; ++t) {
            ids.push_back(toks[t]);
            pos.push_back(pos0 + t);
            slot.push_back(slot_of(i, pos0 + t));
        }
        ph.T += n_rows;
    };
    auto finish_phase = [&](Phase& ph, std::vector<int32_t>& ids, std::vector<int32_t>& pos,
                            std::vector<int32_t>& slot) {
        build_chunks(ph, c->cv.chunk_rows, pt_off, split_heads, hpb);
        ph.off_ids = mw.put(ids.data(), ids.size() * 4);
        ph.off_pos = mw.put(pos.data(), pos.size() * 4);
        ph.off_slot = mw.put(slot.data(), slot.size() * 4);
        ph.off_work = mw.put(ph.work.data(), ph.work.size() * sizeof(AttnWork));
        ph.off_grp = mw.put(ph.groups.data(), ph.groups.size() * sizeof(AttnCombine));
    };

    // load units: token-wise request i, unit u = chunk u in all layers; layer-wise group, unit
    // l = layer l of every layer-wise request
    std::vector<PageJob> jobs;
    std::vector<std::vector<DynUnitLoad>> tw_units(B);
    std::vector<DynUnitLoad> lw_units;
    std::vector<int> lw_members;
    int64_t vec_per_page = (int64_t)(pb / 16);
    auto add_job = [&](DynUnitLoad& ul, int i, int l, int lo, int hi) {
        int np_ctx = (int)ceil_div(n_ctx[i], CF_PAGE_TOKENS);
        int j = lo / CF_PAGE_TOKENS, j1 = (int)ceil_div(hi, CF_PAGE_TOKENS);
        PageJob jb;
        jb.staging_off = (int64_t)(uintptr_t)(host_dev[i] + ((size_t)l * np_ctx + j) * pb);
        jb.layer = l;
        jb.pt_off = pt_off[i];
        jb.page_first = j;
        jb.n_pages = j1 - j;
        jb.tok_first = lo;
        jb.tok_end = hi;
        jb.block_first = ul.n_vblocks;
        jb.pad = 0;
        jobs.push_back(jb);
        ++ul.n_jobs;
        ul.n_vblocks += (int)ceil_div((int64_t)(j1 - j) * vec_per_page, PAGE_LOAD_UNIT_VECS);
        ul.bytes += (size_t)(j1 - j) * pb;
    };
    for (int i = 0; i < B; ++i) {
        if (n_units[i] == 0) continue;
        if (mode[i] == CF_TOKEN_WISE) {
            for (int u = 0; u < n_units[i]; ++u) {
                DynUnitLoad ul{(int)jobs.size(), 0, 0, 0};
                int lo = u * C, hi = std::min(n_ctx[i], lo + C);
                for (int l = 0; l < L; ++l) add_job(ul, i, l, lo, hi);
                ul.page_first = lo / CF_PAGE_TOKENS;
                ul.n_pages = (int)ceil_div(hi, CF_PAGE_TOKENS) - ul.page_first;
                ul.dma_ok = c->load_path == 0 && hi % CF_PAGE_TOKENS == 0;
                for (int pg = ul.page_first + 1; ul.dma_ok && pg < ul.page_first + ul.n_pages; ++pg)
                    ul.dma_ok = pt[i][pg] == pt[i][pg - 1] + 1;
                ul.joins_prev = ul.page_first > 0 && pt[i][ul.page_first] == pt[i][ul.page_first - 1] + 1;
                tw_units[i].push_back(ul);
            }
        } else {
            lw_members.push_back(i);
        }
    }
    if (!lw_members.empty())
        for (int l = 0; l < L; ++l) {
            DynUnitLoad ul{(int)jobs.size(), 0, 0, 0};
            for (int i : lw_members) add_job(ul, i, l, 0, n_ctx[i]);
            lw_units.push_back(ul);
        }
    size_t off_jobs = mw.put(jobs.data(), jobs.size() * sizeof(PageJob));

    Phase lw;
    {
        std::vector<int32_t> ids, pos, slot;
        for (int i : lw_members) add_segment(lw, ids, pos, slot, i, reqs[i].ctx_tokens, n_ctx[i], 0, L, false);
        if (lw.T > 0) finish_phase(lw, ids, pos, slot);
    }
    c->n_last = 0;
    if (mw.overflow)
        return fail(CF_ERR_WORKSPACE, "cf_restore_dynamic: batch metadata exceeds the context's limits "
                    "(%zu load jobs)", jobs.size());
    const size_t step_off = mw.off;      // per-step arrays start here, every step

    // ---- events: one per load unit in flight, one for the compute step.  The copy stream is
    // kept one unit deep, plus more while less than IO_LOOKAHEAD_PS of predicted work is queued
    // (short units need the next launches queued behind them; long ones are claimed one at a time
    // so that the claim is made as late as possible)
    constexpr int IO_DEPTH = 8;
    constexpr int64_t IO_LOOKAHEAD_PS = 4000000000;
    constexpr size_t IO_MERGE_BYTES = (size_t)256 << 20;
    constexpr size_t IO_MERGE_RUN_BYTES = (size_t)8 << 20;
    // events [0, IO_DEPTH): end of the load in that slot; [IO_DEPTH]: the compute step;
    // (IO_DEPTH, 2 IO_DEPTH]: start of the load in that slot (its duration is read on the GPU's
    // clock: the host sees completions late whenever it is busy enqueuing a step)
    // [2 IO_DEPTH + 1]: start of the planned tail's loads
    while ((int)c->dyn_events.size() < 2 * IO_DEPTH + 2) {
        hipEvent_t e = nullptr;
        CF_HIP(hipEventCreate(&e));
        c->dyn_events.push_back(e);
    }
    hipEvent_t ev_step = c->dyn_events[IO_DEPTH];

    char* md = c->meta_dev();
    std::fill(c->waited.begin(), c->waited.end(), 0);
    CF_HIP(hipEventRecord(c->ev_start, c->cs));
    CF_HIP(hipMemcpyAsync(md, c->meta_host, step_off, hipMemcpyHostToDevice, c->cs));
    CF_HIP(hipEventRecord(c->ev_meta, c->cs));
    CF_HIP(hipStreamWaitEvent(c->ps, c->ev_meta, 0));
    KvGeom g;
    g.n_kv_heads = m.n_kv_heads;
    g.head_dim = m.head_dim;
    g.page_elems = (int64_t)(pb / es);
    g.layer_stride = g.page_elems * cache->n_pages;
    double paced_bytes = 0;
    if (c->throttle_gbs > 0) launch_pace_mark(c->ps, c->pace_dev());
    // an error once work is enqueued: let both streams drain before the caller gets control back
    // (its buffers are in use until then)
    auto bail = [&](int code) {
        (void)hipStreamSynchronize(c->cs);
        (void)hipStreamSynchronize(c->ps);
        (void)hipStreamSynchronize(c->ss);       // the second DMA queue of the planned tail
        (void)hipGetLastError();
        c->prof_collect();
        return code;
    };

    // ---- the scheduling loop
    // Layer-wise members share their pointers (the group moves as one).  closed[i]: the compute
    // engine is done with request i for good (the group ran its last layer K/V-only, so there are
    // no hidden states to go on from); the I/O channel takes what is left of it.
    // A request whose cache is complete (pointers crossed, its loads landed, its last recompute
    // step done) has its new-turn rows prefilled in the next compute step, beside whatever else
    // that step recomputes: the new turn of early finishers overlaps the loads of the others.
    // req: the token-wise request, or -1 = layer-wise group; beside: issued while a recompute step ran
    struct Flight { int64_t pred_ps; int req; double t_issue; bool beside; };
    std::deque<Flight> io_flight;                 // loads in flight, oldest first
    int64_t io_issued = 0, io_retired = 0;        // event of load k: dyn_events[k % IO_DEPTH]
    // predicted ps / measured ms of the retired loads, by whether a recompute step ran beside them
    int64_t io_pred_beside = 0, io_pred_alone = 0;
    double io_ms_beside = 0, io_ms_alone = 0;
    double io_t_last = 0;                         // host clock: latest completion
    // c_pred_done: what the finished steps were predicted to take at scale 1 (a step's prediction
    // is made at the scale of the moment, which is taken out again: the ratio measured /
    // predicted is the scale itself, not a correction of the scale in use)
    int64_t c_pred_done = 0, step_pred = 0;
    int step_scale = 1000;                        // the compute scale the running step was predicted at
    double c_meas_done_ms = 0, step_t0 = 0, gap_ms = 0, last_step_end = 0;
    bool step_running = false, ask = true;        // ask: state changed since the last declined claim
    bool step_has_rec = false;                    // the running step recomputes (contends with the channel)
    bool force_io = false, tail_ran = false, merged_last = false;
    bool tail_timed = false, tail_beside = false;
    int64_t tail_pred = 0;                        // predicted ps of the planned tail's loads
    // the ratios measured / predicted start from what the previous call on this context saw
    int scale_c = c->dyn_scale_c, scale_io = c->dyn_scale_io, scale_io_alone = c->dyn_scale_io_alone;
    int n_steps = 0, n_cunits = 0;
    // the channel's scale as things stand: beside a recomputing step, or on its own
    auto sio_now = [&]() { return step_has_rec ? scale_io : scale_io_alone; };
    int64_t loaded_bytes = 0;
    int lw_layer = 0;                             // next layer of the layer-wise group
    std::vector<uint8_t> closed(B, 0);
    std::vector<int32_t> take(B);
    std::vector<int> io_pending(B, 0);            // loads in flight that touch request i
    std::vector<char> in_step(B, 0), prefilled(B, 0);
    int n_prefilled = 0;
    const bool want_new = logits_out != nullptr;
    auto clamp_scale = [](double r) { return (int)std::min(4000.0, std::max(250.0, r * 1000.0 + 0.5)); };
    auto unit_load_ps = [&](size_t bytes) {
        __int128 num = (__int128)bytes * cost->gamma;
        return cost->f_io + (int64_t)((num + (((__int128)1) << 20) - 1) >> 20);
    };
    auto restored = [&](int i) { return p_comp[i] > p_io[i] && io_pending[i] == 0 && !in_step[i]; };
    CF_HIP(hipEventRecord(c->ev_comp, c->cs));    // stands if the compute engine claims nothing
    CF_HIP(hipEventRecord(c->ev_copy, c->ps));    // stands if the channel loads nothing
    // event state: 1 complete, 0 pending, -1 the runtime reports a failure
    auto done = [](hipEvent_t e) {
        hipError_t q = hipEventQuery(e);
        if (q == hipSuccess) return 1;
        (void)hipGetLastError();
        return q == hipErrorNotReady ? 0 : -1;
    };
    double t_progress = now_ms();
    constexpr double STALL_LIMIT_MS = 60000;      // no completion for this long: give up, do not spin for ever

    // The copy stream's side of the loop; also called between the layers of a step that is being
    // enqueued, so that the channel does not run dry while the host is busy launching.
    // Returns < 0 on failure, else whether anything changed.
    auto pump_io = [&]() -> int {
        int changed = 0;
        while (!io_flight.empty()) {              // retire finished loads (they complete in issue order)
            int dn = done(c->dyn_events[io_retired % IO_DEPTH]);
            if (dn < 0) return -1;
            if (dn == 0) break;
            // what the channel spent on this load, on the GPU's clock (idle gaps between claims
            // are not load time, and the host may notice a completion late)
            float load_ms = 0;
            if (hipEventElapsedTime(&load_ms, c->dyn_events[IO_DEPTH + 1 + io_retired % IO_DEPTH],
                                    c->dyn_events[io_retired % IO_DEPTH]) != hipSuccess) {
                (void)hipGetLastError();
                load_ms = (float)(now_ms() - std::max(io_flight.front().t_issue, io_t_last));
            }
            io_t_last = now_ms();
            if (io_flight.front().beside || step_has_rec) {
                io_ms_beside += load_ms;
                io_pred_beside += io_flight.front().pred_ps;
                if (io_pred_beside > 0 && io_ms_beside > 0)
                    scale_io = clamp_scale(io_ms_beside * 1e9 / (double)io_pred_beside);
            } else {
                io_ms_alone += load_ms;
                io_pred_alone += io_flight.front().pred_ps;
                if (io_pred_alone > 0 && io_ms_alone > 0)
                    scale_io_alone = clamp_scale(io_ms_alone * 1e9 / (double)io_pred_alone);
            }
            int r = io_flight.front().req;
            if (r >= 0) --io_pending[r];
            else for (int i : lw_members) --io_pending[i];
            io_flight.pop_front();
            ++io_retired;
            changed = 1;
        }
        while ((int)io_flight.size() < IO_DEPTH) {
            const int sio = sio_now();
            int64_t backlog = 0;
            for (const Flight& f : io_flight) backlog += (int64_t)((__int128)f.pred_ps * sio / 1000);
            if (!io_flight.empty() && backlog >= IO_LOOKAHEAD_PS) break;
            int64_t busy = 0;
            if (step_running)
                busy = std::max<int64_t>(0, step_pred - (int64_t)((now_ms() - step_t0) * 1e9));
            // both engines idle and both declined (cannot happen with consistent costs): the channel takes it
            if (force_io) busy = INT64_MAX / 4;
            force_io = false;
            int32_t pick = -1;
            cf_dynamic_io_pick(cost, opts, B, n_ctx.data(), p_comp.data(), p_io.data(), closed.data(), backlog,
                               busy, scale_c, sio, &pick);
            if (pick < 0) break;
            // A token-wise claim grows by the units below it, as long as the same test keeps
            // naming the same request, up to IO_MERGE_BYTES: long runs of consecutive pages
            // can go by DMA, and either way the channel runs at link speed only on long transfers.
            std::vector<int> us;                  // token-wise: the units of this claim, far end first
            size_t bytes = 0;
            int64_t pred = 0;
            int who;
            if (mode[pick] == CF_TOKEN_WISE) {
                who = pick;
                while (true) {
                    const DynUnitLoad& u = tw_units[pick][p_io[pick]];
                    us.push_back(p_io[pick]);
                    --p_io[pick];
                    bytes += u.bytes;
                    pred += unit_load_ps(u.bytes);
                    // long enough as a whole, and per layer (a unit's bytes are spread over L runs)
                    if ((bytes >= IO_MERGE_BYTES && bytes >= (size_t)L * IO_MERGE_RUN_BYTES) ||
                        bytes >= 4 * IO_MERGE_BYTES || p_comp[pick] > p_io[pick])
                        break;
                    int32_t again = -1;
                    cf_dynamic_io_pick(cost, opts, B, n_ctx.data(), p_comp.data(), p_io.data(), closed.data(),
                                       backlog + (int64_t)((__int128)pred * sio / 1000), busy, scale_c, sio, &again);
                    if (again != pick) break;
                }
                ++io_pending[pick];
            } else {
                bytes = lw_units[p_io[pick]].bytes;
                pred = unit_load_ps(bytes);
                for (int i : lw_members) ++io_pending[i];
                who = -1;
            }
            c->prof_begin(CF_K_H2D_COPY, (double)bytes, c->ps);
            if (hipEventRecord(c->dyn_events[IO_DEPTH + 1 + io_issued % IO_DEPTH], c->ps) != hipSuccess) return -1;
            auto kernel_load = [&](const DynUnitLoad& ul) {
                launch_page_load(c->ps, m.dtype, cache->pool, (const PageJob*)(md + off_jobs) + ul.job_first,
                                 ul.n_jobs, ul.n_vblocks, c->load_wgs, (const int32_t*)md, g);
            };
            if (who >= 0) {
                // bottom unit first; consecutive units whose pages follow one another in the pool
                // form one run: a transfer per layer if that is long enough, else their kernels
                const int np_ctx = (int)ceil_div(n_ctx[pick], CF_PAGE_TOKENS);
                for (size_t k = us.size(); k > 0;) {
                    const DynUnitLoad& first = tw_units[pick][us[k - 1]];
                    size_t e = k - 1;             // the run is us[e .. k-1], ascending as e falls
                    int pages = first.n_pages;
                    if (first.dma_ok)
                        while (e > 0 && tw_units[pick][us[e - 1]].dma_ok && tw_units[pick][us[e - 1]].joins_prev) {
                            --e;
                            pages += tw_units[pick][us[e]].n_pages;
                        }
                    if (first.dma_ok && (size_t)pages * pb >= DMA_MIN_BYTES) {
                        for (int l = 0; l < L; ++l)
                            if (hipMemcpyAsync((char*)cache->pool + ((size_t)l * cache->n_pages + pt[pick][first.page_first]) * pb,
                                               (const char*)reqs[pick].host_kv + ((size_t)l * np_ctx + first.page_first) * pb,
                                               (size_t)pages * pb, hipMemcpyHostToDevice, c->ps) != hipSuccess)
                                return -1;
                    } else {
                        for (size_t q = k; q > e; --q) kernel_load(tw_units[pick][us[q - 1]]);
                    }
                    k = e;
                }
            } else {
                kernel_load(lw_units[p_io[pick]]);
                for (int i : lw_members) --p_io[i];
            }
            if (c->throttle_gbs > 0) {
                paced_bytes += (double)bytes;
                launch_pace_wait(c->ps, c->pace_dev(),
                                 (unsigned long long)(paced_bytes / (c->throttle_gbs * 1e9) * c->wall_hz));
            }
            c->prof_end(CF_K_H2D_COPY, c->ps);
            if (hipEventRecord(c->dyn_events[io_issued % IO_DEPTH], c->ps) != hipSuccess ||
                hipEventRecord(c->ev_copy, c->ps) != hipSuccess)       // the latest record stands
                return -1;
            io_flight.push_back(Flight{pred, who, now_ms(), step_has_rec});
            loaded_bytes += (int64_t)bytes;
            ++io_issued;
            changed = 1;
        }
        return changed;
    };
    std::function<int()> between_layers = [&]() { return pump_io() < 0 ? -1 : 0; };

    // Recompute segments of a step: take[i] consecutive chunks of token-wise request i, from its
    // compute pointer on, as one segment; the pointer moves past them.
    auto add_recompute = [&](Phase& step, std::vector<int32_t>& ids, std::vector<int32_t>& pos,
                             std::vector<int32_t>& slot, const std::vector<int32_t>& tk) {
        bool any = false;
        for (int i = 0; i < B; ++i) {
            if (!tk[i] || mode[i] != CF_TOKEN_WISE) continue;
            const int lo = p_comp[i] * C, hi = std::min(n_ctx[i], lo + tk[i] * C);
            add_segment(step, ids, pos, slot, i, reqs[i].ctx_tokens + lo, hi - lo, lo, L, false);
            p_comp[i] += tk[i];
            n_cunits += tk[i];
            in_step[i] = 1;
            any = true;
        }
        return any;
    };

    // The planned tail.  Once the compute engine will take nothing more, the schedule is known,
    // so the rest is laid out like a planned restore: the channel gets every unclaimed cell,
    // layer by layer from the bottom with an event per layer, and the new turn of every request
    // not yet prefilled is enqueued right away (behind the running step, if there is one); its
    // attention in layer l waits for that layer's event only.  `fresh`: requests known to be
    // restored already (merged into the list of all that are not prefilled).  `last_take`: the
    // units of the compute engine's last recompute step, when that step was recognised as the
    // last before it was launched -- it then runs in the same pass as the new turns, the way a
    // planned restore packs them.
    auto launch_tail = [&](std::vector<int> fresh, int64_t pred_ps, bool behind_step,
                           const std::vector<int32_t>* last_take) -> int {
        Phase step;
        std::vector<int32_t> ids, pos, slot, last_idx;
        const bool with_rec = last_take && add_recompute(step, ids, pos, slot, *last_take);
        std::vector<PageJob> tjobs;
        std::vector<DmaOp> tdma;
        std::vector<LayerLoad> tlayers(L);
        for (int l = 0; l < L; ++l) {
            tlayers[l] = LayerLoad{l, (int)tjobs.size(), 0, 0, 0, (int)tdma.size(), 0};
            for (int i = 0; i < B; ++i) {
                if (p_comp[i] > p_io[i]) continue;
                int lo, hi;
                if (mode[i] == CF_TOKEN_WISE) {
                    lo = p_comp[i] * C;
                    hi = std::min(n_ctx[i], (p_io[i] + 1) * C);
                } else if (l >= p_comp[i] && l <= p_io[i]) {
                    lo = 0;
                    hi = n_ctx[i];
                } else {
                    continue;
                }
                const int np_ctx = (int)ceil_div(n_ctx[i], CF_PAGE_TOKENS);
                split_load_run(tjobs, tdma, tlayers[l], pt[i], pt_off[i], host_dev[i] + (size_t)l * np_ctx * pb,
                               (const char*)reqs[i].host_kv + (size_t)l * np_ctx * pb,
                               (char*)cache->pool + (size_t)l * cache->n_pages * pb, pb, l, lo, hi,
                               c->load_path == 0);
            }
        }
        for (int i = 0; i < B; ++i) {
            if (p_comp[i] <= p_io[i]) p_io[i] = p_comp[i] - 1;     // claimed by the channel
            if (prefilled[i]) continue;
            add_segment(step, ids, pos, slot, i, reqs[i].new_tokens, reqs[i].n_new, n_ctx[i], L, true);
            last_idx.push_back(step.T - 1);
            fresh.push_back(i);
        }
        std::sort(fresh.begin(), fresh.end());    // = every request not prefilled, in segment order
        fresh.erase(std::unique(fresh.begin(), fresh.end()), fresh.end());
        // metadata: behind a running step its arrays are still in use (the copy of them may not
        // even have left the pinned mirror yet), so the tail's go after them
        if (!behind_step) mw.off = step_off;
        // as in the planned restore: when the load kernel only has the ragged ends, one launch
        // ahead of the first transfer moves them for all layers (units numbered through)
        int64_t tail_kernel_bytes = 0, tail_bytes = 0;
        int tail_units = 0;
        for (const PageJob& jb : tjobs) tail_kernel_bytes += (int64_t)jb.n_pages * (int64_t)pb;
        for (const LayerLoad& tl : tlayers) tail_bytes += (int64_t)tl.bytes;
        const bool tail_upfront = !tdma.empty() && tail_kernel_bytes > 0 && tail_kernel_bytes * 64 <= tail_bytes;
        if (tail_upfront)
            for (const LayerLoad& tl : tlayers) {
                for (int k = 0; k < tl.n_jobs; ++k) tjobs[tl.job_first + k].block_first += tail_units;
                tail_units += tl.n_vblocks;
            }
        const size_t off_tjobs = mw.put(tjobs.data(), tjobs.size() * sizeof(PageJob));
        const size_t off_rows = mw.off;
        finish_phase(step, ids, pos, slot);
        const size_t off_idx = mw.put(last_idx.data(), last_idx.size() * 4);
        if (mw.overflow)
            return bail(fail(CF_ERR_WORKSPACE, "cf_restore_dynamic: step metadata exceeds the context's limits"));
        // the jobs travel on the copy stream (it must not wait for the running step), the new
        // turn's arrays on the compute stream
        if (off_rows > off_tjobs)
            CF_HIP(hipMemcpyAsync(md + off_tjobs, c->meta_host + off_tjobs, off_rows - off_tjobs,
                                  hipMemcpyHostToDevice, c->ps));
        CF_HIP(hipMemcpyAsync(md + off_rows, c->meta_host + off_rows, mw.off - off_rows,
                              hipMemcpyHostToDevice, c->cs));
        // Layer l's loads go onto the copy stream right before layer l's kernels go onto the
        // compute stream (a layer's event is recorded before anything waits for it; the host,
        // which issues a transfer per request and layer, never holds the compute stream back).
        std::vector<hipEvent_t> ready(L);
        for (int l = 0; l < L; ++l) ready[l] = c->ev_layer[l];
        int tail_next = 0;
        bool tail_q2_recorded = false;
        auto feed_layer = [&]() -> int {
            if (tail_next >= L) return 0;
            if (tail_next == 0) {
                // the tail's loads are timed as one: from here to the copy stream's end
                if (hipEventRecord(c->dyn_events[2 * IO_DEPTH + 1], c->ps) != hipSuccess) return -1;
                tail_timed = true;
                tail_beside = step_has_rec || with_rec;
                if (tail_upfront)
                    launch_page_load(c->ps, m.dtype, cache->pool, (const PageJob*)(md + off_tjobs), (int)tjobs.size(),
                                     tail_units, c->load_wgs, (const int32_t*)md, g);
            }
            const LayerLoad& tl = tlayers[tail_next];
            if (tl.n_jobs > 0 || tl.n_dma > 0) {
                c->prof_begin(CF_K_H2D_COPY, (double)tl.bytes, c->ps);
                if (issue_layer_dma(c->ps, c->ss, c->ev_q2, c->ev_scat, c->dma_queues > 1 && c->throttle_gbs <= 0,
                                    tail_q2_recorded, tdma.data() + tl.dma_first, tl.n_dma) < 0)
                    return -1;
                if (!tail_upfront)
                    launch_page_load(c->ps, m.dtype, cache->pool, (const PageJob*)(md + off_tjobs) + tl.job_first,
                                     tl.n_jobs, tl.n_vblocks, c->load_wgs, (const int32_t*)md, g);
                if (c->throttle_gbs > 0) {
                    paced_bytes += (double)tl.bytes;
                    launch_pace_wait(c->ps, c->pace_dev(),
                                     (unsigned long long)(paced_bytes / (c->throttle_gbs * 1e9) * c->wall_hz));
                }
                c->prof_end(CF_K_H2D_COPY, c->ps);
                loaded_bytes += (int64_t)tl.bytes;
                tail_pred += unit_load_ps(tl.bytes);
                ++io_issued;
                if (end_layer_dma(c->ps, c->ev_q2, tail_q2_recorded) < 0) return -1;
            }
            // behind everything the copy stream was given so far, units in flight included
            if (hipEventRecord(c->ev_layer[tail_next], c->ps) != hipSuccess) return -1;
            ++tail_next;
            return 0;
        };
        const std::function<int()> feed = [&]() -> int { return (pump_io() < 0 || feed_layer() < 0) ? -1 : 0; };
        if (!behind_step) {
            double t_launch = now_ms();
            if (n_steps > 0) gap_ms += t_launch - last_step_end;
            step_t0 = t_launch;
            step_pred = 0;
            step_scale = scale_c;
            ++n_steps;
        }
        step_pred += pred_ps;
        step_running = true;
        step_has_rec = step_has_rec || with_rec;
        int rc2 = run_phase(c, cache, step, L, ready.data(), nullptr, 0, lw.T, &feed);
        if (rc2) return bail(rc2);
        while (tail_next < L)
            if (feed_layer() < 0) return bail(fail(CF_ERR_HIP, "cf_restore_dynamic: enqueuing a load failed"));
        CF_HIP(hipEventRecord(c->ev_copy, c->ps));
        if (with_rec) CF_HIP(hipEventRecord(c->ev_comp, c->cs));
        // final norm of every request's last row into its LM-head slot (last_idx[k] belongs to
        // fresh[k]); the last layer's down-proj result is still pending in dl
        for (size_t k = 0; k < fresh.size(); ++k) {
            int i = fresh[k];
            launch_rmsnorm(c->cs, m.dtype, c->h() + (size_t)lw.T * m.d_model,
                           c->dl() + (size_t)lw.T * m.d_model, c->w.final_norm,
                           (char*)c->a_last() + (size_t)i * m.d_model * es, 1, m.d_model, m.rms_eps,
                           (const int32_t*)(md + off_idx) + k);
            launch_residual_gather(c->cs, c->h_last() + (size_t)i * m.d_model, c->h() + (size_t)lw.T * m.d_model,
                                   c->dl() + (size_t)lw.T * m.d_model, (const int32_t*)(md + off_idx) + k, 1,
                                   m.d_model, 0, INT32_MAX, 0, 0);
            prefilled[i] = 1;
            ++n_prefilled;
        }
        CF_HIP(hipEventRecord(ev_step, c->cs));   // the running step, if any, now ends here
        tail_ran = true;
        merged_last = merged_last || with_rec;
        return CF_OK;
    };

    // rows a step may hold beside the layer-wise group's and every request's new turn
    const int64_t step_rows_cap = (int64_t)c->opts.max_tokens - lw.T - sum_new;

    // The compute engine is asked first: if its first step turns out to be its last, the whole
    // schedule is known before anything is loaded, and every load goes out layer by layer (a
    // chunk claimed by the channel ahead of that, all its layers in one piece, would hold back
    // the bottom layers that the new turn waits for).
    bool first_round = true;
    while (true) {
        bool progressed = false;
        int pio_rc = first_round ? 0 : pump_io();
        first_round = false;
        if (pio_rc < 0) return bail(fail(CF_ERR_HIP, "cf_restore_dynamic: the copy stream failed"));
        if (pio_rc > 0) progressed = ask = true;
        // compute engine: retire the step ...
        int step_dn = step_running ? done(ev_step) : 0;
        if (step_dn < 0) return bail(fail(CF_ERR_HIP, "cf_restore_dynamic: the compute stream failed"));
        if (step_dn > 0) {
            last_step_end = now_ms();
            c_meas_done_ms += last_step_end - step_t0;
            c_pred_done += (int64_t)((__int128)step_pred * 1000 / step_scale);
            if (c_pred_done > 0) scale_c = clamp_scale(c_meas_done_ms * 1e9 / (double)c_pred_done);
            step_running = false;
            step_has_rec = false;
            std::fill(in_step.begin(), in_step.end(), 0);
            progressed = ask = true;
        }
        // ... and ask for the next one (again after every change of state while it is idle)
        if (!step_running && ask) {
            ask = false;
            // new-turn rows of the requests that are completely restored by now
            // (and the cost of the new turns that are still to come: the compute engine has that
            // work ahead of it whatever it takes now)
            std::vector<int> fresh;
            int64_t fixed = 0, later = 0;
            if (want_new)
                for (int i = 0; i < B; ++i) {
                    if (prefilled[i]) continue;
                    int64_t ps = 0;
                    cf_prefill_cost(cost, L, 1, &n_ctx[i], &reqs[i].n_new, &ps);
                    ps = (int64_t)((__int128)ps * scale_c / 1000);
                    if (restored(i)) { fresh.push_back(i); fixed += ps; }
                    else later += ps;
                }
            // every pass over the layers has a launch-bound floor, the cost model's compute
            // start-up: this step pays it, and so does the new-turn pass that is still to come
            {
                const int64_t floor_ps = (int64_t)((__int128)cost->s_c * scale_c / 1000);
                fixed += floor_ps;
                if (later > 0) later += floor_ps;
            }
            // the channel is priced as it runs beside a recomputing engine; what the units must
            // beat is the channel on its own
            int64_t backlog = 0, pred = 0;
            for (const Flight& f : io_flight) backlog += (int64_t)((__int128)f.pred_ps * scale_io / 1000);
            cf_dynamic_claim(cost, opts, B, n_ctx.data(), p_comp.data(), p_io.data(), closed.data(), backlog,
                             fixed, later, step_cap, order, scale_c, scale_io, units_cap, scale_io_alone,
                             take.data(), &pred);
            // a step holds no more rows than the workspace has for it: the rest stays unclaimed
            {
                int64_t rows = 0;
                for (int i = 0; i < B; ++i) {
                    if (!take[i] || mode[i] != CF_TOKEN_WISE) continue;
                    const int lo = p_comp[i] * C;
                    while (take[i] > 0 && rows + std::min(n_ctx[i], lo + take[i] * C) - lo > step_rows_cap) --take[i];
                    if (take[i] > 0) rows += std::min(n_ctx[i], lo + take[i] * C) - lo;
                }
            }
            Phase step;
            std::vector<int32_t> ids, pos, slot, last_idx;
            bool lw_take = false, lw_last = false, any_rec = false, any_live = false;
            for (int i = 0; i < B; ++i) {
                any_rec |= take[i] != 0;
                any_live |= p_comp[i] <= p_io[i];
                if (take[i] && mode[i] != CF_TOKEN_WISE) {
                    lw_take = true;
                    lw_last = take[i] == 2;
                }
            }
            if (!any_rec && any_live && want_new) {
                // idle and nothing worth taking: the rest is the channel's
                int rc2 = launch_tail(fresh, fixed + later, false, nullptr);
                if (rc2) return bail(rc2);
                continue;
            }
            // Will there be anything to take when this step is over?  Ask for the state it
            // leaves behind, with the step's own duration counted as work still ahead (the
            // channel keeps loading meanwhile).  If not, this is the last recompute step and the
            // rest of the schedule is known now.  Without a layer-wise group the step then carries
            // the planned tail itself: one pass holds the recompute rows and every outstanding
            // new turn, beside the remaining loads laid out layer by layer.  With a group (whose
            // rows keep their own place in the workspace) the tail follows as a pass of its own.
            bool last_step = false;
            if (any_rec && want_new) {
                std::vector<int32_t> pc2(p_comp);
                for (int i = 0; i < B; ++i)
                    if (take[i]) pc2[i] += mode[i] == CF_TOKEN_WISE ? take[i] : 1;
                bool live_left = false;
                for (int i = 0; i < B; ++i)
                    live_left |= pc2[i] <= p_io[i] && !(closed[i] || (mode[i] != CF_TOKEN_WISE && take[i] == 2));
                last_step = true;
                if (live_left) {
                    std::vector<int32_t> take2(B, 0);
                    std::vector<uint8_t> closed2(closed);
                    for (int i = 0; i < B; ++i)
                        if (take[i] == 2 && mode[i] != CF_TOKEN_WISE) closed2[i] = 1;
                    cf_dynamic_claim(cost, opts, B, n_ctx.data(), pc2.data(), p_io.data(), closed2.data(), backlog,
                                     0, later + pred, 0, order, scale_c, scale_io, units_cap, 0, take2.data(),
                                     nullptr);
                    for (int i = 0; i < B; ++i) last_step &= take2[i] == 0;
                }
            }
            if (last_step && !lw_take && lw_members.empty()) {
                std::fill(in_step.begin(), in_step.end(), 0);
                int rc2 = launch_tail(fresh, pred + later, false, &take);
                if (rc2) return bail(rc2);
                progressed = true;
                continue;
            }
            add_recompute(step, ids, pos, slot, take);
            for (int i : fresh) {               // packed after the recompute rows
                add_segment(step, ids, pos, slot, i, reqs[i].new_tokens, reqs[i].n_new, n_ctx[i], L, true);
                last_idx.push_back(step.T - 1);
            }
            if (step.T > 0 || lw_take) {
                double t_launch = now_ms();
                if (n_steps > 0) gap_ms += t_launch - last_step_end;
                step_t0 = t_launch;
                step_pred = pred;
                step_scale = scale_c;
                step_running = true;            // pump_io (between layers) sees the step as running
                step_has_rec = any_rec;
                if (lw_take) {
                    // layer lw_layer of the group: in full if the group goes on, else up to its K/V write
                    for (Segment& sg : lw.segs) sg.layers = lw_layer + (lw_last ? 1 : 2);
                    for (int i : lw_members) in_step[i] = 1;
                    int rc2 = run_phase(c, cache, lw, lw_layer + 1, nullptr, nullptr, lw_layer, 0, &between_layers);
                    if (rc2) return bail(rc2);
                    for (int i : lw_members) {
                        ++p_comp[i];
                        ++n_cunits;
                        if (lw_last) closed[i] = 1;
                    }
                    ++lw_layer;
                }
                if (step.T > 0) {
                    mw.off = step_off;
                    finish_phase(step, ids, pos, slot);
                    size_t off_idx = mw.put(last_idx.data(), last_idx.size() * 4);
                    if (mw.overflow)
                        return bail(fail(CF_ERR_WORKSPACE, "cf_restore_dynamic: step metadata exceeds the context's limits"));
                    CF_HIP(hipMemcpyAsync(md + step_off, c->meta_host + step_off, mw.off - step_off,
                                          hipMemcpyHostToDevice, c->cs));
                    int rc2 = run_phase(c, cache, step, L, nullptr, nullptr, 0, lw.T, &between_layers);
                    if (rc2) return bail(rc2);
                    // final norm of each fresh request's last row into its slot of the LM-head input
                    // (the last layer's down-proj result is still pending in dl)
                    for (size_t k = 0; k < fresh.size(); ++k) {
                        int i = fresh[k];
                        launch_rmsnorm(c->cs, m.dtype, c->h() + (size_t)lw.T * m.d_model,
                                       c->dl() + (size_t)lw.T * m.d_model, c->w.final_norm,
                                       (char*)c->a_last() + (size_t)i * m.d_model * es, 1, m.d_model, m.rms_eps,
                                       (const int32_t*)(md + off_idx) + k);
                        launch_residual_gather(c->cs, c->h_last() + (size_t)i * m.d_model,
                                               c->h() + (size_t)lw.T * m.d_model, c->dl() + (size_t)lw.T * m.d_model,
                                               (const int32_t*)(md + off_idx) + k, 1, m.d_model, 0, INT32_MAX, 0, 0);
                        prefilled[i] = 1;
                        ++n_prefilled;
                    }
                }
                CF_HIP(hipEventRecord(ev_step, c->cs));
                if (any_rec) CF_HIP(hipEventRecord(c->ev_comp, c->cs));
                ++n_steps;
                progressed = true;
                // the last recompute step of a batch with a layer-wise group: the rest is planned
                // now and enqueued behind it, so that neither stream waits for the host to notice
                // the step's end
                if (last_step) {
                    int rc3 = launch_tail({}, later, true, nullptr);
                    if (rc3) return bail(rc3);
                }
            }
        }
        if (!step_running && io_flight.empty()) {
            bool live = false;
            for (int i = 0; i < B; ++i) live |= p_comp[i] <= p_io[i];
            if (!live && (!want_new || n_prefilled == B)) break;
            if (live && !progressed) force_io = true;
        }
        if (progressed) {
            t_progress = now_ms();
        } else {
            if (now_ms() - t_progress > STALL_LIMIT_MS)
                return bail(fail(CF_ERR_HIP, "cf_restore_dynamic: no unit completed within %.0f s", STALL_LIMIT_MS / 1e3));
            std::this_thread::sleep_for(std::chrono::microseconds(20));
        }
    }

    // ---- every cache is complete and every new turn prefilled: first-token logits
    if (logits_out) {
        gemm(c, CF_K_GEMM_LM_HEAD, c->a_last(), c->w.lm_head, nullptr, logits_out, nullptr, B, m.vocab, m.d_model, EPI_STORE_F32);
        c->n_last = B;
    }
    CF_HIP(hipEventRecord(c->ev_end, c->cs));
    CF_HIP(hipGetLastError());
    CF_HIP(hipStreamSynchronize(c->cs));
    CF_HIP(hipStreamSynchronize(c->ps));
    c->prof_collect();
    // the time the compute stream stood waiting for a layer's loads (the pass that carried the
    // planned tail) is not compute time: taken off before the ratio is carried to the next call
    float wait_ms = 0;
    for (int l = 0; l < L; ++l) {
        if (!c->waited[l]) continue;
        float w = 0;
        if (hipEventElapsedTime(&w, c->ev_wait[2 * l], c->ev_wait[2 * l + 1]) == hipSuccess) wait_ms += w;
        else (void)hipGetLastError();
    }
    if (tail_timed && tail_pred > 0) {
        float t_tail = 0;
        if (hipEventElapsedTime(&t_tail, c->dyn_events[2 * IO_DEPTH + 1], c->ev_copy) == hipSuccess && t_tail > 0) {
            if (tail_beside) {
                io_ms_beside += t_tail;
                io_pred_beside += tail_pred;
                scale_io = clamp_scale(io_ms_beside * 1e9 / (double)io_pred_beside);
            } else {
                io_ms_alone += t_tail;
                io_pred_alone += tail_pred;
                scale_io_alone = clamp_scale(io_ms_alone * 1e9 / (double)io_pred_alone);
            }
        } else {
            (void)hipGetLastError();
        }
    }
    if (wait_ms > 0 && c_pred_done > 0) {
        c_meas_done_ms = std::max(0.0, c_meas_done_ms - wait_ms);
        if (c_meas_done_ms > 0) scale_c = clamp_scale(c_meas_done_ms * 1e9 / (double)c_pred_done);
    }

    // ---- what came out
    const double lin = linear_flops_per_token_layer(m);
    const double pair_fl = 4.0 * m.n_q_heads * m.head_dim;
    const double qkv_fl = 2.0 * m.d_model * (double)(m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
    double fr = 0, fs = 0;
    int64_t rec_cells = 0, all_cells = 0;
    for (int i = 0; i < B; ++i) {
        cf_split& sp = splits_out[i];
        sp.mode = mode[i];
        all_cells += (int64_t)n_ctx[i] * L;
        if (mode[i] == CF_TOKEN_WISE) {
            sp.k_tokens = (int32_t)std::min<int64_t>((int64_t)p_comp[i] * C, n_ctx[i]);
            sp.layer_cut = L;
            double k = sp.k_tokens;
            rec_cells += (int64_t)sp.k_tokens * L;
            // chunk by chunk the same pairs as one pass over k tokens; the top layer is K/V only
            fr += (L - 1) * (k * lin + pair_fl * (k * (k + 1) / 2)) + k * qkv_fl;
        } else {
            sp.k_tokens = n_ctx[i];
            sp.layer_cut = p_comp[i];
            double t = n_ctx[i];
            rec_cells += (int64_t)n_ctx[i] * p_comp[i];
            if (p_comp[i] > 0) fr += (p_comp[i] - 1) * (t * lin + pair_fl * (t * (t + 1) / 2)) + t * qkv_fl;
        }
        if (logits_out) {
            double nn = reqs[i].n_new, p0 = n_ctx[i];
            fs += (double)L * (nn * lin + pair_fl * (nn * p0 + nn * (nn + 1) / 2));
        }
    }
    if (logits_out) fs += 2.0 * m.d_model * (double)m.vocab * B;
    if (timing) {
        float t_comp = 0, t_copy = 0, t_end = 0;
        CF_HIP(hipEventElapsedTime(&t_comp, c->ev_start, c->ev_comp));
        CF_HIP(hipEventElapsedTime(&t_copy, c->ev_start, c->ev_copy));
        CF_HIP(hipEventElapsedTime(&t_end, c->ev_start, c->ev_end));
        timing->compute_ms = t_comp;      // end of the last step that recomputed anything
        timing->copy_ms = t_copy;
        timing->restore_ms = std::max(t_comp, t_copy);
        timing->suffix_ms = t_end - timing->restore_ms;
        timing->total_ms = t_end;
        timing->compute_wait_ms = wait_ms;
        timing->recompute_flops = fr;
        timing->suffix_flops = fs;
        timing->loaded_bytes = loaded_bytes;
        timing->recomputed_cells = rec_cells;
        timing->loaded_cells = all_cells - rec_cells;
    }
    if (stats) {
        stats->compute_steps = n_steps;
        stats->compute_units = n_cunits;
        stats->io_units = (int32_t)io_issued;
        stats->scale_c_permille = scale_c;
        stats->scale_io_permille = scale_io;
        stats->scale_io_alone_permille = scale_io_alone;
        stats->compute_gap_ms = gap_ms;
        stats->planned_tail = tail_ran ? 1 : 0;
        stats->last_step_merged = merged_last ? 1 : 0;
    }
    // What the next call starts from.  A call's ratio depends on how much it claimed (the cost
    // model's error is not the same for every unit: a few more rows can cost the GEMMs a whole
    // extra round of tiles), and the claim on the ratio, so a ratio taken over whole flips
    // between a large and a small claim from call to call.  One unit too many on the compute
    // engine costs a multiple of what one too few does (a chunk takes several times longer to
    // recompute than to load), so its ratio follows a rise at once and a fall an eighth of the
    // way; the channel's ratios move halfway.
    if (c_pred_done > 0)
        c->dyn_scale_c = scale_c >= c->dyn_scale_c ? scale_c : c->dyn_scale_c - (c->dyn_scale_c - scale_c) / 8;
    if (io_pred_beside > 0) c->dyn_scale_io = (c->dyn_scale_io + scale_io + 1) / 2;
    if (io_pred_alone > 0) c->dyn_scale_io_alone = (c->dyn_scale_io_alone + scale_io_alone + 1) / 2;
    return CF_OK;
}

extern "C" int cf_offload(cf_ctx* c, cf_cache* cache, uint64_t req_id, int32_t n_ctx, void* host_kv) {
    if (!c || !cache || !host_kv || n_ctx < 0)
        return fail(CF_ERR_INVALID_ARG, "cf_offload: bad argument");
    int np = 0;
    const int32_t* pt = cache->table_of(req_id, &np);
    if (!cache->has(req_id)) return fail(CF_ERR_UNKNOWN_REQUEST, "cf_offload: request %llu has no pages",
                         (unsigned long long)req_id);
    int np_ctx = (int)ceil_div(n_ctx, CF_PAGE_TOKENS);
    if (np_ctx > np) return fail(CF_ERR_INVALID_ARG, "cf_offload: request holds fewer than n_ctx tokens");
    if (np_ctx == 0) return CF_OK;
    const cf_model_desc& m = c->m;
    size_t es = elem_bytes(m.dtype), pb = cache->page_bytes;
    KvGeom g;
    g.n_kv_heads = m.n_kv_heads;
    g.head_dim = m.head_dim;
    g.page_elems = (int64_t)(pb / es);
    g.layer_stride = g.page_elems * cache->n_pages;
    size_t cap_pages = c->cv.staging_bytes / pb;
    char* md = c->meta_dev();
    if ((size_t)np * 4 + sizeof(PageJob) + 64 > c->cv.meta_bytes)
        return fail(CF_ERR_WORKSPACE, "cf_offload: page table exceeds the context's metadata area");
    std::memcpy(c->meta_host, pt, (size_t)np * 4);
    size_t job_off = ((size_t)np * 4 + 15) / 16 * 16;
    // direct path: the host block is pinned, device-mapped memory -> one store kernel writes it
    // over the host link, all layers in one launch
    void* host_dev = nullptr;
    if (c->load_path != 1) {
        hipPointerAttribute_t at;
        if (hipPointerGetAttributes(&at, host_kv) != hipSuccess || at.type != hipMemoryTypeHost ||
            hipHostGetDevicePointer(&host_dev, host_kv, 0) != hipSuccess) {
            (void)hipGetLastError();
            host_dev = nullptr;
        }
        if (!host_dev && c->load_path == 2)
            return fail(CF_ERR_INVALID_ARG, "cf_offload: the direct path needs pinned, device-mapped host memory");
    }
    if (host_dev && (int64_t)np_ctx * (int64_t)(pb / 16) < ((int64_t)1 << 31) &&
        job_off + (size_t)m.n_layers * sizeof(PageJob) <= c->cv.meta_bytes) {
        PageJob* jobs = (PageJob*)(c->meta_host + job_off);
        int units_per_layer = (int)ceil_div((int64_t)np_ctx * (int64_t)(pb / 16), PAGE_LOAD_UNIT_VECS);
        for (int l = 0; l < m.n_layers; ++l)
            jobs[l] = PageJob{(int64_t)(uintptr_t)((char*)host_dev + (size_t)l * np_ctx * pb), l, 0, 0, np_ctx,
                              0, n_ctx, l * units_per_layer, 0};
        CF_HIP(hipMemcpyAsync(md, c->meta_host, job_off + (size_t)m.n_layers * sizeof(PageJob),
                              hipMemcpyHostToDevice, c->cs));
        launch_page_store(c->cs, m.dtype, cache->pool, (const PageJob*)(md + job_off), m.n_layers,
                          m.n_layers * units_per_layer, 2 * c->load_wgs, (const int32_t*)md, g);
        CF_HIP(hipGetLastError());
        CF_HIP(hipStreamSynchronize(c->cs));
        return CF_OK;
    }
    CF_HIP(hipMemcpy(md, c->meta_host, (size_t)np * 4, hipMemcpyHostToDevice));
    for (int l = 0; l < m.n_layers; ++l) {
        for (int j = 0; j < np_ctx; j += (int)cap_pages) {
            int take = (int)std::min<size_t>(cap_pages, (size_t)(np_ctx - j));
            PageJob jb{0, l, 0, j, take, 0, n_ctx, 0, 0};
            CF_HIP(hipMemcpy(md + job_off, &jb, sizeof(jb), hipMemcpyHostToDevice));
            launch_page_move(c->cs, m.dtype, c->staging(), cache->pool, (const PageJob*)(md + job_off),
                             1, take * PAGE_MOVE_SPLIT, (const int32_t*)md, g, false);
            CF_HIP(hipGetLastError());
            CF_HIP(hipStreamSynchronize(c->cs));
            CF_HIP(hipMemcpy((char*)host_kv + ((size_t)l * np_ctx + j) * pb, c->staging(),
                             (size_t)take * pb, hipMemcpyDeviceToHost));
        }
    }
    return CF_OK;
}


// ------------------------------------------------- offload for callers that cannot allocate
// cf_offload's staged path with its device scratch (page table, job record, staging slot) in a
// file-scope device array instead of the context's workspace.  Host code never uses the array's
// name as an address: the device address is looked up once per device with hipGetSymbolAddress
// (each GPU holds its own copy) and kept in g_static_scratch.
namespace {
constexpr size_t STATIC_META_BYTES = (size_t)64 << 10;       // page table + one job record
constexpr size_t STATIC_STAGING_BYTES = (size_t)16 << 20;    // one staging slot
constexpr int STATIC_MAX_DEVICES = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[STATIC_META_BYTES + STATIC_STAGING_BYTES];
static char* g_static_scratch[STATIC_MAX_DEVICES] = {};

// Device address of `scratch` on the current device (looked up on the first call per device).
static int static_scratch_of_current_device(char** out) {
    int dev = -1;
    CF_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= STATIC_MAX_DEVICES)
        return fail(CF_ERR_UNSUPPORTED, "static scratch: device index %d outside [0, %d)", dev, STATIC_MAX_DEVICES);
    if (!g_static_scratch[dev]) {
        void* p = nullptr;
        CF_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(CF_ERR_HIP, "static scratch: hipGetSymbolAddress returned a null address");
        g_static_scratch[dev] = (char*)p;
    }
    *out = g_static_scratch[dev];
    return CF_OK;
}

extern "C" size_t cf_offload_static_max_tokens(void) {
    return ((STATIC_META_BYTES - 256) / 4) * CF_PAGE_TOKENS;
}

extern "C" int cf_offload_static(cf_ctx* c, cf_cache* cache, uint64_t req_id, int32_t n_ctx, void* host_kv) {
    if (!c || !cache || !host_kv || n_ctx < 0)
        return fail(CF_ERR_INVALID_ARG, "cf_offload_static: bad argument");
    int np = 0;
    const int32_t* pt = cache->table_of(req_id, &np);
    if (!cache->has(req_id))
        return fail(CF_ERR_UNKNOWN_REQUEST, "cf_offload_static: request %llu has no pages", (unsigned long long)req_id);
    const int np_ctx = (int)ceil_div(n_ctx, CF_PAGE_TOKENS);
    if (np_ctx > np) return fail(CF_ERR_INVALID_ARG, "cf_offload_static: request holds fewer than n_ctx tokens");
    const cf_model_desc& m = c->m;
    const size_t es = elem_bytes(m.dtype), pb = cache->page_bytes;
    const size_t job_off = STATIC_META_BYTES - 256;          // the job record sits behind the page table
    if ((size_t)np_ctx * 4 > job_off)
        return fail(CF_ERR_WORKSPACE, "cf_offload_static: %d tokens exceed the static scratch's maximum of %zu "
                    "tokens per request", n_ctx, cf_offload_static_max_tokens());
    if (pb > STATIC_STAGING_BYTES || (size_t)np_ctx * 4 + sizeof(PageJob) + 64 > c->cv.meta_bytes)
        return fail(CF_ERR_WORKSPACE, "cf_offload_static: a page of %zu bytes exceeds the static staging slot of "
                    "%zu bytes, or the page table exceeds the context's pinned metadata buffer", pb,
                    STATIC_STAGING_BYTES);
    if (np_ctx == 0) return CF_OK;
    // the destination must be pinned: a copy into pageable memory goes through buffers the
    // runtime allocates
    {
        hipPointerAttribute_t at;
        if (hipPointerGetAttributes(&at, host_kv) != hipSuccess || at.type != hipMemoryTypeHost) {
            (void)hipGetLastError();
            return fail(CF_ERR_INVALID_ARG, "cf_offload_static: host_kv must be pinned host memory");
        }
    }
    char* sc = nullptr;
    int rc = static_scratch_of_current_device(&sc);
    if (rc) return rc;
    char* staging = sc + STATIC_META_BYTES;
    KvGeom g;
    g.n_kv_heads = m.n_kv_heads;
    g.head_dim = m.head_dim;
    g.page_elems = (int64_t)(pb / es);
    g.layer_stride = g.page_elems * cache->n_pages;
    const size_t cap_pages = STATIC_STAGING_BYTES / pb;
    // pinned mirror: page table at 0, the job record of the current piece behind it
    const size_t job_host = ((size_t)np_ctx * 4 + 15) / 16 * 16;
    std::memcpy(c->meta_host, pt, (size_t)np_ctx * 4);
    auto drain = [&](int code) { (void)hipStreamSynchronize(c->cs); (void)hipGetLastError(); return code; };
#define CF_HIP_D(call)                                                                        \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return drain(cf::fail(CF_ERR_HIP, "%s:%d %s -> %s", __FILE__, __LINE__, #call,    \
                                  hipGetErrorString(e_)));                                    \
    } while (0)
    CF_HIP_D(hipMemcpyAsync(sc, c->meta_host, (size_t)np_ctx * 4, hipMemcpyHostToDevice, c->cs));
    for (int l = 0; l < m.n_layers; ++l) {
        for (int j = 0; j < np_ctx; j += (int)cap_pages) {
            const int take = (int)std::min<size_t>(cap_pages, (size_t)(np_ctx - j));
            PageJob jb{0, l, 0, j, take, 0, n_ctx, 0, 0};
            std::memcpy(c->meta_host + job_host, &jb, sizeof(jb));
            CF_HIP_D(hipMemcpyAsync(sc + job_off, c->meta_host + job_host, sizeof(jb), hipMemcpyHostToDevice, c->cs));
            launch_page_move(c->cs, m.dtype, staging, cache->pool, (const PageJob*)(sc + job_off), 1,
                             take * PAGE_MOVE_SPLIT, (const int32_t*)sc, g, false);
            CF_HIP_D(hipGetLastError());
            CF_HIP_D(hipMemcpyAsync((char*)host_kv + ((size_t)l * np_ctx + j) * pb, staging, (size_t)take * pb,
                                    hipMemcpyDeviceToHost, c->cs));
            // the pinned job record and the staging slot are reused by the next piece
            CF_HIP_D(hipStreamSynchronize(c->cs));
        }
    }
#undef CF_HIP_D
    return CF_OK;
}

extern "C" int cf_measure_h2d(cf_ctx* c, const void* host_buf, void* dev_buf, size_t bytes,
                              int32_t reps, double* gb_per_s) {
    if (!c || !host_buf || !dev_buf || bytes == 0 || reps <= 0 || !gb_per_s)
        return fail(CF_ERR_INVALID_ARG, "cf_measure_h2d: bad argument");
    CF_HIP(hipMemcpyAsync(dev_buf, host_buf, bytes, hipMemcpyHostToDevice, c->ps));  // warm-up
    CF_HIP(hipEventRecord(c->ev_t0, c->ps));
    for (int i = 0; i < reps; ++i)
        CF_HIP(hipMemcpyAsync(dev_buf, host_buf, bytes, hipMemcpyHostToDevice, c->ps));
    CF_HIP(hipEventRecord(c->ev_t1, c->ps));
    CF_HIP(hipStreamSynchronize(c->ps));
    float ms = 0;
    CF_HIP(hipEventElapsedTime(&ms, c->ev_t0, c->ev_t1));
    *gb_per_s = (double)bytes * reps / (ms * 1e-3) / 1e9;
    return CF_OK;
}

extern "C" int cf_debug_force_gemm_tile(int32_t tile) {
    if (tile != 0 && tile != 64 && tile != 128 && tile != 256 && tile != 257)
        return fail(CF_ERR_INVALID_ARG, "cf_debug_force_gemm_tile: tile must be 0, 64, 128, 256 or 257");
    gemm_mfma_force_tile(tile);
    return CF_OK;
}

extern "C" int cf_op_gemm(cf_ctx* c, const void* A, const void* W, const void* W2, float* Cf,
                          void* Dt, int32_t M, int32_t N, int32_t K, int32_t epi, int32_t impl,
                          int32_t reps, float* avg_ms) {
    if (!c || !A || !W || M <= 0 || N <= 0 || K <= 0 || reps <= 0 || epi < 0 || epi > EPI_SILU_MUL)
        return fail(CF_ERR_INVALID_ARG, "cf_op_gemm: bad argument");
    if ((epi == EPI_SILU_MUL && !W2) || ((epi == EPI_STORE_F32 || epi == EPI_ADD_F32) && !Cf) ||
        ((epi == EPI_STORE_T || epi == EPI_SILU_MUL) && !Dt))
        return fail(CF_ERR_INVALID_ARG, "cf_op_gemm: missing operand for this epilogue");
    if (impl < 0 || impl > 6) return fail(CF_ERR_INVALID_ARG, "cf_op_gemm: impl must be 0..6");
    bool mfma_ok = gemm_mfma_supported(c->m.dtype, M, N, K, epi);
    if (impl >= 2 && !mfma_ok) return fail(CF_ERR_UNSUPPORTED, "cf_op_gemm: MFMA kernel does not take this problem");
    bool use_mfma = impl >= 2 || (impl == 0 && mfma_ok && !c->simple_only);
    gemm_mfma_force_tile(impl == 3 ? 256 : impl == 4 ? 128 : impl == 5 ? 64 : impl == 6 ? 257 : 0);
    struct Reset { ~Reset() { gemm_mfma_force_tile(0); } } reset_on_exit;
    CF_HIP(hipEventRecord(c->ev_t0, c->cs));
    for (int i = 0; i < reps; ++i) {
        if (use_mfma) launch_gemm_mfma(c->cs, A, W, W2, Cf, Dt, M, N, K, epi);
        else launch_gemm_simple(c->cs, c->m.dtype, A, W, W2, Cf, Dt, M, N, K, epi);
    }
    CF_HIP(hipEventRecord(c->ev_t1, c->cs));
    CF_HIP(hipGetLastError());
    CF_HIP(hipStreamSynchronize(c->cs));
    float ms = 0;
    CF_HIP(hipEventElapsedTime(&ms, c->ev_t0, c->ev_t1));
    if (avg_ms) *avg_ms = ms / reps;
    return CF_OK;
}

extern "C" int cf_ctx_profile(cf_ctx* c, uint32_t kernel_mask) {
    if (!c) return fail(CF_ERR_INVALID_ARG, "cf_ctx_profile: null ctx");
    c->prof_mask = kernel_mask & ((1u << CF_N_KERNELS) - 1);
    return CF_OK;
}

extern "C" int cf_ctx_profile_read(cf_ctx* c, cf_kernel_stat* out, int32_t reset) {
    if (!c || !out) return fail(CF_ERR_INVALID_ARG, "cf_ctx_profile_read: null argument");
    for (int i = 0; i < CF_N_KERNELS; ++i) {
        out[i] = c->prof_acc[i];
        out[i].kernel = i;
        if (reset) c->prof_acc[i] = cf_kernel_stat{};
    }
    return CF_OK;
}

// ------------------------------------------------------------------ calibration
// Times a few recompute passes and host->device loads through cf_restore_batch
// itself and fits the integer cost model by solving the small linear systems
// exactly, then quantises to picoseconds.
extern "C" int cf_calibrate(cf_ctx* c, cf_cache* cache, void* host_buf, size_t host_bytes,
                            cf_cost_model* out) {
    if (!c || !cache || !host_buf || !out) return fail(CF_ERR_INVALID_ARG, "cf_calibrate: null argument");
    const cf_model_desc& m = c->m;
    if (c->stage_begin != 0 || c->stage_end != m.n_layers)
        return fail(CF_ERR_INVALID_ARG, "cf_calibrate: calibrate on the whole model (the per-layer costs "
                    "it measures hold for any stage)");
    const int L = m.n_layers;
    // probe sizes: bounded by the context limits
    int t_big = std::min(std::min(c->opts.max_tokens, c->opts.max_positions), 8192);
    t_big = t_big / 512 * 512;
    if (t_big < 1024) return fail(CF_ERR_WORKSPACE, "cf_calibrate: context too small (needs >= 1024 tokens)");
    int t_small = 512;
    int n_split = std::min(8, c->opts.max_batch);          // t_big tokens as n_split short requests
    int t_part = t_big / n_split / 16 * 16;
    size_t need_host = cf_host_kv_bytes(L, m.n_kv_heads, m.head_dim, m.dtype, t_big);
    if (host_bytes < need_host)
        return fail(CF_ERR_WORKSPACE, "cf_calibrate: host scratch %zu < %zu", host_bytes, need_host);
    std::vector<int32_t> toks(t_big);
    for (int i = 0; i < t_big; ++i) toks[i] = (int32_t)(((int64_t)i * 7919 + 13) % m.vocab);
    const uint64_t base_id = 0xCA11B000ull;
    struct Probe { int n_req, n_tok, k; };      // k = tokens recomputed per request (0 = load all)
    auto run = [&](const Probe& p, cf_timing* tm) -> int {
        std::vector<cf_request> rq(p.n_req);
        std::vector<cf_split> sp(p.n_req);
        int rc = CF_OK;
        int made = 0;
        for (int i = 0; i < p.n_req && rc == CF_OK; ++i) {
            rc = cf_cache_alloc(cache, base_id + i, p.n_tok);
            if (rc == CF_OK) ++made;
            rq[i] = cf_request{base_id + i, toks.data(), p.n_tok, 0, host_buf, nullptr, nullptr};
            sp[i] = cf_split{CF_TOKEN_WISE, p.k, L};
        }
        if (rc == CF_OK) rc = cf_restore_batch(c, cache, p.n_req, rq.data(), sp.data(), nullptr, tm);  // warm-up
        // the faster of two timed runs: a one-off stall (clock ramp, a first transfer) would
        // otherwise end up in a coefficient
        cf_timing t2;
        if (rc == CF_OK) rc = cf_restore_batch(c, cache, p.n_req, rq.data(), sp.data(), nullptr, tm);
        if (rc == CF_OK) rc = cf_restore_batch(c, cache, p.n_req, rq.data(), sp.data(), nullptr, &t2);
        if (rc == CF_OK && (p.k > 0 ? t2.compute_ms < tm->compute_ms : t2.copy_ms < tm->copy_ms)) *tm = t2;
        for (int i = 0; i < made; ++i) cf_cache_free(cache, base_id + i);
        return rc;
    };
    cf_timing tm;
    double y[3], T[3], P[3];
    // recompute is batched over requests, so the probes are batch-shaped: the intercept of the
    // fit is a per-layer-pass floor paid once per batch (-> s_c), not once per chunk
    Probe probes[3] = {{n_split, t_small, t_small}, {n_split, t_part, t_part}, {1, t_big, t_big}};
    for (int i = 0; i < 3; ++i) {
        int rc = run(probes[i], &tm);
        if (rc) return rc;
        y[i] = (double)tm.compute_ms * 1e9 / L;                 // ps per layer
        T[i] = (double)probes[i].n_req * probes[i].n_tok;
        double n = probes[i].n_tok;
        P[i] = probes[i].n_req * (n * (n + 1) / 2) / 1024.0;
    }
    // y = f + a*T + b*P, three equations: eliminate f, then solve the 2x2 system
    double a11 = T[1] - T[0], a12 = P[1] - P[0], b1 = y[1] - y[0];
    double a21 = T[2] - T[0], a22 = P[2] - P[0], b2 = y[2] - y[0];
    double det = a11 * a22 - a12 * a21;
    double alpha = 0, beta = 0;
    if (std::fabs(det) > 1e-9) {
        alpha = (b1 * a22 - a12 * b2) / det;
        beta = (a11 * b2 - b1 * a21) / det;
    }
    if (alpha <= 0 || beta < 0) {      // degenerate fit: fall back to a pure per-token rate
        beta = 0;
        alpha = y[2] / T[2];
    }
    double floor_c = std::max(0.0, y[0] - alpha * T[0] - beta * P[0]);
    // I/O: one large and one small all-load; the intercept is the channel's start-up
    Probe io_big{1, t_big, 0}, io_small{1, t_small, 0};
    int rc = run(io_big, &tm);
    if (rc) return rc;
    double t_big_ps = (double)tm.copy_ms * 1e9, mib_big = (double)tm.loaded_bytes / 1048576.0;
    rc = run(io_small, &tm);
    if (rc) return rc;
    double t_small_ps = (double)tm.copy_ms * 1e9, mib_small = (double)tm.loaded_bytes / 1048576.0;
    double gamma = (t_big_ps - t_small_ps) / std::max(mib_big - mib_small, 1e-9);
    if (gamma <= 0) gamma = t_big_ps / std::max(mib_big, 1e-9);
    double start_io = std::max(0.0, t_small_ps - gamma * mib_small);
    out->f_c = 0;
    out->alpha = std::max<int64_t>(1, (int64_t)std::llround(alpha));
    out->beta = (int64_t)std::llround(beta);
    out->f_io = 0;
    out->gamma = std::max<int64_t>(1, (int64_t)std::llround(gamma));
    out->s_c = (int64_t)std::llround(floor_c * L);
    out->s_io = (int64_t)std::llround(start_io);
    return CF_OK;
}

// One overlapped probe: request A (t tokens) is recomputed in full while request B (t tokens) is
// loaded in full; each engine's time is compared with what the cost model predicts for it alone.
extern "C" int cf_calibrate_overlap(cf_ctx* c, cf_cache* cache, void* host_buf, size_t host_bytes,
                                    const cf_cost_model* cost, cf_overlap_model* out) {
    if (!c || !cache || !host_buf || !cost || !out)
        return fail(CF_ERR_INVALID_ARG, "cf_calibrate_overlap: null argument");
    const cf_model_desc& m = c->m;
    if (c->stage_begin != 0 || c->stage_end != m.n_layers)
        return fail(CF_ERR_INVALID_ARG, "cf_calibrate_overlap: calibrate on the whole model");
    const int L = m.n_layers;
    int t = std::min(std::min(c->opts.max_tokens, c->opts.max_positions), 8192) / 512 * 512;
    if (t < 1024) return fail(CF_ERR_WORKSPACE, "cf_calibrate_overlap: context too small (needs >= 1024 tokens)");
    if (c->opts.max_batch < 2) return fail(CF_ERR_WORKSPACE, "cf_calibrate_overlap: needs max_batch >= 2");
    const size_t need_host = cf_host_kv_bytes(L, m.n_kv_heads, m.head_dim, m.dtype, t);
    if (host_bytes < need_host)
        return fail(CF_ERR_WORKSPACE, "cf_calibrate_overlap: host scratch %zu < %zu", host_bytes, need_host);
    std::vector<int32_t> toks(t);
    for (int i = 0; i < t; ++i) toks[i] = (int32_t)(((int64_t)i * 7919 + 13) % m.vocab);
    const uint64_t id_a = 0xCA11B100ull, id_b = 0xCA11B101ull;
    int rc = cf_cache_alloc(cache, id_a, t);
    if (rc) return rc;
    rc = cf_cache_alloc(cache, id_b, t);
    if (rc) { cf_cache_free(cache, id_a); return rc; }
    cf_request rq[2] = {cf_request{id_a, toks.data(), t, 0, nullptr, nullptr, nullptr},
                        cf_request{id_b, toks.data(), t, 0, host_buf, nullptr, nullptr}};
    cf_split sp[2] = {cf_split{CF_TOKEN_WISE, t, L}, cf_split{CF_TOKEN_WISE, 0, L}};
    cf_timing tm;
    rc = cf_restore_batch(c, cache, 2, rq, sp, nullptr, &tm);                 // warm-up
    if (rc == CF_OK) rc = cf_restore_batch(c, cache, 2, rq, sp, nullptr, &tm);
    cf_cache_free(cache, id_a);
    cf_cache_free(cache, id_b);
    if (rc) return rc;
    // predictions for each engine alone (the executor stops the top layer after its K/V write,
    // which the planner prices separately; this probe's figure is rough either way)
    const double pairs = (double)t * ((double)t + 1) / 2 / 1024.0;
    const double pred_c = (double)cost->s_c + (double)L * ((double)cost->f_c + (double)cost->alpha * t + (double)cost->beta * pairs);
    const double pred_io = (double)cost->s_io + (double)cost->f_io * L + (double)cost->gamma * ((double)tm.loaded_bytes / 1048576.0);
    const double meas_c = (double)tm.compute_ms * 1e9, meas_io = (double)tm.copy_ms * 1e9;
    double f_io = pred_io > 0 ? meas_io / pred_io : 1.0;
    // the compute stream is slowed only while the load runs beside it
    double f_c = (meas_io > 0 && pred_c > 0) ? 1.0 + (meas_c - pred_c) / meas_io : 1.0;
    auto clampf = [](double v) { return std::min(2.0, std::max(1.0, v)); };
    out->comp_permille = (int32_t)std::llround(1000.0 * clampf(f_c));
    out->io_permille = (int32_t)std::llround(1000.0 * clampf(f_io));
    return CF_OK;
}

extern "C" int cf_read_final_hidden(cf_ctx* c, int32_t B, float* out_host) {
    if (!c || !out_host || B <= 0) return fail(CF_ERR_INVALID_ARG, "cf_read_final_hidden: bad argument");
    if (c->n_last != B)
        return fail(CF_ERR_INVALID_ARG, "cf_read_final_hidden: the last restore call produced logits for %d requests",
                    c->n_last);
    CF_HIP(hipMemcpy(out_host, c->h_last(), (size_t)B * c->m.d_model * sizeof(float), hipMemcpyDeviceToHost));
    return CF_OK;
}
