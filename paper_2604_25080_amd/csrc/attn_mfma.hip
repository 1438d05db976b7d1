// Varlen causal attention over the paged KV cache on CDNA4 matrix cores
// (bf16 operands, float softmax and accumulation), grouped-query heads.
//
// grid = (attention work items, Q heads).  A work item is up to 128 packed
// query rows of one request whose first row sits at absolute position pos0;
// the query at position p attends to keys 0..p, read from the request's pages.
// A long key range may be split over several work items (tile_begin/tile_end);
// those write un-normalised partial results that a small combine kernel merges.
// Each of the 4 wavefronts owns 32 query rows.  Keys are walked in tiles of 64
// (4 pages).  The K tile [64 keys][hd] and the transposed V tile [hd][64 keys]
// (V is stored transposed inside a page) are staged in LDS, double-buffered;
// tile t+2 is fetched into registers while tile t is consumed, and the page ids
// of tile t+3 are fetched (scalar) at the same time, so neither the page-table
// lookup nor the memory latency sits on the critical path.
//
// The scores are computed transposed, S^T = K Q^T, so that in the MFMA result
// layout every lane holds 16 keys of ONE query row: the softmax row statistics
// stay in the lane (one exchange with the lane 32 apart), and the exponentiated
// scores are already in the register layout the second product,
// O^T = V^T P^T, needs for its B operand -- P never goes through LDS.
// The running output is rescaled only when some row's maximum actually moved.
#include "kernels.h"
#include "cacheflow.h"

namespace cf {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;

namespace {

constexpr int KT = 64;                      // keys per tile
constexpr int PAGES_PER_TILE = KT / CF_PAGE_TOKENS;

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// HPB = query heads per workgroup (1 or 2): with 2, wavefronts 0-3 and 4-7 work on two heads of
// the same KV group and share every K/V tile in LDS, which halves the L2 -> LDS traffic per
// FLOP (what bounds this kernel); 8 wavefronts per CU either way.
template <int HD, int HPB>
__global__ void __launch_bounds__(256 * HPB, 3 - HPB)
attention_mfma_kernel(const bf16* __restrict__ q, bf16* __restrict__ out, float* __restrict__ part_buf,
                      const bf16* __restrict__ pool_layer, const AttnWork* __restrict__ work,
                      const int32_t* __restrict__ page_tables, int n_q_heads, KvGeom g) {
    constexpr int K_ROWB = HD * 2;                 // bytes per key row of the K tile
    constexpr int K_NCH = HD / 8;                  // 16-byte chunks per key row
    constexpr int K_TILE = KT * K_ROWB;
    constexpr int V_ROWB = KT * 2;                 // bytes per hd row of the V^T tile (128)
    constexpr int V_TILE = HD * V_ROWB;
    constexpr int STAGE = K_TILE + V_TILE;
    constexpr int VEC_PER_PAGE = CF_PAGE_TOKENS * K_NCH;       // 16-byte vectors of one page's K (= V) part
    constexpr int NT = 256 * HPB;
    constexpr int PAGES_PER_LOAD = NT / VEC_PER_PAGE;          // pages covered by one block-wide load (1, 2 or 4)
    static_assert(PAGES_PER_LOAD >= 1 && PAGES_PER_LOAD <= PAGES_PER_TILE, "loader shape");
    constexpr int NLD = PAGES_PER_TILE / PAGES_PER_LOAD;       // loads per thread per tile, each of K and V
    constexpr int QK_STEPS = HD / 16;
    constexpr int D_TILES = HD / 32;
    __shared__ __align__(16) char smem[2 * STAGE];

    // Workgroup ids are item-major and walk the work list backwards: the host lists the items of
    // a launch lightest first (new-turn items: sorted by key tiles; recompute items: in row
    // order, a request's later rows see more keys), and all head blocks of an item are dispatched
    // before the next item's, so the launch ends with its lightest items on every head instead
    // of a few long ones running alone.  Consecutive workgroups go to different
    // XCDs, eight apart to the same one: the head blocks of an item are numbered so that those
    // that share a KV head (and its K/V tiles in L2) are a multiple of the KV-head count apart.
    const int n_blocks_h = n_q_heads / HPB;                          // head blocks per item
    const int per_kv = (n_q_heads / g.n_kv_heads) / HPB;             // ... of which share a KV head
    const int n_kv_b = n_blocks_h / per_kv;
    const int item = blockIdx.x / n_blocks_h, hb = blockIdx.x % n_blocks_h;
    AttnWork w = work[gridDim.x / n_blocks_h - 1 - item];
    int tid = threadIdx.x, lane = tid & 63;
    int wave = (tid >> 6) & 3;                     // which 32 query rows
    // wavefronts 4-7 take the second head of the pair
    int head = ((hb % n_kv_b) * per_kv + hb / n_kv_b) * HPB + (tid >> 8);
    int gk = head / (n_q_heads / g.n_kv_heads);    // the same KV head for both (group size is even)
    const int32_t* pt = page_tables + w.pt_off;
    int lq = lane & 31, lh = lane >> 5;

    int kv_end = min(w.pos0 + w.n_rows, w.tile_end * KT);   // keys [tile_begin*KT, kv_end) are read
    int last_page = (kv_end - 1) / CF_PAGE_TOKENS;
    int row = min(wave * 32 + lq, w.n_rows - 1);   // padded rows repeat the last row
    int qpos = w.pos0 + row;
    int wave_last_q = w.pos0 + min(wave * 32 + 31, w.n_rows - 1);   // wave-uniform
    int wave_first_q = w.pos0 + min(wave * 32, w.n_rows - 1);

    // ---- Q fragments: B operand of S^T = K Q^T, lane = query row lq, 8 hd values per step
    u32x4_t qf[QK_STEPS];
    {
        const bf16* qrow = q + ((int64_t)(w.row0 + row) * n_q_heads + head) * HD;
#pragma unroll
        for (int kk = 0; kk < QK_STEPS; ++kk)
            qf[kk] = *reinterpret_cast<const u32x4_t*>(qrow + kk * 16 + lh * 8);
    }

    // ---- tile loader: block-wide load j covers page(s) j*PAGES_PER_LOAD.. of the tile.
    // Within a page, thread slot v handles K vector (row v / K_NCH, chunk v % K_NCH) and
    // V^T vector (hd row v / 2, half v % 2).
    const int64_t k_head_off = (int64_t)gk * CF_PAGE_TOKENS * HD;
    const int64_t v_head_off = (int64_t)g.n_kv_heads * CF_PAGE_TOKENS * HD + (int64_t)gk * HD * CF_PAGE_TOKENS;
    int sub_page = tid / VEC_PER_PAGE;             // which page of the load (wave-uniform)
    int pv = tid % VEC_PER_PAGE;
    int k_r = pv / K_NCH, k_c = pv % K_NCH;        // key row within page, chunk
    int v_d = pv / 2, v_half = pv % 2;             // hd row, which 8 keys of the page
    int k_goff = k_r * HD + k_c * 8;
    int v_goff = v_d * CF_PAGE_TOKENS + v_half * 8;
    int k_lds[NLD], v_lds0[NLD], v_lds1[NLD], v_key0[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        int page_in_tile = j * PAGES_PER_LOAD + sub_page;
        int r = page_in_tile * CF_PAGE_TOKENS + k_r;
        int ksw = (HD == 128) ? (r & 15) : ((r >> 1) & 7);
        k_lds[j] = r * K_ROWB + ((k_c ^ ksw) << 4);
        // V^T row v_d, page p: chunk 2p+h holds [keys 4h..4h+3 | keys 8+4h..8+4h+3] of the page,
        // i.e. exactly the 16 bytes lane half h of the second product needs (one 16-byte read).
        // This thread's vector (keys 8*v_half .. +7) therefore goes out as two 8-byte pieces:
        // keys +0..3 into chunk 2p, keys +4..7 into chunk 2p+1, both at half v_half.
        int vsw = (v_d >> 1) & 7;
        v_lds0[j] = K_TILE + v_d * V_ROWB + (((page_in_tile * 2) ^ vsw) << 4) + v_half * 8;
        v_lds1[j] = K_TILE + v_d * V_ROWB + (((page_in_tile * 2 + 1) ^ vsw) << 4) + v_half * 8;
        v_key0[j] = page_in_tile * CF_PAGE_TOKENS + v_half * 8;
    }

    // page ids of one tile, wave-uniform (clamped to the last page that is needed)
    int pg[NLD];
#define CF_PAGES(TILE)                                                                        \
    {                                                                                         \
        int p0_ = (TILE) * PAGES_PER_TILE;                                                    \
        _Pragma("unroll") for (int j = 0; j < NLD; ++j) {                                     \
            int idx_ = __builtin_amdgcn_readfirstlane(min(p0_ + j * PAGES_PER_LOAD + sub_page, last_page)); \
            pg[j] = pt[idx_];                                                                 \
        }                                                                                     \
    }
    u32x4_t rk[NLD], rv[NLD];
    // Global -> registers for one tile (page ids already in pg).  Slots past the last needed
    // key may hold anything (even NaN patterns): they are zeroed so that their zero
    // probabilities cannot poison the second product.
#define CF_FETCH(TILE)                                                                        \
    {                                                                                         \
        int tile_ = (TILE);                                                                   \
        _Pragma("unroll") for (int j = 0; j < NLD; ++j) {                                     \
            const bf16* page_ = pool_layer + (int64_t)pg[j] * g.page_elems;                   \
            rk[j] = *reinterpret_cast<const u32x4_t*>(page_ + k_head_off + k_goff);           \
            u32x4_t val = *reinterpret_cast<const u32x4_t*>(page_ + v_head_off + v_goff);     \
            int left = kv_end - (tile_ * KT + v_key0[j]);   /* valid keys in this vector */   \
            if (left < 8) {                                                                   \
                val.x = left <= 0 ? 0u : (left == 1 ? val.x & 0xFFFFu : val.x);               \
                val.y = left <= 2 ? 0u : (left == 3 ? val.y & 0xFFFFu : val.y);               \
                val.z = left <= 4 ? 0u : (left == 5 ? val.z & 0xFFFFu : val.z);               \
                val.w = left <= 6 ? 0u : (left == 7 ? val.w & 0xFFFFu : val.w);               \
            }                                                                                 \
            rv[j] = val;                                                                      \
        }                                                                                     \
    }
#define CF_STASH(STAGE_PTR)                                                                   \
    {                                                                                         \
        char* st_ = (STAGE_PTR);                                                              \
        _Pragma("unroll") for (int j = 0; j < NLD; ++j) {                                     \
            *reinterpret_cast<u32x4_t*>(st_ + k_lds[j]) = rk[j];                              \
            *reinterpret_cast<u32x2_t*>(st_ + v_lds0[j]) = u32x2_t{rv[j].x, rv[j].y};         \
            *reinterpret_cast<u32x2_t*>(st_ + v_lds1[j]) = u32x2_t{rv[j].z, rv[j].w};         \
        }                                                                                     \
    }

    f32x16_t o_acc[D_TILES];
#pragma unroll
    for (int t = 0; t < D_TILES; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[t][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;          // running max (log2 domain), partial row sum
    const float scale_log2e = rsqrtf((float)HD) * 1.4426950408889634f;

    // fragment read offsets
    int ksw_l = (HD == 128) ? (lq & 15) : ((lq >> 1) & 7);
    int vsw_l = (lq >> 1) & 7;

    int t0 = w.tile_begin, t1 = w.tile_end;        // tiles [t0, t1), t1 > t0
    CF_PAGES(t0);
    CF_FETCH(t0);
    CF_PAGES(min(t0 + 1, t1 - 1));
    CF_STASH(smem);
    CF_FETCH(min(t0 + 1, t1 - 1));
    CF_PAGES(min(t0 + 2, t1 - 1));
    __syncthreads();

    for (int tile = t0; tile < t1; ++tile) {
        char* cur = smem + ((tile - t0) & 1) * STAGE;
        char* nxt = smem + ((tile - t0 + 1) & 1) * STAGE;
        int key_base = tile * KT;
        if (key_base <= wave_last_q) {               // wave-uniform: tile not fully masked
            // ---- S^T = K Q^T : two 32-key fragments
            f32x16_t s[2];
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
                for (int kk = 0; kk < QK_STEPS; ++kk) {
                    u32x4_t kf = *reinterpret_cast<const u32x4_t*>(
                        cur + (tt * 32 + lq) * K_ROWB + (((2 * kk + lh) ^ ksw_l) << 4));
                    // the first step starts from a zero accumulator operand (no register clearing)
                    s[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8_t, kf), __builtin_bit_cast(bf16x8_t, qf[kk]),
                        kk == 0 ? f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}
                                : s[tt], 0, 0, 0);
                }
            }
            // ---- causal mask on the diagonal tiles only (lane = one query row, 32 of its 64 keys)
            if (key_base + KT - 1 > wave_first_q) {
#pragma unroll
                for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int kpos = key_base + tt * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                        s[tt][r] = (kpos > qpos) ? -INFINITY : s[tt][r];
                    }
            }
            // ---- online softmax in the log2 domain: p = 2^(s*scale - m)
            float tmax = s[0][0];
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[tt][r]);
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            float m_new = fmaxf(m_run, tmax * scale_log2e);   // finite: a visible key exists
            if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {   // some row's maximum moved
                float corr = __builtin_amdgcn_exp2f(m_run - m_new);
                l_run *= corr;
#pragma unroll
                for (int t = 0; t < D_TILES; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o_acc[t][r] *= corr;
                m_run = m_new;
            }
            float psum = 0.f;
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[tt][r], scale_log2e, -m_run));
                    s[tt][r] = p;
                    psum += p;
                }
            l_run += psum;
            // ---- O^T += V^T P^T : 4 steps of 16 keys (one page each)
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                int tt = st >> 1, b0 = (st & 1) * 2;
                u32x4_t pf;
                pf.x = pack_bf16x2(s[tt][4 * b0 + 0], s[tt][4 * b0 + 1]);
                pf.y = pack_bf16x2(s[tt][4 * b0 + 2], s[tt][4 * b0 + 3]);
                pf.z = pack_bf16x2(s[tt][4 * b0 + 4], s[tt][4 * b0 + 5]);
                pf.w = pack_bf16x2(s[tt][4 * b0 + 6], s[tt][4 * b0 + 7]);
#pragma unroll
                for (int t = 0; t < D_TILES; ++t) {
                    // keys 4*lh..4*lh+3 and 8+4*lh.. of page `st`, for hd row 32t + lq: one chunk
                    u32x4_t vf = *reinterpret_cast<const u32x4_t*>(
                        cur + K_TILE + (t * 32 + lq) * V_ROWB + (((2 * st + lh) ^ vsw_l) << 4));
                    o_acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8_t, vf), __builtin_bit_cast(bf16x8_t, pf), o_acc[t], 0, 0, 0);
                }
            }
        }
        CF_STASH(nxt);                               // tile+1, fetched during the previous iteration
        CF_FETCH(min(tile + 2, t1 - 1));             // consumed two iterations from now
        CF_PAGES(min(tile + 3, t1 - 1));
        __syncthreads();
    }
#undef CF_PAGES
#undef CF_FETCH
#undef CF_STASH

    // ---- store: lane holds hd = 32t + 8b + 4*lh + i of query row lq
    float l_tot = l_run + __shfl_xor(l_run, 32);
    if (wave * 32 + lq >= w.n_rows) return;
    if (w.part < 0) {
        float inv = 1.0f / l_tot;
        bf16* orow = out + ((int64_t)(w.row0 + wave * 32 + lq) * n_q_heads + head) * HD;
#pragma unroll
        for (int t = 0; t < D_TILES; ++t)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                u32x2_t val;
                val.x = pack_bf16x2(o_acc[t][4 * b + 0] * inv, o_acc[t][4 * b + 1] * inv);
                val.y = pack_bf16x2(o_acc[t][4 * b + 2] * inv, o_acc[t][4 * b + 3] * inv);
                *reinterpret_cast<u32x2_t*>(orow + t * 32 + 8 * b + 4 * lh) = val;
            }
    } else {
        // partial result of one key range: [part][head][row] -> (o[HD], m, l, pad, pad) in float
        float* prow = part_buf + (((int64_t)w.part * n_q_heads + head) * ATTN_BLOCK_ROWS + wave * 32 + lq) * (HD + 4);
        if (lh == 0) { prow[HD] = m_run; prow[HD + 1] = l_tot; }
#pragma unroll
        for (int t = 0; t < D_TILES; ++t)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                float4 val = make_float4(o_acc[t][4 * b + 0], o_acc[t][4 * b + 1], o_acc[t][4 * b + 2], o_acc[t][4 * b + 3]);
                *reinterpret_cast<float4*>(prow + t * 32 + 8 * b + 4 * lh) = val;
            }
    }
}

// Merge the partial results of one (q-block, head): one wavefront per query row, four rows
// per workgroup (blockIdx.z picks the row quad), so the merge is spread over thousands of
// wavefronts instead of walking 32 rows per wavefront through dependent loads.
template <int HD>
__global__ void __launch_bounds__(256)
attention_combine_kernel(bf16* __restrict__ out, const float* __restrict__ part_buf,
                         const AttnCombine* __restrict__ groups, int n_q_heads) {
    AttnCombine cgrp = groups[blockIdx.x];
    int head = blockIdx.y;
    int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    {
        int r = blockIdx.z * 4 + wave;
        if (r >= cgrp.n_rows) return;
        float m = -INFINITY;
        for (int p = 0; p < cgrp.n_parts; ++p) {
            const float* prow = part_buf + (((int64_t)(cgrp.part_first + p) * n_q_heads + head) * ATTN_BLOCK_ROWS + r) * (HD + 4);
            m = fmaxf(m, prow[HD]);
        }
        float l = 0.f, acc[HD / 64];
#pragma unroll
        for (int i = 0; i < HD / 64; ++i) acc[i] = 0.f;
        for (int p = 0; p < cgrp.n_parts; ++p) {
            const float* prow = part_buf + (((int64_t)(cgrp.part_first + p) * n_q_heads + head) * ATTN_BLOCK_ROWS + r) * (HD + 4);
            float f = __builtin_amdgcn_exp2f(prow[HD] - m);
            l += prow[HD + 1] * f;
#pragma unroll
            for (int i = 0; i < HD / 64; ++i) acc[i] += prow[lane + 64 * i] * f;
        }
        bf16* orow = out + ((int64_t)(cgrp.row0 + r) * n_q_heads + head) * HD;
        float inv = 1.0f / l;
#pragma unroll
        for (int i = 0; i < HD / 64; ++i) {
            float v = acc[i] * inv;
            orow[lane + 64 * i].x = (uint16_t)(pack_bf16x2(v, 0.f) & 0xFFFFu);
        }
    }
}

}  // namespace

int attention_mfma_heads_per_block(int n_q_heads, int n_kv_heads) {
    return (n_q_heads / n_kv_heads) % 2 == 0 ? 2 : 1;
}

bool attention_mfma_supported(int dtype, int head_dim, int n_q_heads, int n_kv_heads) {
    return dtype == CF_BF16 && (head_dim == 64 || head_dim == 128) && n_q_heads % n_kv_heads == 0;
}

void launch_attention_mfma(hipStream_t s, const void* q, void* out, float* part_buf,
                           const void* pool_layer, const AttnWork* work, int n_work,
                           const AttnCombine* groups, int n_groups, const int32_t* page_tables,
                           int n_q_heads, KvGeom g) {
    if (n_work <= 0) return;
    const bool pair = attention_mfma_heads_per_block(n_q_heads, g.n_kv_heads) == 2;
    dim3 grid((unsigned)n_work * (pair ? n_q_heads / 2 : n_q_heads));
    if (g.head_dim == 128 && pair)
        attention_mfma_kernel<128, 2><<<grid, 512, 0, s>>>((const bf16*)q, (bf16*)out, part_buf, (const bf16*)pool_layer, work, page_tables, n_q_heads, g);
    else if (g.head_dim == 128)
        attention_mfma_kernel<128, 1><<<grid, 256, 0, s>>>((const bf16*)q, (bf16*)out, part_buf, (const bf16*)pool_layer, work, page_tables, n_q_heads, g);
    else if (pair)
        attention_mfma_kernel<64, 2><<<grid, 512, 0, s>>>((const bf16*)q, (bf16*)out, part_buf, (const bf16*)pool_layer, work, page_tables, n_q_heads, g);
    else
        attention_mfma_kernel<64, 1><<<grid, 256, 0, s>>>((const bf16*)q, (bf16*)out, part_buf, (const bf16*)pool_layer, work, page_tables, n_q_heads, g);
    if (n_groups > 0) {
        dim3 cgrid(n_groups, n_q_heads, ATTN_BLOCK_ROWS / 4);
        if (g.head_dim == 128)
            attention_combine_kernel<128><<<cgrid, 256, 0, s>>>((bf16*)out, part_buf, groups, n_q_heads);
        else
            attention_combine_kernel<64><<<cgrid, 256, 0, s>>>((bf16*)out, part_buf, groups, n_q_heads);
    }
}

}  // namespace cf
