// Varlen causal attention over the paged KV cache on CDNA4 matrix cores
// (bf16 operands, float softmax and accumulation), grouped-query heads.
//
// grid = (attention work items, Q heads).  A work item is up to 128 packed
// query rows of one request whose first row sits at absolute position pos0;
// the query at position p attends to keys 0..p, read from the request's pages.
// Each of the 4 wavefronts owns 32 query rows.  Keys are walked in tiles of 64
// (4 pages).  The K tile [64 keys][hd] and the transposed V tile [hd][64 keys]
// (V is stored transposed inside a page) are staged in LDS, double-buffered,
// with the next tile prefetched into registers during the current one.
//
// The scores are computed transposed, S^T = K Q^T, so that in the MFMA result
// layout every lane holds 16 keys of ONE query row: the softmax row statistics
// stay in the lane (one exchange with the lane 32 apart), and the exponentiated
// scores are already in the register layout the second product,
// O^T = V^T P^T, needs for its B operand -- P never goes through LDS.
#include "kernels.h"
#include "cacheflow.h"

namespace cf {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

namespace {

constexpr int KT = 64;                      // keys per tile

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
    ua += 0x7FFFu + ((ua >> 16) & 1u);
    ub += 0x7FFFu + ((ub >> 16) & 1u);
    return (ua >> 16) | (ub & 0xFFFF0000u);
}

template <int HD>
__global__ void __launch_bounds__(256)
attention_mfma_kernel(const bf16* __restrict__ q, bf16* __restrict__ out,
                      const bf16* __restrict__ pool_layer, const AttnWork* __restrict__ work,
                      const int32_t* __restrict__ page_tables, int n_q_heads, KvGeom g) {
    constexpr int K_ROWB = HD * 2;                 // bytes per key row of the K tile
    constexpr int K_NCH = HD / 8;                  // 16-byte chunks per key row
    constexpr int K_TILE = KT * K_ROWB;
    constexpr int V_ROWB = KT * 2;                 // bytes per hd row of the V^T tile (128)
    constexpr int V_TILE = HD * V_ROWB;
    constexpr int STAGE = K_TILE + V_TILE;
    constexpr int NLD = KT * K_NCH / 256;          // 16-byte loads per thread per tile, each of K and V
    constexpr int QK_STEPS = HD / 16;
    constexpr int D_TILES = HD / 32;
    __shared__ __align__(16) char smem[2 * STAGE];

    // heaviest work items (largest positions) are scheduled first
    AttnWork w = work[gridDim.x - 1 - blockIdx.x];
    int head = blockIdx.y;
    int gk = head / (n_q_heads / g.n_kv_heads);
    const int32_t* pt = page_tables + w.pt_off;
    int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int lq = lane & 31, lh = lane >> 5;

    int kv_end = w.pos0 + w.n_rows;                // keys [0, kv_end) are needed by this block
    int n_tiles = (kv_end + KT - 1) / KT;
    int last_page = (kv_end - 1) / CF_PAGE_TOKENS;
    int row = min(wave * 32 + lq, w.n_rows - 1);   // padded rows repeat the last row
    int qpos = w.pos0 + row;
    int wave_last_q = w.pos0 + min(wave * 32 + 31, w.n_rows - 1);   // wave-uniform
    int wave_first_q = w.pos0 + min(wave * 32, w.n_rows - 1);

    // ---- Q fragments: B operand of S^T = K Q^T, lane = query row lq, 8 hd values per step
    uint4 qf[QK_STEPS];
    {
        const bf16* qrow = q + ((int64_t)(w.row0 + row) * n_q_heads + head) * HD;
#pragma unroll
        for (int kk = 0; kk < QK_STEPS; ++kk)
            qf[kk] = *reinterpret_cast<const uint4*>(qrow + kk * 16 + lh * 8);
    }

    // ---- tile loader geometry
    const int64_t k_head_off = (int64_t)gk * CF_PAGE_TOKENS * HD;
    const int64_t v_head_off = (int64_t)g.n_kv_heads * CF_PAGE_TOKENS * HD + (int64_t)gk * HD * CF_PAGE_TOKENS;
    int k_row[NLD], k_lds[NLD], k_goff[NLD];
    int v_page[NLD], v_lds[NLD], v_goff[NLD], v_key0[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        int v = tid + j * 256;
        int r = v / K_NCH, c = v % K_NCH;          // key row, chunk
        int ksw = (HD == 128) ? (r & 15) : ((r >> 1) & 7);
        k_row[j] = r;
        k_lds[j] = r * K_ROWB + ((c ^ ksw) << 4);
        k_goff[j] = (r % CF_PAGE_TOKENS) * HD + c * 8;
        int d = v / 8, cv = v % 8;                 // hd row, chunk = page*2 + half
        v_page[j] = cv >> 1;
        v_lds[j] = K_TILE + d * V_ROWB + ((cv ^ ((d >> 1) & 7)) << 4);
        v_goff[j] = d * CF_PAGE_TOKENS + (cv & 1) * 8;
        v_key0[j] = (cv >> 1) * CF_PAGE_TOKENS + (cv & 1) * 8;   // first key of the vector in the tile
    }

    uint4 rk[NLD], rv[NLD];
    // Global -> registers for one tile.  Slots past the last needed key may hold anything
    // (even NaN patterns): they are zeroed so that their zero probabilities cannot poison
    // the second product.
#define CF_FETCH(TILE)                                                                          \
    {                                                                                           \
        int tile_ = (TILE);                                                                     \
        int page0_ = tile_ * (KT / CF_PAGE_TOKENS);                                             \
        _Pragma("unroll") for (int j = 0; j < NLD; ++j) {                                       \
            int pk = min(page0_ + k_row[j] / CF_PAGE_TOKENS, last_page);                        \
            rk[j] = *reinterpret_cast<const uint4*>(pool_layer + (int64_t)pt[pk] * g.page_elems + \
                                                    k_head_off + k_goff[j]);                    \
            int pv = min(page0_ + v_page[j], last_page);                                        \
            uint4 val = *reinterpret_cast<const uint4*>(pool_layer + (int64_t)pt[pv] * g.page_elems + \
                                                        v_head_off + v_goff[j]);                \
            int left = kv_end - (tile_ * KT + v_key0[j]);   /* valid keys in this vector */     \
            if (left < 8) {                                                                     \
                val.x = left <= 0 ? 0u : (left == 1 ? val.x & 0xFFFFu : val.x);                 \
                val.y = left <= 2 ? 0u : (left == 3 ? val.y & 0xFFFFu : val.y);                 \
                val.z = left <= 4 ? 0u : (left == 5 ? val.z & 0xFFFFu : val.z);                 \
                val.w = left <= 6 ? 0u : (left == 7 ? val.w & 0xFFFFu : val.w);                 \
            }                                                                                   \
            rv[j] = val;                                                                        \
        }                                                                                       \
    }
#define CF_STASH(STAGE_PTR)                                                                     \
    {                                                                                           \
        char* st_ = (STAGE_PTR);                                                                \
        _Pragma("unroll") for (int j = 0; j < NLD; ++j) {                                       \
            *reinterpret_cast<uint4*>(st_ + k_lds[j]) = rk[j];                                  \
            *reinterpret_cast<uint4*>(st_ + v_lds[j]) = rv[j];                                  \
        }                                                                                       \
    }

    f32x16_t o_acc[D_TILES];
#pragma unroll
    for (int t = 0; t < D_TILES; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[t][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float scale_log2e = rsqrtf((float)HD) * 1.4426950408889634f;

    // fragment read offsets
    int ksw_l = (HD == 128) ? (lq & 15) : ((lq >> 1) & 7);
    int vsw_l = (lq >> 1) & 7;

    CF_FETCH(0);
    CF_STASH(smem);
    __syncthreads();

    for (int tile = 0; tile < n_tiles; ++tile) {
        char* cur = smem + (tile & 1) * STAGE;
        char* nxt = smem + ((tile + 1) & 1) * STAGE;
        CF_FETCH(min(tile + 1, n_tiles - 1));
        int key_base = tile * KT;
        if (key_base <= wave_last_q) {               // wave-uniform: tile not fully masked
            // ---- S^T = K Q^T : two 32-key fragments
            f32x16_t s[2];
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[tt][r] = 0.f;
#pragma unroll
                for (int kk = 0; kk < QK_STEPS; ++kk) {
                    uint4 kf = *reinterpret_cast<const uint4*>(
                        cur + (tt * 32 + lq) * K_ROWB + (((2 * kk + lh) ^ ksw_l) << 4));
                    s[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8_t, kf), __builtin_bit_cast(bf16x8_t, qf[kk]), s[tt], 0, 0, 0);
                }
            }
            // ---- scale, causal mask, online softmax (lane = one query row, 32 of its 64 keys)
            bool need_mask = key_base + KT - 1 > wave_first_q;
            float tmax = -INFINITY;
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float v = s[tt][r] * scale_log2e;
                    if (need_mask) {
                        int kpos = key_base + tt * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                        v = (kpos > qpos) ? -INFINITY : v;
                    }
                    s[tt][r] = v;
                    tmax = fmaxf(tmax, v);
                }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            float m_new = fmaxf(m_run, tmax);        // finite: key 0 is visible to every row
            float corr = exp2f(m_run - m_new);
            float psum = 0.f;
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float p = exp2f(s[tt][r] - m_new);
                    s[tt][r] = p;
                    psum += p;
                }
            l_run = l_run * corr + psum;
            m_run = m_new;
#pragma unroll
            for (int t = 0; t < D_TILES; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[t][r] *= corr;
            // ---- O^T += V^T P^T : 4 steps of 16 keys (one page each)
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                int tt = st >> 1, b0 = (st & 1) * 2;
                uint4 pf;
                pf.x = pack_bf16x2(s[tt][4 * b0 + 0], s[tt][4 * b0 + 1]);
                pf.y = pack_bf16x2(s[tt][4 * b0 + 2], s[tt][4 * b0 + 3]);
                pf.z = pack_bf16x2(s[tt][4 * b0 + 4], s[tt][4 * b0 + 5]);
                pf.w = pack_bf16x2(s[tt][4 * b0 + 6], s[tt][4 * b0 + 7]);
#pragma unroll
                for (int t = 0; t < D_TILES; ++t) {
                    // keys 4*lh..4*lh+3 and 8+4*lh.. of page `st`, for hd row 32t + lq
                    const char* vrow = cur + K_TILE + (t * 32 + lq) * V_ROWB;
                    uint2 v0 = *reinterpret_cast<const uint2*>(vrow + (((2 * st) ^ vsw_l) << 4) + lh * 8);
                    uint2 v1 = *reinterpret_cast<const uint2*>(vrow + (((2 * st + 1) ^ vsw_l) << 4) + lh * 8);
                    uint4 vf = make_uint4(v0.x, v0.y, v1.x, v1.y);
                    o_acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8_t, vf), __builtin_bit_cast(bf16x8_t, pf), o_acc[t], 0, 0, 0);
                }
            }
        }
        CF_STASH(nxt);
        __syncthreads();
    }
#undef CF_FETCH
#undef CF_STASH

    // ---- normalise and store: lane holds hd = 32t + 8b + 4*lh + i of query row lq
    float l_tot = l_run + __shfl_xor(l_run, 32);
    float inv = 1.0f / l_tot;
    if (wave * 32 + lq < w.n_rows) {
        bf16* orow = out + ((int64_t)(w.row0 + wave * 32 + lq) * n_q_heads + head) * HD;
#pragma unroll
        for (int t = 0; t < D_TILES; ++t)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                uint2 val;
                val.x = pack_bf16x2(o_acc[t][4 * b + 0] * inv, o_acc[t][4 * b + 1] * inv);
                val.y = pack_bf16x2(o_acc[t][4 * b + 2] * inv, o_acc[t][4 * b + 3] * inv);
                *reinterpret_cast<uint2*>(orow + t * 32 + 8 * b + 4 * lh) = val;
            }
    }
}

}  // namespace

bool attention_mfma_supported(int dtype, int head_dim, int n_q_heads, int n_kv_heads) {
    return dtype == CF_BF16 && (head_dim == 64 || head_dim == 128) && n_q_heads % n_kv_heads == 0;
}

void launch_attention_mfma(hipStream_t s, const void* q, void* out, const void* pool_layer,
                           const AttnWork* work, int n_work, const int32_t* page_tables,
                           int n_q_heads, KvGeom g) {
    if (n_work <= 0) return;
    dim3 grid(n_work, n_q_heads);
    if (g.head_dim == 128)
        attention_mfma_kernel<128><<<grid, 256, 0, s>>>((const bf16*)q, (bf16*)out, (const bf16*)pool_layer, work, page_tables, n_q_heads, g);
    else
        attention_mfma_kernel<64><<<grid, 256, 0, s>>>((const bf16*)q, (bf16*)out, (const bf16*)pool_layer, work, page_tables, n_q_heads, g);
}

}  // namespace cf
