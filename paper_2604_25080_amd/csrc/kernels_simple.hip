// Plain HIP kernels: embedding gather, RMSNorm, a tiled FMA GEMM, RoPE + paged
// K/V write, a lane-per-key attention, and the page scatter/gather.  These are
// the float32 path of the tiny configuration and the reference the MFMA
// kernels are tested against on the GPU; the page mover, norm, embed and RoPE
// kernels serve every configuration.
#include "kernels.h"
#include "rope.h"
#include "cacheflow.h"

namespace cf {

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return __uint_as_float((uint32_t)v.x << 16); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) {
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);   // round to nearest even (finite inputs)
    return bf16{(uint16_t)(u >> 16)};
}

// ------------------------------------------------------------------ embedding
template <typename T>
__global__ void embed_kernel(const T* __restrict__ E, const int32_t* __restrict__ tok,
                             float* __restrict__ h, int d) {
    int t = blockIdx.x;
    const T* src = E + (int64_t)tok[t] * d;
    float* dst = h + (int64_t)t * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) dst[i] = to_f32(src[i]);
}

void launch_embed(hipStream_t s, int dtype, const void* E, const int32_t* tok, float* h, int T,
                  int d) {
    if (T <= 0) return;
    if (dtype == CF_F32)
        embed_kernel<float><<<T, 256, 0, s>>>((const float*)E, tok, h, d);
    else
        embed_kernel<bf16><<<T, 256, 0, s>>>((const bf16*)E, tok, h, d);
}

// -------------------------------------------------------------------- RMSNorm
// One 256-thread block per row; the row stays in registers between the two passes.
// With `delta` the pending residual update is folded in first: h += delta (written
// back unless the rows are gathered through row_idx), then the norm of the new h.
// NV > 0: the row is exactly NV float4 per thread (d = 1024 NV), so nothing in the loops is
// conditional and all of a thread's loads are in flight together; NV = 0: any d up to 8192.
// Same order of additions either way, so the same bits.
template <typename T, int NV>
__global__ void __launch_bounds__(256)
rmsnorm_kernel(float* __restrict__ h, const float* __restrict__ delta,
               const float* __restrict__ gain, T* __restrict__ out, int d, float eps,
               const int32_t* __restrict__ row_idx) {
    __shared__ float red[4];
    int t = blockIdx.x;
    int64_t srow = row_idx ? row_idx[t] : t;
    float* src = h + srow * d;
    const float* dsrc = delta ? delta + srow * d : nullptr;
    T* dst = out + (int64_t)t * d;
    constexpr int MAXV = NV > 0 ? NV : 8;   // d <= 256*4*8 = 8192
    float4 v[MAXV];
    int nvec = NV > 0 ? NV * 256 : d / 4;
    float ss = 0.f;
    if constexpr (NV > 0) {
        float4 dv[MAXV];
#pragma unroll
        for (int i = 0; i < MAXV; ++i) v[i] = reinterpret_cast<const float4*>(src)[threadIdx.x + i * 256];
        if (dsrc) {
#pragma unroll
            for (int i = 0; i < MAXV; ++i) dv[i] = reinterpret_cast<const float4*>(dsrc)[threadIdx.x + i * 256];
#pragma unroll
            for (int i = 0; i < MAXV; ++i) {
                v[i].x += dv[i].x; v[i].y += dv[i].y; v[i].z += dv[i].z; v[i].w += dv[i].w;
                if (!row_idx) reinterpret_cast<float4*>(src)[threadIdx.x + i * 256] = v[i];
            }
        }
#pragma unroll
        for (int i = 0; i < MAXV; ++i)
            ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
    } else
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        int idx = threadIdx.x + i * 256;
        if (idx < nvec) {
            v[i] = reinterpret_cast<const float4*>(src)[idx];
            if (dsrc) {
                float4 dv = reinterpret_cast<const float4*>(dsrc)[idx];
                v[i].x += dv.x; v[i].y += dv.y; v[i].z += dv.z; v[i].w += dv.w;
                if (!row_idx) reinterpret_cast<float4*>(src)[idx] = v[i];
            }
            ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
        }
    }
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = red[0] + red[1] + red[2] + red[3];
    float r = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        int idx = threadIdx.x + i * 256;
        if (idx < nvec) {
            float4 g = reinterpret_cast<const float4*>(gain)[idx];
            dst[idx * 4 + 0] = from_f32<T>(v[i].x * r * g.x);
            dst[idx * 4 + 1] = from_f32<T>(v[i].y * r * g.y);
            dst[idx * 4 + 2] = from_f32<T>(v[i].z * r * g.z);
            dst[idx * 4 + 3] = from_f32<T>(v[i].w * r * g.w);
        }
    }
}

void launch_rmsnorm(hipStream_t s, int dtype, float* h, const float* delta, const float* gain,
                    void* out, int T, int d, float eps, const int32_t* row_idx) {
    if (T <= 0) return;
    if (dtype == CF_F32)
        rmsnorm_kernel<float, 0><<<T, 256, 0, s>>>(h, delta, gain, (float*)out, d, eps, row_idx);
    else if (d == 4096)
        rmsnorm_kernel<bf16, 4><<<T, 256, 0, s>>>(h, delta, gain, (bf16*)out, d, eps, row_idx);
    else if (d == 8192)
        rmsnorm_kernel<bf16, 8><<<T, 256, 0, s>>>(h, delta, gain, (bf16*)out, d, eps, row_idx);
    else
        rmsnorm_kernel<bf16, 0><<<T, 256, 0, s>>>(h, delta, gain, (bf16*)out, d, eps, row_idx);
}

// ---------------------------------------------------------------- simple GEMM
// 64x64 tile, 256 threads, 4x4 outputs per thread, K in steps of 16, float FMA.
template <typename T, int EPI>
__global__ void __launch_bounds__(256)
gemm_simple_kernel(const T* __restrict__ A, const T* __restrict__ W, const T* __restrict__ W2,
                   float* __restrict__ Cf, T* __restrict__ Dt, int M, int N, int K) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 4];
    __shared__ float Ws[BK][BN + 4];
    __shared__ float W2s[EPI == EPI_SILU_MUL ? BK : 1][BN + 4];
    int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    float acc[4][4] = {}, acc2[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += BK) {
        for (int i = threadIdx.x; i < BM * BK; i += 256) {
            int r = i / BK, c = i % BK;
            int gm = m0 + r, gn = n0 + r, gk = k0 + c;
            As[c][r] = (gm < M && gk < K) ? to_f32(A[(int64_t)gm * K + gk]) : 0.f;
            Ws[c][r] = (gn < N && gk < K) ? to_f32(W[(int64_t)gn * K + gk]) : 0.f;
            if (EPI == EPI_SILU_MUL)
                W2s[c][r] = (gn < N && gk < K) ? to_f32(W2[(int64_t)gn * K + gk]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float a[4], b[4], b2[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Ws[k][tx * 4 + j];
            if (EPI == EPI_SILU_MUL) {
#pragma unroll
                for (int j = 0; j < 4; ++j) b2[j] = W2s[k][tx * 4 + j];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
                    if (EPI == EPI_SILU_MUL) acc2[i][j] = fmaf(a[i], b2[j], acc2[i][j]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int gn = n0 + tx * 4 + j;
            if (gn >= N) continue;
            int64_t o = (int64_t)gm * N + gn;
            float v = acc[i][j];
            if (EPI == EPI_STORE_F32) Cf[o] = v;
            else if (EPI == EPI_ADD_F32) Cf[o] += v;
            else if (EPI == EPI_STORE_T) Dt[o] = from_f32<T>(v);
            else Dt[o] = from_f32<T>(v / (1.0f + expf(-v)) * acc2[i][j]);
        }
    }
}

template <typename T>
static void gemm_simple_dispatch(hipStream_t s, const T* A, const T* W, const T* W2, float* Cf,
                                 T* Dt, int M, int N, int K, int epi) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    switch (epi) {
        case EPI_STORE_F32: gemm_simple_kernel<T, EPI_STORE_F32><<<grid, 256, 0, s>>>(A, W, W2, Cf, Dt, M, N, K); break;
        case EPI_ADD_F32: gemm_simple_kernel<T, EPI_ADD_F32><<<grid, 256, 0, s>>>(A, W, W2, Cf, Dt, M, N, K); break;
        case EPI_STORE_T: gemm_simple_kernel<T, EPI_STORE_T><<<grid, 256, 0, s>>>(A, W, W2, Cf, Dt, M, N, K); break;
        default: gemm_simple_kernel<T, EPI_SILU_MUL><<<grid, 256, 0, s>>>(A, W, W2, Cf, Dt, M, N, K); break;
    }
}

void launch_gemm_simple(hipStream_t s, int dtype, const void* A, const void* W, const void* W2,
                        float* Cf, void* Dt, int M, int N, int K, int epi) {
    if (M <= 0 || N <= 0) return;
    if (dtype == CF_F32)
        gemm_simple_dispatch<float>(s, (const float*)A, (const float*)W, (const float*)W2, Cf, (float*)Dt, M, N, K, epi);
    else
        gemm_simple_dispatch<bf16>(s, (const bf16*)A, (const bf16*)W, (const bf16*)W2, Cf, (bf16*)Dt, M, N, K, epi);
}

// ------------------------------------------------------- RoPE + paged KV write
// One block per token.  Rotates Q and K in float with table angles (built on the
// host in double), writes Q to the packed query buffer and K/V into the
// token's page slot: K as [head][slot][hd], V transposed as [head][hd][slot].
template <typename T>
__global__ void __launch_bounds__(256)
rope_write_kernel(const float* __restrict__ qkv, const int32_t* __restrict__ pos,
                  const int32_t* __restrict__ slot, const float2* __restrict__ cos_sin,
                  T* __restrict__ q_out, T* __restrict__ pool_layer, int n_q_heads, KvGeom g) {
    int t = blockIdx.x;
    int hd = g.head_dim, half = hd >> 1;
    int nq = n_q_heads * hd, nk = g.n_kv_heads * hd;
    const float* row = qkv + (int64_t)t * (nq + 2 * nk);
    const float2* cs = cos_sin + (int64_t)pos[t] * half;
    int sl = slot[t];
    T* page = pool_layer + (int64_t)(sl / CF_PAGE_TOKENS) * g.page_elems;
    int s16 = sl % CF_PAGE_TOKENS;
    T* kpage = page;
    T* vpage = page + (int64_t)g.n_kv_heads * CF_PAGE_TOKENS * hd;
    int n_rot = (n_q_heads + g.n_kv_heads) * half;
    for (int i = threadIdx.x; i < n_rot; i += blockDim.x) {
        int head = i / half, j = i % half;
        float2 c = cs[j];
        float x1 = row[head * hd + j], x2 = row[head * hd + j + half];
        float y1, y2;
        rope_rotate(x1, x2, c, y1, y2);
        if (head < n_q_heads) {
            T* dst = q_out + (int64_t)t * nq + head * hd;
            dst[j] = from_f32<T>(y1);
            dst[j + half] = from_f32<T>(y2);
        } else {
            int gk = head - n_q_heads;
            T* dst = kpage + ((int64_t)gk * CF_PAGE_TOKENS + s16) * hd;
            dst[j] = from_f32<T>(y1);
            dst[j + half] = from_f32<T>(y2);
        }
    }
    for (int i = threadIdx.x; i < nk; i += blockDim.x) {
        int gk = i / hd, j = i % hd;
        vpage[((int64_t)gk * hd + j) * CF_PAGE_TOKENS + s16] = from_f32<T>(row[nq + nk + i]);
    }
}

void launch_rope_write(hipStream_t s, int dtype, const float* qkv, const int32_t* pos,
                       const int32_t* slot, const float2* cos_sin, void* q_out, void* pool_layer,
                       int T, int n_q_heads, KvGeom g) {
    if (T <= 0) return;
    if (dtype == CF_F32)
        rope_write_kernel<float><<<T, 256, 0, s>>>(qkv, pos, slot, cos_sin, (float*)q_out, (float*)pool_layer, n_q_heads, g);
    else
        rope_write_kernel<bf16><<<T, 256, 0, s>>>(qkv, pos, slot, cos_sin, (bf16*)q_out, (bf16*)pool_layer, n_q_heads, g);
}

// ------------------------------------------------------------ simple attention
// grid (work item, q head); 4 waves per block, each wave takes rows w, w+4, ...
// Within a row every lane owns keys lane, lane+64, ... and keeps its own online
// softmax state; lanes are merged at the end.  All float arithmetic.
template <typename T, int HD>
__global__ void __launch_bounds__(256)
attention_simple_kernel(const T* __restrict__ q, T* __restrict__ out,
                        const T* __restrict__ pool_layer, const AttnWork* __restrict__ work,
                        const int32_t* __restrict__ page_tables, int n_q_heads, KvGeom g) {
    __shared__ float qs[4][HD];
    AttnWork w = work[blockIdx.x];
    int head = blockIdx.y;
    int gk = head / (n_q_heads / g.n_kv_heads);
    int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int32_t* pt = page_tables + w.pt_off;
    float scale = rsqrtf((float)HD);
    int64_t v_off = (int64_t)g.n_kv_heads * CF_PAGE_TOKENS * HD;
    for (int rb = 0; rb < w.n_rows; rb += 4) {      // uniform trip count for the barriers
        int r = rb + wave;
        bool active = r < w.n_rows;
        __syncthreads();
        if (active) {
            const T* qrow = q + ((int64_t)(w.row0 + r) * n_q_heads + head) * HD;
            for (int i = lane; i < HD; i += 64) qs[wave][i] = to_f32(qrow[i]) * scale;
        }
        __syncthreads();
        if (!active) continue;
        int p = w.pos0 + r;
        float m = -INFINITY, l = 0.f, acc[HD];
#pragma unroll
        for (int i = 0; i < HD; ++i) acc[i] = 0.f;
        for (int j = lane; j <= p; j += 64) {
            const T* page = pool_layer + (int64_t)pt[j / CF_PAGE_TOKENS] * g.page_elems;
            int s16 = j % CF_PAGE_TOKENS;
            const T* krow = page + ((int64_t)gk * CF_PAGE_TOKENS + s16) * HD;
            float sc = 0.f;
#pragma unroll 8
            for (int i = 0; i < HD; ++i) sc = fmaf(qs[wave][i], to_f32(krow[i]), sc);
            float mn = fmaxf(m, sc);
            float corr = expf(m - mn), pj = expf(sc - mn);
            l = l * corr + pj;
            const T* vcol = page + v_off + (int64_t)gk * HD * CF_PAGE_TOKENS + s16;
#pragma unroll 8
            for (int i = 0; i < HD; ++i)
                acc[i] = acc[i] * corr + pj * to_f32(vcol[(int64_t)i * CF_PAGE_TOKENS]);
            m = mn;
        }
        float mall = m;
        for (int o = 32; o > 0; o >>= 1) mall = fmaxf(mall, __shfl_xor(mall, o));
        float f = (m == -INFINITY) ? 0.f : expf(m - mall);
        float lsum = l * f;
        for (int o = 32; o > 0; o >>= 1) lsum += __shfl_xor(lsum, o);
        T* orow = out + ((int64_t)(w.row0 + r) * n_q_heads + head) * HD;
        float inv = 1.0f / lsum;
#pragma unroll
        for (int i = 0; i < HD; ++i) {
            float a = acc[i] * f;
            for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
            if (lane == (i & 63)) orow[i] = from_f32<T>(a * inv);
        }
    }
}

void launch_attention_simple(hipStream_t s, int dtype, const void* q, void* out,
                             const void* pool_layer, const AttnWork* work, int n_work,
                             const int32_t* page_tables, int n_q_heads, KvGeom g) {
    if (n_work <= 0) return;
    dim3 grid(n_work, n_q_heads);
#define CF_ATTN(TT, HD) attention_simple_kernel<TT, HD><<<grid, 256, 0, s>>>((const TT*)q, (TT*)out, (const TT*)pool_layer, work, page_tables, n_q_heads, g)
    if (dtype == CF_F32) { if (g.head_dim == 64) CF_ATTN(float, 64); else CF_ATTN(float, 128); }
    else { if (g.head_dim == 64) CF_ATTN(bf16, 64); else CF_ATTN(bf16, 128); }
#undef CF_ATTN
}

// --------------------------------------------------- page scatter / page gather
// Moves runs of whole pages between a contiguous staging area and the page
// pool.  One block per (page, quarter-page); 16-byte vectors.  A page whose
// token range [lo,hi) is not the full [0,16) is moved slot by slot so that
// bytes of slots outside the range are never written (the other stream may be
// writing them).
template <typename T, bool TO_PAGES>
__global__ void __launch_bounds__(256)
page_move_kernel(T* __restrict__ staging, T* __restrict__ pool, const PageJob* __restrict__ jobs,
                 int n_jobs, const int32_t* __restrict__ page_tables, KvGeom g, int split) {
    // find the job of this block by bisection over the jobs' first block index
    int b = blockIdx.x;
    int ji = 0, jhi = n_jobs - 1;   // last job whose block_first <= b
    while (ji < jhi) {
        int mid = (ji + jhi + 1) >> 1;
        if (jobs[mid].block_first <= b) ji = mid; else jhi = mid - 1;
    }
    PageJob job = jobs[ji];
    int local = b - job.block_first;
    int pg = local / split, part = local % split;
    int jpage = job.page_first + pg;
    int lo = max(job.tok_first - jpage * CF_PAGE_TOKENS, 0);
    int hi = min(job.tok_end - jpage * CF_PAGE_TOKENS, CF_PAGE_TOKENS);
    constexpr int VE = 16 / sizeof(T);              // elements per 16-byte vector
    int64_t nvec = g.page_elems / VE;
    int64_t per = (nvec + split - 1) / split;
    int64_t v0 = part * per, v1 = min(nvec, v0 + per);
    T* spage = staging + job.staging_off / (int64_t)sizeof(T) + (int64_t)pg * g.page_elems;
    T* dpage = pool + (int64_t)job.layer * g.layer_stride +
               (int64_t)page_tables[job.pt_off + jpage] * g.page_elems;
    T* src = TO_PAGES ? spage : dpage;
    T* dst = TO_PAGES ? dpage : spage;
    bool full = (lo == 0 && hi == CF_PAGE_TOKENS);
    int64_t k_elems = (int64_t)g.n_kv_heads * CF_PAGE_TOKENS * g.head_dim;
    for (int64_t v = v0 + threadIdx.x; v < v1; v += 256) {
        uint4 val = reinterpret_cast<const uint4*>(src)[v];
        if (full) {
            reinterpret_cast<uint4*>(dst)[v] = val;
            continue;
        }
        int64_t e = v * VE;
        if (e < k_elems) {  // K part: the vector lies inside one slot row
            int s16 = (int)((e / g.head_dim) % CF_PAGE_TOKENS);
            if (s16 >= lo && s16 < hi) reinterpret_cast<uint4*>(dst)[v] = val;
            else if (!TO_PAGES) reinterpret_cast<uint4*>(dst)[v] = make_uint4(0, 0, 0, 0);
        } else {            // V part: the vector spans VE consecutive slots of one column
            int s0 = (int)((e - k_elems) % CF_PAGE_TOKENS);
            const T* sv = reinterpret_cast<const T*>(&val);
            for (int i = 0; i < VE; ++i) {
                bool in = (s0 + i >= lo && s0 + i < hi);
                if (in) dst[e + i] = sv[i];
                else if (!TO_PAGES) dst[e + i] = T{};
            }
        }
    }
}

// Host -> pages in one step: a few resident workgroups stream the loaded KV straight out of
// pinned (device-mapped) host memory over the host link and store it into the page slots --
// no staging copy, no per-transfer DMA set-up, full link bandwidth at any run length.  A job is
// a run of consecutive pages of one (request, layer), contiguous in host memory; it is cut into
// units of PAGE_LOAD_UNIT_VECS 16-byte vectors, and each workgroup walks the units
// u = blockIdx.x, blockIdx.x + gridDim.x, ... with all of a unit's loads (16 per thread, 64 KiB
// per workgroup) in flight before the first store: the link's bandwidth-delay product is about
// 256 KiB, so a handful of workgroups saturates it.  job.staging_off holds the ADDRESS of the
// run's first page in host memory, job.block_first the job's first unit.
template <typename T>
__global__ void __launch_bounds__(256)
page_load_kernel(T* __restrict__ pool, const PageJob* __restrict__ jobs, int n_jobs, int n_units,
                 const int32_t* __restrict__ page_tables, KvGeom g) {
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    constexpr int VE = 16 / sizeof(T);
    constexpr int U = PAGE_LOAD_UNIT_VECS / 256;
    const int nvec = (int)(g.page_elems / VE);
    const int64_t k_elems = (int64_t)g.n_kv_heads * CF_PAGE_TOKENS * g.head_dim;
    for (int b = blockIdx.x; b < n_units; b += gridDim.x) {
        int ji = 0, jhi = n_jobs - 1;
        while (ji < jhi) {
            int mid = (ji + jhi + 1) >> 1;
            if (jobs[mid].block_first <= b) ji = mid; else jhi = mid - 1;
        }
        PageJob job = jobs[ji];
        // 32-bit index arithmetic inside the unit (host code keeps n_pages * nvec below 2^31)
        const unsigned job_vecs = (unsigned)job.n_pages * (unsigned)nvec;
        const unsigned base = (unsigned)(b - job.block_first) * PAGE_LOAD_UNIT_VECS;
        const unsigned pg0 = base / (unsigned)nvec, rem0 = base - pg0 * (unsigned)nvec;
        typedef const v4u __attribute__((address_space(1))) * gsrc_t;   // global, not flat, loads
        gsrc_t src = (gsrc_t)((uintptr_t)job.staging_off) + base;
        T* layer_base = pool + (int64_t)job.layer * g.layer_stride;
        const int32_t* table = page_tables + job.pt_off + job.page_first;
        v4u val[U];
        int pid[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // unconditional (clamped) so that all U loads are in flight together: a load under
            // a branch is waited for before the branch rejoins
            unsigned o = min((unsigned)(u * 256 + threadIdx.x), job_vecs - 1 - base);
            val[u] = __builtin_nontemporal_load(src + o);
            pid[u] = table[pg0 + (rem0 + o) / (unsigned)nvec];
        }
        // everything has landed before the first store, so that the stores below are not
        // separated by waits of their own
        __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            unsigned o = u * 256 + threadIdx.x;
            if (base + o >= job_vecs) continue;
            int pg = (int)(pg0 + (rem0 + o) / (unsigned)nvec);
            int v = (int)(rem0 + o - (unsigned)(pg - (int)pg0) * (unsigned)nvec);
            int jpage = job.page_first + pg;
            int lo = max(job.tok_first - jpage * CF_PAGE_TOKENS, 0);
            int hi = min(job.tok_end - jpage * CF_PAGE_TOKENS, CF_PAGE_TOKENS);
            T* dst = layer_base + (int64_t)pid[u] * g.page_elems;
            if (lo == 0 && hi == CF_PAGE_TOKENS) {
                reinterpret_cast<v4u*>(dst)[v] = val[u];
                continue;
            }
            int64_t e = (int64_t)v * VE;
            if (e < k_elems) {  // K part: the vector lies inside one slot row
                int s16 = (int)((e / g.head_dim) % CF_PAGE_TOKENS);
                if (s16 >= lo && s16 < hi) reinterpret_cast<v4u*>(dst)[v] = val[u];
            } else {            // V part: the vector spans VE consecutive slots of one column
                int s0 = (int)((e - k_elems) % CF_PAGE_TOKENS);
                const T* sv = reinterpret_cast<const T*>(&val[u]);
                for (int i = 0; i < VE; ++i)
                    if (s0 + i >= lo && s0 + i < hi) dst[e + i] = sv[i];
            }
        }
    }
}

// Pages -> pinned host memory, the mirror image of page_load_kernel: whole pages of a run are
// read from the pool (16 loads per thread in flight) and stored straight into the host block
// over the host link.  job.staging_off holds the host ADDRESS of the run's first page.
template <typename T>
__global__ void __launch_bounds__(256)
page_store_kernel(const T* __restrict__ pool, const PageJob* __restrict__ jobs, int n_jobs, int n_units,
                  const int32_t* __restrict__ page_tables, KvGeom g) {
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    constexpr int VE = 16 / sizeof(T);
    constexpr int U = PAGE_LOAD_UNIT_VECS / 256;
    const int nvec = (int)(g.page_elems / VE);
    for (int b = blockIdx.x; b < n_units; b += gridDim.x) {
        int ji = 0, jhi = n_jobs - 1;
        while (ji < jhi) {
            int mid = (ji + jhi + 1) >> 1;
            if (jobs[mid].block_first <= b) ji = mid; else jhi = mid - 1;
        }
        PageJob job = jobs[ji];
        const unsigned job_vecs = (unsigned)job.n_pages * (unsigned)nvec;
        const unsigned base = (unsigned)(b - job.block_first) * PAGE_LOAD_UNIT_VECS;
        const unsigned pg0 = base / (unsigned)nvec, rem0 = base - pg0 * (unsigned)nvec;
        v4u* dst = reinterpret_cast<v4u*>((uintptr_t)job.staging_off) + base;
        const T* layer_base = pool + (int64_t)job.layer * g.layer_stride;
        const int32_t* table = page_tables + job.pt_off + job.page_first;
        v4u val[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            unsigned o = min((unsigned)(u * 256 + threadIdx.x), job_vecs - 1 - base);   // clamped, unconditional
            unsigned pg = pg0 + (rem0 + o) / (unsigned)nvec;
            unsigned v = rem0 + o - (pg - pg0) * (unsigned)nvec;
            const T* src = layer_base + (int64_t)table[pg] * g.page_elems;
            val[u] = reinterpret_cast<const v4u*>(src)[v];
        }
        // slots past the run's last token (the tail of a request's last page) go out as zero,
        // whatever the pool holds there
        const int64_t k_elems = (int64_t)g.n_kv_heads * CF_PAGE_TOKENS * g.head_dim;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            unsigned o = u * 256 + threadIdx.x;
            if (base + o >= job_vecs) continue;
            unsigned pg = pg0 + (rem0 + o) / (unsigned)nvec;
            int hi = job.tok_end - (job.page_first + (int)pg) * CF_PAGE_TOKENS;
            if (hi < CF_PAGE_TOKENS) {
                int64_t e = (int64_t)(rem0 + o - (pg - pg0) * (unsigned)nvec) * VE;
                if (e < k_elems) {          // K part: the vector lies inside one slot row
                    if ((int)((e / g.head_dim) % CF_PAGE_TOKENS) >= hi) val[u] = v4u{0, 0, 0, 0};
                } else {                    // V part: VE consecutive slots of one column
                    int s0 = (int)((e - k_elems) % CF_PAGE_TOKENS);
                    T* sv = reinterpret_cast<T*>(&val[u]);
                    for (int i = 0; i < VE; ++i)
                        if (s0 + i >= hi) sv[i] = T{};
                }
            }
            __builtin_nontemporal_store(val[u], dst + o);
        }
    }
}

void launch_page_store(hipStream_t s, int dtype, const void* pool, const PageJob* jobs, int n_jobs,
                       int n_units, int n_workgroups, const int32_t* page_tables, KvGeom g) {
    if (n_jobs <= 0 || n_units <= 0) return;
    int grid = n_workgroups < n_units ? n_workgroups : n_units;
    if (dtype == CF_F32)
        page_store_kernel<float><<<grid, 256, 0, s>>>((const float*)pool, jobs, n_jobs, n_units, page_tables, g);
    else
        page_store_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)pool, jobs, n_jobs, n_units, page_tables, g);
}

// Pacing of the copy stream (emulation of a slower storage tier): a mark kernel stores the
// constant-rate wall clock, a wait kernel holds the stream until `ticks` of that clock have
// passed since the mark.  One lane; the spin is bounded (2^26 sleeps of ~1 us), so the kernel
// always ends.
__global__ void pace_mark_kernel(unsigned long long* t0) { *t0 = wall_clock64(); }

__global__ void pace_wait_kernel(const unsigned long long* t0, unsigned long long ticks) {
    unsigned long long start = *t0;
    for (int i = 0; i < (1 << 26); ++i) {
        if (wall_clock64() - start >= ticks) break;
        __builtin_amdgcn_s_sleep(32);
    }
}

void launch_pace_mark(hipStream_t s, void* t0) { pace_mark_kernel<<<1, 1, 0, s>>>((unsigned long long*)t0); }
void launch_pace_wait(hipStream_t s, const void* t0, unsigned long long ticks) {
    pace_wait_kernel<<<1, 1, 0, s>>>((const unsigned long long*)t0, ticks);
}

// out[i] = h[i] (+ dl[i]): the residual stream of packed rows as it enters a layer
__global__ void __launch_bounds__(256)
residual_rows_kernel(float* __restrict__ out, const float* __restrict__ h, const float* __restrict__ dl,
                     int64_t n4) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    float4 a = reinterpret_cast<const float4*>(h)[i];
    if (dl) {
        float4 b = reinterpret_cast<const float4*>(dl)[i];
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    reinterpret_cast<float4*>(out)[i] = a;
}

// out[j] = h[idx[j]] (+ dl[idx[j]]) for the listed rows that lie in [a0, a1) or [b0, b1);
// others are skipped
__global__ void __launch_bounds__(256)
residual_gather_kernel(float* __restrict__ out, const float* __restrict__ h, const float* __restrict__ dl,
                       const int32_t* __restrict__ idx, int d4, int a0, int a1, int b0, int b1) {
    int r = idx[blockIdx.x];
    if (!((r >= a0 && r < a1) || (r >= b0 && r < b1))) return;
    const float4* hr = reinterpret_cast<const float4*>(h) + (int64_t)r * d4;
    const float4* dr = dl ? reinterpret_cast<const float4*>(dl) + (int64_t)r * d4 : nullptr;
    float4* o = reinterpret_cast<float4*>(out) + (int64_t)blockIdx.x * d4;
    for (int i = threadIdx.x; i < d4; i += 256) {
        float4 a = hr[i];
        if (dr) { float4 b = dr[i]; a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w; }
        o[i] = a;
    }
}

void launch_residual_gather(hipStream_t s, float* out, const float* h, const float* dl, const int32_t* idx,
                            int n, int d, int a0, int a1, int b0, int b1) {
    if (n <= 0) return;
    residual_gather_kernel<<<n, 256, 0, s>>>(out, h, dl, idx, d / 4, a0, a1, b0, b1);
}

void launch_residual_rows(hipStream_t s, float* out, const float* h, const float* dl, int T, int d) {
    int64_t n4 = (int64_t)T * d / 4;
    if (n4 <= 0) return;
    residual_rows_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, s>>>(out, h, dl, n4);
}

void launch_page_load(hipStream_t s, int dtype, void* pool, const PageJob* jobs, int n_jobs,
                      int n_units, int n_workgroups, const int32_t* page_tables, KvGeom g) {
    if (n_jobs <= 0 || n_units <= 0) return;
    int grid = n_workgroups < n_units ? n_workgroups : n_units;
    if (dtype == CF_F32)
        page_load_kernel<float><<<grid, 256, 0, s>>>((float*)pool, jobs, n_jobs, n_units, page_tables, g);
    else
        page_load_kernel<bf16><<<grid, 256, 0, s>>>((bf16*)pool, jobs, n_jobs, n_units, page_tables, g);
}

void launch_page_move(hipStream_t s, int dtype, void* staging, void* pool, const PageJob* jobs,
                      int n_jobs, int n_blocks, const int32_t* page_tables, KvGeom g,
                      bool to_pages) {
    if (n_jobs <= 0 || n_blocks <= 0) return;
    // the host computed block_first with the same split
    int split = 4;
    if (dtype == CF_F32) {
        if (to_pages) page_move_kernel<float, true><<<n_blocks, 256, 0, s>>>((float*)staging, (float*)pool, jobs, n_jobs, page_tables, g, split);
        else page_move_kernel<float, false><<<n_blocks, 256, 0, s>>>((float*)staging, (float*)pool, jobs, n_jobs, page_tables, g, split);
    } else {
        if (to_pages) page_move_kernel<bf16, true><<<n_blocks, 256, 0, s>>>((bf16*)staging, (bf16*)pool, jobs, n_jobs, page_tables, g, split);
        else page_move_kernel<bf16, false><<<n_blocks, 256, 0, s>>>((bf16*)staging, (bf16*)pool, jobs, n_jobs, page_tables, g, split);
    }
}

}  // namespace cf
