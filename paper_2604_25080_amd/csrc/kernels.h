// Kernel launchers of the restoration library (internal).  Every launcher
// enqueues on the given stream and returns; none synchronises or allocates.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace cf {

// bf16 carried as its 16 raw bits; conversions are explicit.
struct bf16 {
    uint16_t x;
};

enum Epilogue {
    EPI_STORE_F32 = 0,  // C[m,n] = acc                     (float out)
    EPI_ADD_F32 = 1,    // C[m,n] += acc                    (float residual stream)
    EPI_STORE_T = 2,    // D[m,n] = (T)acc                  (model dtype out)
    EPI_SILU_MUL = 3,   // D[m,n] = (T)(silu(acc) * acc2)   acc2 from second weight W2
    // QKV projection with RoPE and the paged K/V write done on the accumulators (head_dim 128 / 64)
    EPI_QKV_ROPE128 = 4,
    EPI_QKV_ROPE64 = 5
};

// One q-block of attention work: rows [row0, row0+n_rows) of the packed query
// buffer belong to one request, the first of them sits at absolute position
// pos0, and the request's page ids start at page_tables[pt_off].
// Keys are walked in tiles of 64; the item covers tiles [tile_begin, tile_end).  part < 0:
// the item covers the whole key range and writes the normalised output; part >= 0: it is one
// slice of a split key range and writes an un-normalised partial result to slot `part`.
struct AttnWork {
    int32_t row0, n_rows, pos0, pt_off;
    int32_t tile_begin, tile_end, part, pad;
};
// Partial results [part_first, part_first + n_parts) belong to query rows [row0, row0 + n_rows).
struct AttnCombine {
    int32_t row0, n_rows, part_first, n_parts;
};
constexpr int ATTN_BLOCK_ROWS = 128;
constexpr int ATTN_KEY_TILE = 64;
constexpr int ATTN_MAX_PART_BLOCKS = 2048;   // (partial slots) x (Q heads) the partial buffer holds
inline size_t attn_part_bytes(int head_dim) {
    return (size_t)ATTN_MAX_PART_BLOCKS * ATTN_BLOCK_ROWS * (head_dim + 4) * sizeof(float);
}

// One contiguous run of pages of one layer of one request, staged in order.
struct PageJob {
    int64_t staging_off;   // byte offset of the run's first page in the staging buffer (staged
                           // path) or its ADDRESS in device-mapped host memory (direct path)
    int32_t layer;
    int32_t pt_off;        // request's page table offset
    int32_t page_first;    // index into the request's page table of the first page
    int32_t n_pages;
    int32_t tok_first;     // first token (absolute in request) to move
    int32_t tok_end;       // one past the last token to move
    int32_t block_first;   // first block index of this job in the launch grid
    int32_t pad;
};

struct KvGeom {
    int n_kv_heads, head_dim;
    int64_t page_elems;        // elements per page
    int64_t layer_stride;      // elements between layers in the pool
};

void launch_embed(hipStream_t s, int dtype, const void* E, const int32_t* tok, float* h, int T, int d);
// out = rmsnorm(h (+ delta)) * gain; with delta, h += delta is written back unless row_idx
// gathers the rows (delta is then indexed like h).
void launch_rmsnorm(hipStream_t s, int dtype, float* h, const float* delta, const float* gain,
                    void* out, int T, int d, float eps, const int32_t* row_idx);
// A[M,K], W[N,K] (and W2) in the model dtype; Cf float [M,N] or Dt model dtype [M,N].
void launch_gemm_simple(hipStream_t s, int dtype, const void* A, const void* W, const void* W2,
                        float* Cf, void* Dt, int M, int N, int K, int epi);
// true if the MFMA kernel supports this problem (bf16, aligned K)
bool gemm_mfma_supported(int dtype, int M, int N, int K, int epi);
void gemm_mfma_force_tile(int tile);   // 0 = heuristic, 256 or 128 = forced (tuning)
void launch_gemm_mfma(hipStream_t s, const void* A, const void* W, const void* W2, float* Cf,
                      void* Dt, int M, int N, int K, int epi);
// What the QKV projection needs to finish its own output: per packed row its absolute position
// (the RoPE angle) and pool slot (page * CF_PAGE_TOKENS + slot in page), the angle table
// [position][head_dim / 2] of (cos, sin), and the layer's slice of the page pool.
struct RopeEpilogue {
    const int32_t* pos;
    const int32_t* slot;
    const float2* cos_sin;
    void* pool_layer;
    int n_q_heads;
    KvGeom g;
};
// true if the MFMA GEMM can take the QKV projection [M, N = (Hq + 2 Hkv) * head_dim] with RoPE
// and the page write in its epilogue (the 256x256 tile, whose wave tile spans whole heads)
bool gemm_mfma_qkv_rope_supported(int dtype, int M, int N, int K, int head_dim);
// q_out[M][Hq * head_dim] = rotated Q; rotated K and V go to the rows' page slots.  Same bits as
// the float-output GEMM followed by launch_rope_write.
void launch_gemm_mfma_qkv_rope(hipStream_t s, const void* A, const void* Wqkv, void* q_out, int M,
                               int N, int K, const RopeEpilogue& rope);
void launch_rope_write(hipStream_t s, int dtype, const float* qkv, const int32_t* pos,
                       const int32_t* slot, const float2* cos_sin, void* q_out, void* pool_layer,
                       int T, int n_q_heads, KvGeom g);
void launch_attention_simple(hipStream_t s, int dtype, const void* q, void* out,
                             const void* pool_layer, const AttnWork* work, int n_work,
                             const int32_t* page_tables, int n_q_heads, KvGeom g);
bool attention_mfma_supported(int dtype, int head_dim, int n_q_heads, int n_kv_heads);
// query heads one workgroup of the MFMA attention kernel works on (they share the K/V tiles)
int attention_mfma_heads_per_block(int n_q_heads, int n_kv_heads);
void launch_attention_mfma(hipStream_t s, const void* q, void* out, float* part_buf,
                           const void* pool_layer, const AttnWork* work, int n_work,
                           const AttnCombine* groups, int n_groups, const int32_t* page_tables,
                           int n_q_heads, KvGeom g);
// pinned host memory -> pages, directly: job.staging_off is the host ADDRESS of the run's first
// page; block_first counts units of PAGE_LOAD_UNIT_VECS 16-byte vectors of the run (a run of p
// pages has ceil(p * page_bytes / 16 / PAGE_LOAD_UNIT_VECS) units); n_workgroups resident
// workgroups walk the units
constexpr int PAGE_LOAD_UNIT_VECS = 4096;
void launch_page_load(hipStream_t s, int dtype, void* pool, const PageJob* jobs, int n_jobs,
                      int n_units, int n_workgroups, const int32_t* page_tables, KvGeom g);
// out[T][d] = h (+ dl when non-null): the residual stream of packed rows entering a layer (d % 4 == 0)
void launch_residual_rows(hipStream_t s, float* out, const float* h, const float* dl, int T, int d);
// out[j][d] = h[idx[j]] (+ dl[idx[j]] when non-null) for j < n; a listed row is skipped unless it
// lies in [a0, a1) or [b0, b1) (d % 4 == 0)
void launch_residual_gather(hipStream_t s, float* out, const float* h, const float* dl, const int32_t* idx,
                            int n, int d, int a0, int a1, int b0, int b1);
// copy-stream pacing: mark stores the wall clock at *t0 (device, 8 bytes), wait holds the stream
// until `ticks` wall-clock ticks have passed since the mark (bounded spin)
void launch_pace_mark(hipStream_t s, void* t0);
void launch_pace_wait(hipStream_t s, const void* t0, unsigned long long ticks);
// pages -> pinned host memory, directly (whole pages; job fields as for launch_page_load)
void launch_page_store(hipStream_t s, int dtype, const void* pool, const PageJob* jobs, int n_jobs,
                       int n_units, int n_workgroups, const int32_t* page_tables, KvGeom g);
// staging -> pages (to_pages = true) or pages -> staging (false; zero-fills unused slots)
void launch_page_move(hipStream_t s, int dtype, void* staging, void* pool, const PageJob* jobs,
                      int n_jobs, int n_blocks, const int32_t* page_tables, KvGeom g, bool to_pages);

}  // namespace cf
