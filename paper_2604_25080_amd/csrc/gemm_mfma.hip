// bf16 GEMM on CDNA4 matrix cores for the linear layers of recompute:
//   acc[M,N] = A[M,K] * W[N,K]^T   (both operands K-contiguous, float accumulate)
// with the layer's epilogue fused: float store (QKV), float residual add
// (O-proj, down-proj), bf16 store, or SiLU(gate)*up -> bf16 (gate/up pair).
//
// Tiling: 256x256 block tile, 4 wavefronts (2x2), each a 128x128 wave tile =
// 4x4 MFMA 32x32x16 fragments (256 accumulator registers per lane).  K is
// walked in steps of BK = 64 through a double-buffered LDS tile; the next
// K-step is fetched from global memory into registers while the current one
// is multiplied, then written to the other LDS buffer.  LDS rows are
// K-contiguous (128 bytes) with the 16-byte chunk index XOR-swizzled by the
// row so that the 16-byte fragment reads of a wavefront spread over all banks.
// Workgroups are renumbered so that the 32 workgroups resident on one XCD
// (one L2) cover an 8x4 patch of tiles.
#include "kernels.h"
#include "cacheflow.h"

namespace cf {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int NCH = BK / 8;               // 16-byte chunks per LDS row
constexpr int ROW_BYTES = BK * 2;
constexpr int TILE_BYTES = BM * ROW_BYTES;  // one operand tile
constexpr int STAGE_BYTES = 2 * TILE_BYTES;
constexpr int N_STAGES = 2;
constexpr int LOADS = BM * NCH / 256;     // 16-byte loads per thread per operand tile (8)

__device__ __forceinline__ int swz(int row) { return (row >> 1) & (NCH - 1); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float v) {
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int EPI>
__global__ void __launch_bounds__(256)
gemm_mfma_kernel(const bf16* __restrict__ A, const bf16* __restrict__ W,
                 const bf16* __restrict__ W2, float* __restrict__ Cf, bf16* __restrict__ Dt, int M,
                 int N, int K, int tiles_m, int tiles_n) {
    extern __shared__ __align__(16) char smem[];
    constexpr bool SILU = (EPI == EPI_SILU_MUL);
    constexpr int BN_OUT = SILU ? BN / 2 : BN;    // output columns per block

    // ---- workgroup -> tile: XCD-contiguous renumbering, then 8-row groups
    int nb = tiles_m * tiles_n;
    int bid = blockIdx.x;
    int per = nb >> 3, rem = nb & 7, xcd = bid & 7, idx = bid >> 3;
    int pid = xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
    constexpr int GM = 8;
    int in_group = GM * tiles_n;
    int first_m = (pid / in_group) * GM;
    int gsz = min(tiles_m - first_m, GM);
    int tile_m = first_m + (pid % in_group) % gsz;
    int tile_n = (pid % in_group) / gsz;
    int m0 = tile_m * BM, n0 = tile_n * BN_OUT;

    int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int wm = wave >> 1, wn = wave & 1;

    // ---- global -> register -> LDS loader: thread handles chunk (tid % NCH) of rows
    // tid / NCH + j * (256 / NCH), j = 0..LOADS-1, for both operand tiles
    int ld_chunk = tid % NCH, ld_row0 = tid / NCH;
    const bf16* a_src[LOADS];
    const bf16* b_src[LOADS];
    int lds_off[LOADS];
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        int r = ld_row0 + j * (256 / NCH);
        int gm = min(m0 + r, M - 1);
        a_src[j] = A + (int64_t)gm * K + ld_chunk * 8;
        if (SILU) {
            int gn = min(n0 + (r & 127), N - 1);
            b_src[j] = (r < 128 ? W : W2) + (int64_t)gn * K + ld_chunk * 8;
        } else {
            int gn = min(n0 + r, N - 1);
            b_src[j] = W + (int64_t)gn * K + ld_chunk * 8;
        }
        lds_off[j] = r * ROW_BYTES + ((ld_chunk ^ swz(r)) << 4);
    }

    // ---- fragment read offsets: lane reads row (lane % 32) of a 32-row fragment,
    // chunk 2*kk + lane/32 (swizzled)
    int frow = lane & 31, fhalf = lane >> 5;
    int fswz = swz(frow);                   // fragment bases are multiples of 32 rows
    int a_base = (wm * 128 + frow) * ROW_BYTES;
    int b_row[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int r = SILU ? ((j < 2) ? wn * 64 + j * 32 : 128 + wn * 64 + (j - 2) * 32) : wn * 128 + j * 32;
        b_row[j] = (r + frow) * ROW_BYTES;
    }

    f32x16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    uint4 ra[LOADS], rb[LOADS];
    int nk = K / BK;
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        ra[j] = *reinterpret_cast<const uint4*>(a_src[j]);
        rb[j] = *reinterpret_cast<const uint4*>(b_src[j]);
    }
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        *reinterpret_cast<uint4*>(smem + lds_off[j]) = ra[j];
        *reinterpret_cast<uint4*>(smem + TILE_BYTES + lds_off[j]) = rb[j];
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        char* cur = smem + (kt & 1) * STAGE_BYTES;
        char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
        // fetch the next K-step (the last iteration refetches its own step; unused)
        int koff = min(kt + 1, nk - 1) * BK;
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            ra[j] = *reinterpret_cast<const uint4*>(a_src[j] + koff);
            rb[j] = *reinterpret_cast<const uint4*>(b_src[j] + koff);
        }
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            int coff = ((2 * kk + fhalf) ^ fswz) << 4;
            uint4 fa[4], fb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                fa[i] = *reinterpret_cast<const uint4*>(cur + a_base + i * 32 * ROW_BYTES + coff);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                fb[j] = *reinterpret_cast<const uint4*>(cur + TILE_BYTES + b_row[j] + coff);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8_t, fa[i]), __builtin_bit_cast(bf16x8_t, fb[j]),
                        acc[i][j], 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            *reinterpret_cast<uint4*>(nxt + lds_off[j]) = ra[j];
            *reinterpret_cast<uint4*>(nxt + TILE_BYTES + lds_off[j]) = rb[j];
        }
        __syncthreads();
    }

    // ---- epilogue.  Fragment (i,j), register r: row = 32i + 8(r/4) + 4(lane/32) + r%4,
    // column = 32j + lane%32.
    int col_l = lane & 31;
    int row_l = 4 * (lane >> 5);
    if (SILU) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                int gn = n0 + wn * 64 + j * 32 + col_l;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int gm = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + row_l + (r & 3);
                    if (gm < M && gn < N) {
                        float g = acc[i][j][r], u = acc[i][j + 2][r];
                        float v = g / (1.0f + __expf(-g)) * u;
                        Dt[(int64_t)gm * N + gn].x = f32_to_bf16_bits(v);
                    }
                }
            }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int gn = n0 + wn * 128 + j * 32 + col_l;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int gm = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + row_l + (r & 3);
                    if (gm < M && gn < N) {
                        int64_t o = (int64_t)gm * N + gn;
                        float v = acc[i][j][r];
                        if (EPI == EPI_STORE_F32) Cf[o] = v;
                        else if (EPI == EPI_ADD_F32) Cf[o] += v;
                        else Dt[o].x = f32_to_bf16_bits(v);
                    }
                }
            }
    }
}

template <int EPI>
void launch(hipStream_t s, const void* A, const void* W, const void* W2, float* Cf, void* Dt, int M,
            int N, int K) {
    constexpr int BN_OUT = (EPI == EPI_SILU_MUL) ? BN / 2 : BN;
    int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN_OUT - 1) / BN_OUT;
    static bool configured = false;
    auto kern = gemm_mfma_kernel<EPI>;
    if (!configured) {
        (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                  N_STAGES * STAGE_BYTES);
        configured = true;
    }
    kern<<<tiles_m * tiles_n, 256, N_STAGES * STAGE_BYTES, s>>>(
        (const bf16*)A, (const bf16*)W, (const bf16*)W2, Cf, (bf16*)Dt, M, N, K, tiles_m, tiles_n);
}

}  // namespace

bool gemm_mfma_supported(int dtype, int M, int N, int K, int epi) {
    (void)epi;
    return dtype == CF_BF16 && M > 0 && N > 0 && K >= BK && K % BK == 0;
}

void launch_gemm_mfma(hipStream_t s, const void* A, const void* W, const void* W2, float* Cf,
                      void* Dt, int M, int N, int K, int epi) {
    switch (epi) {
        case EPI_STORE_F32: launch<EPI_STORE_F32>(s, A, W, W2, Cf, Dt, M, N, K); break;
        case EPI_ADD_F32: launch<EPI_ADD_F32>(s, A, W, W2, Cf, Dt, M, N, K); break;
        case EPI_STORE_T: launch<EPI_STORE_T>(s, A, W, W2, Cf, Dt, M, N, K); break;
        default: launch<EPI_SILU_MUL>(s, A, W, W2, Cf, Dt, M, N, K); break;
    }
}

}  // namespace cf
