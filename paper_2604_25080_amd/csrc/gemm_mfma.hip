// bf16 GEMM on CDNA4 matrix cores for the linear layers of recompute:
//   acc[M,N] = A[M,K] * W[N,K]^T   (both operands K-contiguous, float accumulate)
// with the layer's epilogue fused: float store (QKV), float residual add
// (O-proj, down-proj), bf16 store, SiLU(gate)*up -> bf16 (gate/up pair), or -- for the QKV
// projection on the big tile -- RoPE on the accumulators with Q stored as bf16 and K/V written
// straight into their page slots.
//
// Tiling: 256x256 block tile, 4 wavefronts (2x2), each a 128x128 wave tile =
// 4x4 MFMA 32x32x16 fragments (256 accumulator registers per lane); problems
// too small to fill the chip with such tiles use 128x128 or 64x64 block tiles instead (the
// latter with four K-steps of operands in flight per workgroup).  K is
// walked in steps of BK = 64 through a double-buffered LDS tile; the next
// K-step is fetched from global memory into registers while the current one
// is multiplied, then written to the other LDS buffer.  LDS rows are
// K-contiguous (128 bytes) with the 16-byte chunk index XOR-swizzled by the
// row so that the 16-byte fragment reads of a wavefront spread over all banks.
// Workgroups are renumbered so that the 32 workgroups resident on one XCD
// (one L2) cover an 8x4 patch of tiles.
#include "kernels.h"
#include "rope.h"
#include "cacheflow.h"

namespace cf {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;   // native 16-byte register vector

namespace {

constexpr int BK = 64;
constexpr int NCH = BK / 8;               // 16-byte chunks per LDS row
constexpr int ROW_BYTES = BK * 2;
constexpr int N_STAGES = 2;

__device__ __forceinline__ int swz(int row) { return (row >> 1) & (NCH - 1); }

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
// two floats -> two bf16 (round to nearest even), low half = a
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float v) {
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// BM x BN block tile (256x256 for large problems, 128x128 when that would leave CUs idle);
// the 4 wavefronts form a 2x2 grid of (BM/2)x(BN/2) wave tiles.
// `bid` of `nb` workgroups walk the tiles_m x tiles_n tiles whose origin is (m_off, n_off); M, N
// are the bounds of the whole matrix.
template <int EPI, int BM, int BN, int NW>
__device__ __forceinline__ void
gemm_mfma_body(char* smem, const bf16* __restrict__ A, const bf16* __restrict__ W,
               const bf16* __restrict__ W2, float* __restrict__ Cf, bf16* __restrict__ Dt, int M,
               int N, int K, int tiles_m, int tiles_n, int m_off, int n_off, int bid, int nb,
               const RopeEpilogue& rope) {
    constexpr bool SILU = (EPI == EPI_SILU_MUL);
    constexpr bool ROPE = (EPI == EPI_QKV_ROPE128 || EPI == EPI_QKV_ROPE64);
    // 16-bit outputs: the MFMAs take the W fragment as their first operand, which leaves the
    // TRANSPOSED product in the accumulators (see the epilogue)
    constexpr bool SWAP = (EPI == EPI_SILU_MUL || EPI == EPI_STORE_T || ROPE);
    constexpr int BN_OUT = SILU ? BN / 2 : BN;    // output columns per block
    constexpr int WGN = NW / 2;                   // wavefront grid: 2 x WGN
    constexpr int NT = 64 * NW;                   // threads
    constexpr int WM = BM / 2, WN = BN / WGN;     // wave tile
    constexpr int FM = WM / 32, FN = WN / 32;     // MFMA fragments per wave tile
    constexpr int A_TILE = BM * ROW_BYTES, B_TILE = BN * ROW_BYTES;
    constexpr int STAGE_BYTES = A_TILE + B_TILE;
    constexpr int LA = BM * NCH / NT, LB = BN * NCH / NT;     // 16-byte loads per thread

    // ---- workgroup -> tile: XCD-contiguous renumbering, then 8-row groups
    int per = nb >> 3, rem = nb & 7, xcd = bid & 7, idx = bid >> 3;
    int pid = xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
    constexpr int GM = 8;             // = GROUP_M of the launcher
    int in_group = GM * tiles_n;
    int first_m = (pid / in_group) * GM;
    int gsz = min(tiles_m - first_m, GM);
    int tile_m = first_m + (pid % in_group) % gsz;
    int tile_n = (pid % in_group) / gsz;
    int m0 = m_off + tile_m * BM, n0 = n_off + tile_n * BN_OUT;
    constexpr bool BIG = (BM == 256 && NW == 4);
    if constexpr (BIG) {
        // Edge tiles are shifted back inside the matrix (the host guarantees M >= BM and
        // N >= BN_OUT); the overlap is recomputed and stored twice with identical values.
        // This keeps every row of a tile a fixed stride apart, so the loader needs one
        // per-thread offset instead of one per row.
        m0 = min(m0, M - BM);
        n0 = min(n0, N - BN_OUT);
    }

    int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int wm = wave / WGN, wn = wave % WGN;

    // ---- global -> register -> LDS loader: thread handles chunk (tid % NCH) of rows
    // tid / NCH + j * (256 / NCH), j = 0..LOADS-1, for both operand tiles
    // Rows come from wave-uniform base pointers plus small per-thread element offsets.
    int ld_chunk = tid % NCH, ld_row0 = tid / NCH;
    const bf16* a_tile = A + (int64_t)m0 * K;
    const bf16* w_tile = W + (int64_t)n0 * K;
    const bf16* w2_tile = SILU ? W2 + (int64_t)n0 * K : nullptr;
    int a_off[LA], b_off[LB];
    int a_lds[LA], b_lds[LB];
#pragma unroll
    for (int j = 0; j < LA; ++j) {
        int r = ld_row0 + j * (NT / NCH);
        a_off[j] = (min(m0 + r, M - 1) - m0) * K + ld_chunk * 8;
        a_lds[j] = r * ROW_BYTES + ((ld_chunk ^ swz(r)) << 4);
    }
#pragma unroll
    for (int j = 0; j < LB; ++j) {
        int r = ld_row0 + j * (NT / NCH);
        // gate/up pair: tile rows [0, BN/2) are gate rows, [BN/2, BN) the same rows of up
        int rn = SILU ? r % (BN / 2) : r;
        b_off[j] = (min(n0 + rn, N - 1) - n0) * K + ld_chunk * 8;
        b_lds[j] = A_TILE + r * ROW_BYTES + ((ld_chunk ^ swz(r)) << 4);
    }
#define CF_B_BASE(j) ((SILU && (j) >= LB / 2) ? w2_tile : w_tile)

    // ---- fragment read offsets: lane reads row (lane % 32) of a 32-row fragment,
    // chunk 2*kk + lane/32 (swizzled)
    int frow = lane & 31, fhalf = lane >> 5;
    int fswz = swz(frow);                   // fragment bases are multiples of 32 rows
    int a_base = (wm * WM + frow) * ROW_BYTES;
    int b_row[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        // gate/up pair: the first FN/2 fragments are gate columns, the rest the same columns of up
        int r = SILU ? ((j < FN / 2) ? wn * (WN / 2) + j * 32
                                     : BN / 2 + wn * (WN / 2) + (j - FN / 2) * 32)
                     : wn * WN + j * 32;
        b_row[j] = A_TILE + (r + frow) * ROW_BYTES;
    }

    f32x16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Software pipeline over K-steps of 64 (four 16-deep MFMA sub-steps each).  Tile kt is
    // multiplied out of LDS buffer kt&1; fragments are double-buffered in registers and always
    // read one sub-step ahead of the MFMAs that use them; one barrier per K-step, placed after
    // sub-step 2, when every wave already holds its sub-step-3 fragments in registers.
    int nk = K / BK;
#define CF_FETCH_A(KT, RA)                                                                    \
    {                                                                                         \
        int koff_ = min((KT), nk - 1) * BK;   /* past the end: refetch the last step, unused */ \
        _Pragma("unroll") for (int j = 0; j < LA; ++j)                                        \
            RA[j] = *reinterpret_cast<const u32x4_t*>(a_tile + koff_ + a_off[j]);             \
    }
#define CF_FETCH_B(KT, RB)                                                                    \
    {                                                                                         \
        int koff_ = min((KT), nk - 1) * BK;                                                   \
        _Pragma("unroll") for (int j = 0; j < LB; ++j)                                        \
            RB[j] = *reinterpret_cast<const u32x4_t*>(CF_B_BASE(j) + koff_ + b_off[j]);       \
    }
#define CF_STASH_A(BUF, RA)                                                                   \
    _Pragma("unroll") for (int j = 0; j < LA; ++j) *reinterpret_cast<u32x4_t*>((BUF) + a_lds[j]) = RA[j];
#define CF_STASH_B(BUF, RB)                                                                   \
    _Pragma("unroll") for (int j = 0; j < LB; ++j) *reinterpret_cast<u32x4_t*>((BUF) + b_lds[j]) = RB[j];
#define CF_READ_FRAGS(FA, FB, BUF, KK)                                                        \
    {                                                                                         \
        const char* buf_ = (BUF);                                                             \
        int coff_ = ((2 * (KK) + fhalf) ^ fswz) << 4;                                         \
        _Pragma("unroll") for (int i = 0; i < FM; ++i)                                        \
            FA[i] = *reinterpret_cast<const u32x4_t*>(buf_ + a_base + i * 32 * ROW_BYTES + coff_); \
        _Pragma("unroll") for (int j = 0; j < FN; ++j)                                        \
            FB[j] = *reinterpret_cast<const u32x4_t*>(buf_ + b_row[j] + coff_);               \
    }
#define CF_MFMA(FA, FB)                                                                       \
    _Pragma("unroll") for (int i = 0; i < FM; ++i)                                            \
        _Pragma("unroll") for (int j = 0; j < FN; ++j)                                        \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                              \
                __builtin_bit_cast(bf16x8_t, SWAP ? FB[j] : FA[i]),                           \
                __builtin_bit_cast(bf16x8_t, SWAP ? FA[i] : FB[j]), acc[i][j], 0, 0, 0);

    u32x4_t fa0[FM], fb0[FN], fa1[FM], fb1[FN];
    if constexpr (BIG) {
        // loader of the big tile: row j of a thread is 32 rows below row j-1, in global memory
        // (wave-uniform base + one 32-bit per-thread byte offset) and in LDS (immediate offsets)
        const unsigned a_voff = (unsigned)((ld_row0 * K + ld_chunk * 8) * 2);
        const unsigned b_voff = a_voff;
        const int lds0 = ld_row0 * ROW_BYTES + ((ld_chunk ^ swz(ld_row0)) << 4);
        const int64_t row_stride_b = (int64_t)(NT / NCH) * K * 2;          // bytes between loader rows
#define CF_BIG_FETCH_A(KT, RA)                                                                \
        {                                                                                     \
            const char* base_ = (const char*)a_tile + (int64_t)min((KT), nk - 1) * (BK * 2);  \
            _Pragma("unroll") for (int j = 0; j < LA; ++j)                                    \
                RA[j] = *reinterpret_cast<const u32x4_t*>(base_ + j * row_stride_b + a_voff); \
        }
#define CF_BIG_FETCH_B(KT, RB)                                                                \
        {                                                                                     \
            int64_t koffb_ = (int64_t)min((KT), nk - 1) * (BK * 2);                           \
            _Pragma("unroll") for (int j = 0; j < LB; ++j) {                                  \
                /* gate/up pair: loader rows [0, BN/2) come from W, [BN/2, BN) from W2 */     \
                const char* base_ = (const char*)CF_B_BASE(j) + koffb_ +                      \
                                    (SILU ? (j % (LB / 2)) : j) * row_stride_b;               \
                RB[j] = *reinterpret_cast<const u32x4_t*>(base_ + b_voff);                    \
            }                                                                                 \
        }
#define CF_BIG_STASH_A(BUF, RA)                                                               \
        _Pragma("unroll") for (int j = 0; j < LA; ++j)                                        \
            *reinterpret_cast<u32x4_t*>((BUF) + lds0 + j * (NT / NCH) * ROW_BYTES) = RA[j];
#define CF_BIG_STASH_B(BUF, RB)                                                               \
        _Pragma("unroll") for (int j = 0; j < LB; ++j)                                        \
            *reinterpret_cast<u32x4_t*>((BUF) + A_TILE + lds0 + j * (NT / NCH) * ROW_BYTES) = RB[j];
        // 16 MFMAs per sub-step and exactly 16 memory instructions beside them: 8 fragment reads
        // plus 8 of {LDS fill of the A half, global fetch of the A half, LDS fill of the B half,
        // global fetch of the B half} -- never more than one memory instruction per MFMA, which
        // is what keeps the matrix pipe fed (two per MFMA cost ~25 %).  Two register sets hold
        // tiles in flight: the set written to LDS in iteration kt was fetched in iteration kt-2,
        // so two full K-steps of MFMAs cover the memory latency.  The host guarantees an even
        // number of K-steps for this variant.
        // Order hints (masks: 0x8 MFMA, 0x20 VMEM read, 0x100 LDS read, 0x200 LDS write); the
        // builtin wants literal arguments.
#define CF_GROUP(MASK, SIZE) __builtin_amdgcn_sched_group_barrier((MASK), (SIZE), 0)
#define CF_REP4(X) X X X X
#define CF_REP8(X) CF_REP4(X) CF_REP4(X)
#define CF_SECTION(OTHER)                                                                     \
        CF_REP8(CF_GROUP(0x8, 1); CF_GROUP(0x100, 1);) CF_REP8(CF_GROUP(0x8, 1); CF_GROUP((OTHER), 1);) \
        __builtin_amdgcn_sched_barrier(0);
#define CF_KSTEP(KT, RA, RB)                                                                  \
        {                                                                                     \
            char* cur = smem + ((KT) & 1) * STAGE_BYTES;                                      \
            char* nxt = smem + (((KT) + 1) & 1) * STAGE_BYTES;                                \
            CF_READ_FRAGS(fa1, fb1, cur, 1); CF_BIG_STASH_A(nxt, RA); CF_MFMA(fa0, fb0); CF_SECTION(0x200) \
            CF_READ_FRAGS(fa0, fb0, cur, 2); CF_BIG_FETCH_A((KT) + 3, RA); CF_MFMA(fa1, fb1); CF_SECTION(0x20) \
            CF_READ_FRAGS(fa1, fb1, cur, 3); CF_BIG_STASH_B(nxt, RB); CF_MFMA(fa0, fb0); CF_SECTION(0x200) \
            __syncthreads();                                                                  \
            CF_READ_FRAGS(fa0, fb0, nxt, 0); CF_BIG_FETCH_B((KT) + 3, RB); CF_MFMA(fa1, fb1); CF_SECTION(0x20) \
        }
        u32x4_t ra0[LA], rb0[LB], ra1[LA], rb1[LB];
        CF_BIG_FETCH_A(0, ra0); CF_BIG_FETCH_B(0, rb0);
        CF_BIG_STASH_A(smem, ra0); CF_BIG_STASH_B(smem, rb0);
        CF_BIG_FETCH_A(1, ra1); CF_BIG_FETCH_B(1, rb1);
        CF_BIG_FETCH_A(2, ra0); CF_BIG_FETCH_B(2, rb0);
        __syncthreads();
        CF_READ_FRAGS(fa0, fb0, smem, 0);
        for (int kt = 0; kt < nk; kt += 2) {
            CF_KSTEP(kt, ra1, rb1);
            CF_KSTEP(kt + 1, ra0, rb0);
        }
#undef CF_GROUP
#undef CF_REP4
#undef CF_REP8
#undef CF_SECTION
#undef CF_KSTEP
#undef CF_BIG_FETCH_A
#undef CF_BIG_FETCH_B
#undef CF_BIG_STASH_A
#undef CF_BIG_STASH_B
    } else if (BM == 64 && (nk & 3) == 0) {
        // The 64x64 tile is for launches with few rows against long K (the new turn of a small
        // batch, a tensor-parallel shard's narrow projections): few workgroups, each walking K
        // alone, so what counts is how many K-steps a workgroup has in flight.  Four register
        // sets hold tiles kt+1 .. kt+4 (tile t lives in set t % 4): the set written to LDS in
        // step kt was requested four steps earlier and is refilled with tile kt+5 right away
        // (eight sets measured no faster).  Same MFMA order along K as every other tile shape,
        // so the same bits.
        u32x4_t ra0[LA], rb0[LB], ra1[LA], rb1[LB], ra2[LA], rb2[LB], ra3[LA], rb3[LB];
        CF_FETCH_A(0, ra0); CF_FETCH_B(0, rb0);
        CF_FETCH_A(1, ra1); CF_FETCH_B(1, rb1);
        CF_FETCH_A(2, ra2); CF_FETCH_B(2, rb2);
        CF_FETCH_A(3, ra3); CF_FETCH_B(3, rb3);
        CF_STASH_A(smem, ra0); CF_STASH_B(smem, rb0);
        CF_FETCH_A(4, ra0); CF_FETCH_B(4, rb0);
        __syncthreads();
        CF_READ_FRAGS(fa0, fb0, smem, 0);
#define CF_RSTEP(KT, RA, RB)                                                                  \
        {                                                                                     \
            char* cur = smem + ((KT) & 1) * STAGE_BYTES;                                      \
            char* nxt = smem + (((KT) + 1) & 1) * STAGE_BYTES;                                \
            CF_READ_FRAGS(fa1, fb1, cur, 1);                                                  \
            CF_MFMA(fa0, fb0);                                                                \
            CF_READ_FRAGS(fa0, fb0, cur, 2);                                                  \
            CF_MFMA(fa1, fb1);                                                                \
            CF_READ_FRAGS(fa1, fb1, cur, 3);                                                  \
            CF_STASH_A(nxt, RA); CF_STASH_B(nxt, RB);          /* tile KT+1 */                \
            CF_MFMA(fa0, fb0);                                                                \
            __syncthreads();                                                                  \
            CF_READ_FRAGS(fa0, fb0, nxt, 0);                                                  \
            CF_FETCH_A((KT) + 5, RA); CF_FETCH_B((KT) + 5, RB);                               \
            CF_MFMA(fa1, fb1);                                                                \
        }
        for (int kt = 0; kt < nk; kt += 4) {
            CF_RSTEP(kt, ra1, rb1)
            CF_RSTEP(kt + 1, ra2, rb2)
            CF_RSTEP(kt + 2, ra3, rb3)
            CF_RSTEP(kt + 3, ra0, rb0)
        }
#undef CF_RSTEP
    } else {
        // Smaller tiles: tile kt+1 (fetched during the previous iteration) is written to the other
        // buffer during sub-step 2 and tile kt+2 fetched during sub-step 3; instruction order is
        // left to the compiler, which does better than explicit hints at 4 MFMAs per sub-step.
        u32x4_t ra[LA], rb[LB];
        CF_FETCH_A(0, ra); CF_FETCH_B(0, rb);
        CF_STASH_A(smem, ra); CF_STASH_B(smem, rb);
        CF_FETCH_A(1, ra); CF_FETCH_B(1, rb);
        __syncthreads();
        CF_READ_FRAGS(fa0, fb0, smem, 0);
        for (int kt = 0; kt < nk; ++kt) {
            char* cur = smem + (kt & 1) * STAGE_BYTES;
            char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
            CF_READ_FRAGS(fa1, fb1, cur, 1);
            CF_MFMA(fa0, fb0);
            CF_READ_FRAGS(fa0, fb0, cur, 2);
            CF_MFMA(fa1, fb1);
            CF_READ_FRAGS(fa1, fb1, cur, 3);
            CF_STASH_A(nxt, ra); CF_STASH_B(nxt, rb);
            CF_MFMA(fa0, fb0);
            __syncthreads();
            CF_READ_FRAGS(fa0, fb0, nxt, 0);
            CF_FETCH_A(kt + 2, ra); CF_FETCH_B(kt + 2, rb);
            CF_MFMA(fa1, fb1);
        }
    }
#undef CF_FETCH_A
#undef CF_FETCH_B
#undef CF_STASH_A
#undef CF_STASH_B
#undef CF_READ_FRAGS
#undef CF_MFMA

#undef CF_B_BASE
    // ---- epilogue.
    // float outputs: fragment (i,j), register r = row 32i + 8(r/4) + 4(lane/32) + r%4, column
    // 32j + lane%32: one store instruction writes two rows of 32 consecutive floats (whole
    // 128-byte lines, which is what the memory system likes best for 4-byte elements).
    // 16-bit outputs (SWAP): the accumulators hold the transposed product, register r = output
    // row 32i + lane%32, column 32j + 8(r/4) + 4(lane/32) + r%4, so a lane owns runs of four
    // consecutive columns of one row and stores them as one 8-byte vector -- a quarter of the
    // store instructions and address arithmetic of a column-per-lane layout, whose 2-byte stores
    // would fill only half a line per instruction anyway.
    // The big tile lies wholly inside the matrix (shifted back at the edges): no bounds tests.
    if constexpr (!SWAP) {
        const int col_l = lane & 31, row_l = 4 * (lane >> 5);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int gn = n0 + wn * WN + j * 32 + col_l;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int gm = m0 + wm * WM + i * 32 + 8 * (r >> 2) + row_l + (r & 3);
                    if (BIG || (gm < M && gn < N)) {
                        const int64_t o = (int64_t)gm * N + gn;
                        if (EPI == EPI_STORE_F32) Cf[o] = acc[i][j][r];
                        else Cf[o] += acc[i][j][r];
                    }
                }
            }
    } else if constexpr (ROPE) {
        // QKV projection (big tile only, N a multiple of the tile): a wave tile spans whole
        // heads, and both elements (j, j + head_dim/2) of a rotation pair sit in the same lane,
        // HALF_F fragments apart.  Per row the lane looks up the position (angle) and the page
        // slot; whether a head is Q, K or V is the same for the whole wavefront.
        static_assert(BIG, "the fused QKV epilogue exists for the 256x256 tile only");
        constexpr int HD = (EPI == EPI_QKV_ROPE128) ? 128 : 64;
        constexpr int HALF_F = HD / 64;               // fragments per half head
        static_assert(WN % HD == 0 && FN % (2 * HALF_F) == 0, "wave tile must span whole heads");
        const int row_l = lane & 31, col_l = 4 * (lane >> 5);
        const int nq = rope.n_q_heads * HD, nkv = rope.g.n_kv_heads * HD;
        bf16* pool = (bf16*)rope.pool_layer;
        // Loads first, and ahead of the stores they could alias with as far as the compiler
        // knows: the rows' positions and slots up front, then the angles of row group i + 1
        // while row group i is rotated and stored (one wavefront per SIMD: nothing else hides
        // the latency of a load that waits behind a store).
        int rpos[FM], rslot[FM];
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const int gm = m0 + wm * WM + i * 32 + row_l;
            rpos[i] = rope.pos[gm];
            rslot[i] = rope.slot[gm];
        }
        constexpr int NTAB = HALF_F * 8;              // float4 loads per row: 16 * HALF_F (cos, sin) pairs
        constexpr int FH = 2 * HALF_F;                // fragments per head
#define CF_LOAD_ANGLES(I, T)                                                                  \
        {                                                                                     \
            const float2* cs_ = rope.cos_sin + (int64_t)rpos[I] * (HD / 2) + col_l;           \
            _Pragma("unroll") for (int u = 0; u < HALF_F * 4; ++u) {                          \
                T[2 * u] = *reinterpret_cast<const float4*>(cs_ + 8 * u);                     \
                T[2 * u + 1] = *reinterpret_cast<const float4*>(cs_ + 8 * u + 2);             \
            }                                                                                 \
        }
        // Head by head; Q, K or V is decided once per head, outside the row loop, so that each
        // branch is straight-line code over the four row groups.
#pragma unroll
        for (int hh = 0; hh < WN / HD; ++hh) {
            // first column of this head (the same for every lane: kept in a scalar register)
            const int hc = __builtin_amdgcn_readfirstlane(n0 + wn * WN + hh * HD);
            if (hc < nq + nkv) {
                float4 tab[2][NTAB];
                CF_LOAD_ANGLES(0, tab[0]);
#pragma unroll
                for (int i = 0; i < FM; ++i) {
                    if (i + 1 < FM) CF_LOAD_ANGLES(i + 1, tab[(i + 1) & 1]);
                    const float4* tb = tab[i & 1];
                    const int gm = m0 + wm * WM + i * 32 + row_l;
                    // Q row of the packed query buffer, or the K row [head][slot][HD] of the page
                    bf16* dst = hc < nq ? Dt + (int64_t)gm * nq + hc
                                        : pool + (int64_t)(rslot[i] / CF_PAGE_TOKENS) * rope.g.page_elems +
                                              ((int64_t)((hc - nq) / HD) * CF_PAGE_TOKENS + rslot[i] % CF_PAGE_TOKENS) * HD;
#pragma unroll
                    for (int jj = 0; jj < HALF_F; ++jj)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int cj = jj * 32 + 8 * q + col_l;        // pair index, multiple of 4
                            const float4 t0 = tb[2 * (jj * 4 + q)], t1 = tb[2 * (jj * 4 + q) + 1];
                            const float2 cc[4] = {{t0.x, t0.y}, {t0.z, t0.w}, {t1.x, t1.y}, {t1.z, t1.w}};
                            float y1[4], y2[4];
#pragma unroll
                            for (int t = 0; t < 4; ++t)
                                rope_rotate(acc[i][hh * FH + jj][4 * q + t],
                                            acc[i][hh * FH + HALF_F + jj][4 * q + t], cc[t], y1[t], y2[t]);
                            uint2 lo, hi;
                            lo.x = pack_bf16x2(y1[0], y1[1]); lo.y = pack_bf16x2(y1[2], y1[3]);
                            hi.x = pack_bf16x2(y2[0], y2[1]); hi.y = pack_bf16x2(y2[2], y2[3]);
                            *reinterpret_cast<uint2*>(dst + cj) = lo;
                            *reinterpret_cast<uint2*>(dst + cj + HD / 2) = hi;
                        }
                }
            } else {
                // V, stored transposed in the page: [head][HD][slot]; the 32 rows of a fragment
                // are mostly consecutive slots, so a store instruction still fills 32-byte runs
#pragma unroll
                for (int i = 0; i < FM; ++i) {
                    bf16* dst = pool + (int64_t)(rslot[i] / CF_PAGE_TOKENS) * rope.g.page_elems +
                                (int64_t)rope.g.n_kv_heads * CF_PAGE_TOKENS * HD +
                                (int64_t)((hc - nq - nkv) / HD) * HD * CF_PAGE_TOKENS + rslot[i] % CF_PAGE_TOKENS;
#pragma unroll
                    for (int j = 0; j < FH; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int col = j * 32 + 8 * (r >> 2) + col_l + (r & 3);
                            dst[col * CF_PAGE_TOKENS].x = f32_to_bf16_bits(acc[i][hh * FH + j][r]);
                        }
                }
            }
        }
#undef CF_LOAD_ANGLES
    } else {
        const int row_l = lane & 31, col_l = 4 * (lane >> 5);
        const bool vec_ok = (N & 3) == 0;             // row starts stay 8-byte aligned
        constexpr int FN_OUT = SILU ? FN / 2 : FN;
        constexpr int WN_OUT = SILU ? WN / 2 : WN;
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const int gm = m0 + wm * WM + i * 32 + row_l;
            if (!BIG && gm >= M) continue;
#pragma unroll
            for (int j = 0; j < FN_OUT; ++j) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int gn = n0 + wn * WN_OUT + j * 32 + 8 * q + col_l;
                    const int64_t o = (int64_t)gm * N + gn;
                    float v[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        float g = acc[i][j][4 * q + t];
                        if (SILU) {
                            // silu(g) * u with the hardware exp2 and reciprocal (each within 1 ulp;
                            // the result is rounded to bf16 right after)
                            float u = acc[i][j + FN / 2][4 * q + t];
                            float e = __builtin_amdgcn_exp2f(g * -1.4426950408889634f);
                            g = g * __builtin_amdgcn_rcpf(1.0f + e) * u;
                        }
                        v[t] = g;
                    }
                    if (BIG || (vec_ok && gn + 3 < N)) {
                        uint2 pk;
                        pk.x = pack_bf16x2(v[0], v[1]);
                        pk.y = pack_bf16x2(v[2], v[3]);
                        *reinterpret_cast<uint2*>(Dt + o) = pk;
                    } else {
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            if (gn + t < N) Dt[o + t].x = f32_to_bf16_bits(v[t]);
                    }
                }
            }
        }
    }
}

template <int EPI, int BM, int BN, int NW>
__global__ void __launch_bounds__(64 * NW)
gemm_mfma_kernel(const bf16* __restrict__ A, const bf16* __restrict__ W,
                 const bf16* __restrict__ W2, float* __restrict__ Cf, bf16* __restrict__ Dt, int M,
                 int N, int K, int tiles_m, int tiles_n, RopeEpilogue rope) {
    extern __shared__ __align__(16) char smem[];
    gemm_mfma_body<EPI, BM, BN, NW>(smem, A, W, W2, Cf, Dt, M, N, K, tiles_m, tiles_n, 0, 0,
                                    (int)blockIdx.x, tiles_m * tiles_n, rope);
}

// Big tiles with a quartered tail.  With one 256x256 tile per CU at a time, a launch whose tile
// count is not a multiple of the CU count ends with a round in which most CUs idle for a whole
// tile time (5152 tiles on 256 CUs: 20 rounds and 32 tiles).  Here the first n_big workgroups
// take the big tiles in the usual order EXCEPT a rectangle at its end -- the last tail_cols
// tile columns of the last 8-row group -- and the remaining workgroups cover that rectangle
// with 128x128 tiles, four times as many and a quarter as long (done only when they fit one
// round themselves: measured, more of them cost more than the idle round they replace).  The K
// order of an output element does not depend on the tile shape, so the result bits are those
// of any other tiling.
template <int EPI>
__global__ void __launch_bounds__(256)
gemm_mfma_tail_kernel(const bf16* __restrict__ A, const bf16* __restrict__ W,
                      const bf16* __restrict__ W2, float* __restrict__ Cf, bf16* __restrict__ Dt,
                      int M, int N, int K, int tiles_m, int tiles_n, int n_big, int tail_m_off,
                      int tail_n_off, int tail_tiles_m, int tail_tiles_n) {
    extern __shared__ __align__(16) char smem[];
    const RopeEpilogue none{};
    if ((int)blockIdx.x < n_big)
        gemm_mfma_body<EPI, 256, 256, 4>(smem, A, W, W2, Cf, Dt, M, N, K, tiles_m, tiles_n, 0, 0,
                                         (int)blockIdx.x, n_big, none);
    else
        gemm_mfma_body<EPI, 128, 128, 4>(smem, A, W, W2, Cf, Dt, M, N, K, tail_tiles_m, tail_tiles_n,
                                         tail_m_off, tail_n_off, (int)blockIdx.x - n_big,
                                         tail_tiles_m * tail_tiles_n, none);
}

constexpr int N_CUS = 256;            // MI355X
constexpr int GROUP_M = 8;            // tile rows per group of the tile order (see the body)

template <int EPI, int BM, int BN, int NW>
void launch_tile(hipStream_t s, const void* A, const void* W, const void* W2, float* Cf, void* Dt,
                 int M, int N, int K, bool tail_ok = false, const RopeEpilogue& rope = RopeEpilogue{}) {
    constexpr int BN_OUT = (EPI == EPI_SILU_MUL) ? BN / 2 : BN;
    constexpr int LDS = N_STAGES * (BM + BN) * ROW_BYTES;
    int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN_OUT - 1) / BN_OUT;
    if constexpr (BM == 256 && NW == 4 && EPI != EPI_ADD_F32 && EPI != EPI_QKV_ROPE128 && EPI != EPI_QKV_ROPE64) {
        // tail: the last nb % N_CUS tiles, rounded up to whole columns of the last row group
        const int nb = tiles_m * tiles_n, tail = nb % N_CUS;
        const int gsz = tiles_m - (tiles_m - 1) / GROUP_M * GROUP_M;       // rows of the last group
        const int cols = (tail + gsz - 1) / gsz;
        if (tail_ok && nb > N_CUS && tail > 0 && gsz * cols <= N_CUS / 4 && cols <= tiles_n) {
            static bool configured = false;
            auto kern = gemm_mfma_tail_kernel<EPI>;
            if (!configured) {
                (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
                configured = true;
            }
            constexpr int SBN_OUT = (EPI == EPI_SILU_MUL) ? 64 : 128;
            const int m_off = (tiles_m - gsz) * BM, n_off = (tiles_n - cols) * BN_OUT;
            const int tm = (M - m_off + 127) / 128, tn = (N - n_off + SBN_OUT - 1) / SBN_OUT;
            const int n_big = nb - gsz * cols;
            kern<<<n_big + tm * tn, 256, LDS, s>>>((const bf16*)A, (const bf16*)W, (const bf16*)W2, Cf, (bf16*)Dt,
                                                   M, N, K, tiles_m, tiles_n, n_big, m_off, n_off, tm, tn);
            return;
        }
    }
    static bool configured = false;
    auto kern = gemm_mfma_kernel<EPI, BM, BN, NW>;
    if (!configured) {
        (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        configured = true;
    }
    kern<<<tiles_m * tiles_n, 64 * NW, LDS, s>>>((const bf16*)A, (const bf16*)W, (const bf16*)W2, Cf,
                                             (bf16*)Dt, M, N, K, tiles_m, tiles_n, rope);
}

int g_force_tile = 0;   // 0 = heuristic; 256 / 128 / 64 = forced tile, 257 = 256 with the quartered tail
int g_small_below = 160;   // 64x64 tiles when there are fewer 128x128 tiles than this

template <int EPI>
void launch(hipStream_t s, const void* A, const void* W, const void* W2, float* Cf, void* Dt, int M,
            int N, int K) {
    constexpr int BN_OUT256 = (EPI == EPI_SILU_MUL) ? 128 : 256;
    int64_t tiles256 = (int64_t)((M + 255) / 256) * ((N + BN_OUT256 - 1) / BN_OUT256);
    // big tiles once there is at least one per CU (thresholds measured per epilogue); the
    // read-modify-write epilogue always takes the small tile (two blocks per CU overlap it)
    int64_t need = EPI == EPI_SILU_MUL ? 200 : 256;
    bool big = (g_force_tile ? g_force_tile >= 256 : tiles256 >= need) && K % (2 * BK) == 0 &&
               M >= 256 && N >= BN_OUT256 && EPI != EPI_ADD_F32;
    if (big) { launch_tile<EPI, 256, 256, 4>(s, A, W, W2, Cf, Dt, M, N, K, g_force_tile == 0 || g_force_tile == 257); return; }
    if constexpr (EPI != EPI_SILU_MUL) {
        // few rows against a narrow weight (a tensor-parallel shard's QKV projection): 128x128
        // tiles would leave most CUs idle, so quarter the tile.  The K order of every output
        // element is the same for all tile shapes, so the result bits do not depend on the choice.
        int64_t tiles128 = (int64_t)((M + 127) / 128) * ((N + 127) / 128);
        bool small = g_force_tile ? g_force_tile == 64 : tiles128 < g_small_below;
        if (small) { launch_tile<EPI, 64, 64, 4>(s, A, W, W2, Cf, Dt, M, N, K); return; }
    }
    launch_tile<EPI, 128, 128, 4>(s, A, W, W2, Cf, Dt, M, N, K);
}

}  // namespace

void gemm_mfma_force_tile(int t) { g_force_tile = t; }

bool gemm_mfma_qkv_rope_supported(int dtype, int M, int N, int K, int head_dim) {
    // the shapes for which the float-output QKV GEMM would take the big tile anyway, with whole
    // tiles along N (no shifted edge tile: head boundaries stay on wave-tile boundaries)
    const int64_t tiles256 = (int64_t)((M + 255) / 256) * (N / 256);
    const bool big = g_force_tile ? g_force_tile >= 256 : tiles256 >= 256;
    return dtype == CF_BF16 && (head_dim == 128 || head_dim == 64) && big && M >= 256 && N >= 256 &&
           N % 256 == 0 && K >= 2 * BK && K % (2 * BK) == 0;
}

void launch_gemm_mfma_qkv_rope(hipStream_t s, const void* A, const void* Wqkv, void* q_out, int M,
                               int N, int K, const RopeEpilogue& rope) {
    if (rope.g.head_dim == 128)
        launch_tile<EPI_QKV_ROPE128, 256, 256, 4>(s, A, Wqkv, nullptr, nullptr, q_out, M, N, K, false, rope);
    else
        launch_tile<EPI_QKV_ROPE64, 256, 256, 4>(s, A, Wqkv, nullptr, nullptr, q_out, M, N, K, false, rope);
}

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
