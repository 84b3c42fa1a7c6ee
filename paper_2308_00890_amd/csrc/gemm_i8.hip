// int8 x int8 -> int32 -> fp32 GEMM for operands that are already quantized (Sec. 3.2 Fig. 3), tiled for the
// matrix cores: this is the kernel for shapes where the product, not the HBM traffic, is the bound (wide K and N).
// The GNN layer shapes (K = 64..602) are HBM-bound and use the panel kernels of gemm.hip instead.
//
// C[m][n] = (float)(sum_k A[m][k] * BT[n][k]) * (s_A*s_B); both operands row-major with K contiguous.
// Two kernels: k_gemm_i8_dma128 (further down) for reductions that are a multiple of 128, and this one, which stages
// through registers and takes any reduction that is a multiple of 16.
// Workgroup: 256 x 256 tile of C, 4 waves, each wave a 128 x 128 sub-tile = 4 x 4 MFMA tiles of 32 x 32
// (v_mfma_i32_32x32x32_i8): 8 fragment reads of 1 KB feed 16 MFMAs per 32-deep sub-step.  One wave per SIMD (the 256
// accumulator registers allow no more), so latency is hidden by software pipelining inside the wave, not by occupancy.
#include "internal.hip.h"

#include <type_traits>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int TM = 256, TN = 256, TK = 128;  // a K-step moves whole 128-byte lines of every operand row
constexpr int LDT = TK + 16;                 // LDS row stride: 36 dwords, so 8 rows x 16 bytes hit 32 distinct banks
constexpr int OPB = TM * LDT;                // bytes of one operand tile in LDS
constexpr int NJ = TM / 32;                  // staging passes: 8 lanes x 16 bytes per row, 32 rows per pass

struct i8gemm_args {
    int64_t M;
    int N, K;
    int lda, ldb;      // row strides in bytes (>= K, multiples of 16)
    const int8_t *A;   // M x K
    const int8_t *BT;  // N x K
    const float *s_A, *s_B;
    float *C;          // M x N
    float *absmax_C;   // or NULL
};

struct stage_regs {
    v4i a[NJ], b[NJ];
};

template <int V> using ic = std::integral_constant<int, V>;

// Pipeline (tile t = K-columns [128t, 128t+128) of both operands, LDS stage t%2, staging registers R[t%2]).  Step s:
//   sub-steps 0,1: MFMAs on tile s; tile s+1 goes from R[(s+1)%2] to LDS stage (s+1)%2 (free since the barrier that
//                  ended step s-1); barrier
//   sub-steps 2,3: MFMAs on tile s; global loads of tile s+3 into the registers just freed (they are consumed 1.5
//                  steps = about 3000 MFMA cycles later); first fragments of tile s+1 read from LDS; barrier
// The fragments of every sub-step are read from LDS during the sub-step before it, and every LDS or global access
// is issued between two MFMAs, so their latencies sit under the 32-cycle MFMAs of the same wave.
__global__ __launch_bounds__(256) void k_gemm_i8(i8gemm_args a)
{
    __shared__ __align__(16) int8_t lds[2 * 2 * OPB];  // [stage][A or B][row * LDT + k]
    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int tiles_n = (a.N + TN - 1) / TN;
    const int64_t m0 = static_cast<int64_t>(blockIdx.x / tiles_n) * TM;
    const int n0 = static_cast<int>(blockIdx.x % tiles_n) * TN;
    const int wm = (wave / 2) * 128, wn = (wave % 2) * 128;

    v16i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v16i{0};

    // staging: thread t moves rows t/8 + 32*j (j = 0..7), 16 bytes at k-offset 16*(t%8), of both operands.
    // Loads are unconditional from addresses clamped into the matrix.  Rows past M or N only feed elements of C that
    // are never stored; columns past K are zeroed when the registers are written to LDS (not at the load, so that
    // no use of the loaded value sits next to it).  Addresses are a wave-uniform base plus a 32-bit lane offset.
    const int srow = tid / 8, sk = (tid % 8) * 16;
    const int8_t *baseA = a.A + m0 * a.lda;
    const int8_t *baseB = a.BT + static_cast<int64_t>(n0) * a.ldb;
    unsigned offA[NJ], offB[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int64_t ra = m0 + srow + 32 * j, rb = static_cast<int64_t>(n0) + srow + 32 * j;
        offA[j] = static_cast<unsigned>(((ra < a.M ? ra : a.M - 1) - m0) * a.lda);  // < 256 * lda < 2^32
        offB[j] = static_cast<unsigned>(((rb < a.N ? rb : a.N - 1) - n0) * a.ldb);
    }
    auto gload = [&](stage_regs &r, int tile, auto masked) {
        unsigned k = static_cast<unsigned>(tile * TK + sk);
        if (decltype(masked)::value) k = k < static_cast<unsigned>(a.K) ? k : static_cast<unsigned>(a.K - 16);
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            r.a[j] = *reinterpret_cast<const v4i *>(baseA + (offA[j] + k));
            r.b[j] = *reinterpret_cast<const v4i *>(baseB + (offB[j] + k));
        }
    };
    auto lstore = [&](const stage_regs &r, auto stage, int tile, auto masked, auto half) {
        int8_t *base = lds + decltype(stage)::value * 2 * OPB + srow * LDT + sk;
        const bool ok = !decltype(masked)::value || tile * TK + sk < a.K;
        const v4i zero = v4i{0, 0, 0, 0};
#pragma unroll
        for (int j = decltype(half)::value * (NJ / 2); j < (decltype(half)::value + 1) * (NJ / 2); ++j) {
            *reinterpret_cast<v4i *>(base + 32 * j * LDT) = ok ? r.a[j] : zero;
            *reinterpret_cast<v4i *>(base + OPB + 32 * j * LDT) = ok ? r.b[j] : zero;
        }
    };
    const int frag_off = (lane % 32) * LDT + 16 * (lane / 32);
    auto read_frags = [&](v4i(&fa)[4], v4i(&fb)[4], auto stage, int ks) {
        const int8_t *pa = lds + decltype(stage)::value * 2 * OPB + wm * LDT + frag_off + ks;
        const int8_t *pb = lds + decltype(stage)::value * 2 * OPB + OPB + wn * LDT + frag_off + ks;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[i] = *reinterpret_cast<const v4i *>(pa + i * 32 * LDT);
            fb[i] = *reinterpret_cast<const v4i *>(pb + i * 32 * LDT);
        }
    };
    auto mfma_block = [&](const v4i(&fa)[4], const v4i(&fb)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
    };
    // issue order of one 16-MFMA sub-step: 8 LDS reads, then 8 accesses of another kind (mask), one per MFMA
    // (masks: 0x8 MFMA, 0x100 LDS read, 0x200 LDS write, 0x20 global read)
    auto interleave = [&](auto second) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(decltype(second)::value, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
    };

    stage_regs R0, R1;
    v4i fa0[4], fb0[4], fa1[4], fb1[4];
    // prologue: tile 0 in LDS stage 0, tiles 1 and 2 in flight, fragments of (tile 0, sub-step 0) read
    // (the scheduling fences keep the loads in this order, which is the order the loop's wait counts assume)
    gload(R0, 0, std::true_type{});
    __builtin_amdgcn_sched_barrier(0);
    gload(R1, 1, std::true_type{});
    __builtin_amdgcn_sched_barrier(0);
    lstore(R0, ic<0>{}, 0, std::true_type{}, ic<0>{});
    lstore(R0, ic<0>{}, 0, std::true_type{}, ic<1>{});
    __builtin_amdgcn_sched_barrier(0);
    gload(R0, 2, std::true_type{});
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    read_frags(fa0, fb0, ic<0>{}, 0);

    // Rn: the staging registers that hold tile s+1 on entry
    auto step = [&](stage_regs &Rn, int s, auto cur, auto masked) {
        constexpr int nxt = 1 - decltype(cur)::value;
        read_frags(fa1, fb1, cur, 32);
        lstore(Rn, ic<nxt>{}, s + 1, masked, ic<0>{});
        mfma_block(fa0, fb0);
        interleave(ic<0x200>{});
        read_frags(fa0, fb0, cur, 64);
        lstore(Rn, ic<nxt>{}, s + 1, masked, ic<1>{});
        mfma_block(fa1, fb1);
        interleave(ic<0x200>{});
        __syncthreads();
        read_frags(fa1, fb1, cur, 96);
        gload(Rn, s + 3, masked);
        mfma_block(fa0, fb0);
        read_frags(fa0, fb0, ic<nxt>{}, 0);
        mfma_block(fa1, fb1);
        interleave(ic<0x020>{});
        interleave(ic<0x020>{});
        __syncthreads();
    };
    const int nsteps = ((a.K + TK - 1) / TK + 1) & ~1;  // even; a tile past K is all zeros
    int s = 0;
    for (; (s + 5) * TK <= a.K; s += 2) {  // tiles up to s+4 lie inside K: nothing to clamp or zero
        step(R1, s, ic<0>{}, std::false_type{});
        step(R0, s + 1, ic<1>{}, std::false_type{});
    }
    for (; s < nsteps; s += 2) {
        step(R1, s, ic<0>{}, std::true_type{});
        step(R0, s + 1, ic<1>{}, std::true_type{});
    }

    // epilogue: dequantize, store, abs-max (element r of a 32x32 tile: column lane%32, row 8*(r/4) + 4*(lane/32) + r%4).
    const float sc = (*a.s_A) * (*a.s_B);
    int maxabs = 0;
    const int col0 = n0 + wn + lane % 32;
    const int64_t row0 = m0 + wm + (lane / 32) * 4;
    if (m0 + TM <= a.M && n0 + TN <= a.N && a.N < (1 << 22)) {
        // interior tile: no guards; every address is a wave-uniform pointer plus one 32-bit lane offset
        float *ct = a.C + (m0 + wm) * a.N + (n0 + wn);
        const unsigned lane_off = static_cast<unsigned>((lane / 32) * 4 * a.N + lane % 32);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float *cu = ct + static_cast<int64_t>(i * 32 + (r / 4) * 8 + (r % 4)) * a.N + j * 32;
                    cu[lane_off] = static_cast<float>(acc[i][j][r]) * sc;
                    maxabs = max(maxabs, abs(acc[i][j][r]));
                    if (r % 4 == 3) __builtin_amdgcn_sched_barrier(0);  // keep the register footprint of this part small
                }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = col0 + j * 32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t row = row0 + i * 32 + (r / 4) * 8 + (r % 4);
                    if (row < a.M && col < a.N) {
                        a.C[row * a.N + col] = static_cast<float>(acc[i][j][r]) * sc;
                        maxabs = max(maxabs, abs(acc[i][j][r]));
                    }
                }
            }
    }
    if (a.absmax_C) {
        float m = static_cast<float>(maxabs) * sc;
        m = tango_wave_max(m);
        if (lane == 0 && m > 0.0f) tango_atomic_max_nonneg(a.absmax_C, m);
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Second kernel, for reductions that are a multiple of 128.  Operand tiles go from global memory straight into LDS
// (global_load_lds_dwordx4: lane i's 16 bytes land at the wave's LDS base + 16 i; no staging registers, no LDS-write
// instructions), and eight waves share a 256 x 256 tile of C, two per SIMD, so that one wave's waits (barrier, LDS
// latency) sit under the other's MFMAs.  A wave owns a 128 x 64 sub-tile: 4 x 2 MFMA tiles, 128 accumulator registers.
//
// Every load instruction moves whole 128-byte lines (8 lanes per row, 8 rows per wave-wide load).  K-step 128, two LDS
// stages of 2 x 32 KB.  A row of a stage is eight 16-byte chunks, chunk c of row r in slot c ^ ((r >> 1) & 7): the DMA
// writes contiguous kilobytes (which global chunk a lane fetches is chosen to produce this layout), and the sixteen
// consecutive rows of one LDS cycle of a fragment read (16 lanes x 16 bytes) cover all 64 banks once.
//
// Pipeline: a step is four half-steps of eight MFMAs (k = 32 each).  The last half-step of tile s-1 is held back in
// registers across the barrier that opens step s: wait for my loads of tile s -> barrier (tile s complete; nobody
// reads tile s-1 from LDS any more) -> issue the loads of tile s+1 into the stage of tile s-1 -> MFMAs (s-1, last
// quarter) while the fragments (s, first quarter) are read -> ... -> MFMAs (s, third quarter) while (s, last quarter)
// is read.  The first MFMA behind a barrier never waits for a fresh LDS read, fragment requests go out one at a time,
// each behind an MFMA and at least six MFMAs ahead of its first use (the barrier keeps the eight waves in step: requested
// together they would hit the LDS all at once), and a load has a whole step (about 2,000 MFMA cycles per SIMD) to arrive.
// ---------------------------------------------------------------------------------------------------------------
__device__ __forceinline__ void dma16(const int8_t *g, int8_t *l)
{
    __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t *>(g), reinterpret_cast<uint32_t *>(l), 16, 0, 0);
}

constexpr int EK = 128;
constexpr int EOPB = TM * EK;       // 32 KB per operand tile
constexpr int ESTB = 2 * EOPB;      // 64 KB per stage
constexpr int ELDS = 2 * ESTB;      // 128 KB

__global__ __launch_bounds__(512) void k_gemm_i8_dma128(i8gemm_args a)
{
    extern __shared__ __align__(16) int8_t dlds[];
    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int tiles_n = (a.N + TN - 1) / TN;
    int tile_m, tile_n;
    if (tiles_n % 8 == 0) {
        // workgroups go to the 8 XCDs in turn (each with an L2 of its own): XCD x takes the tile columns
        // [x, x+1) * tiles_n / 8, row by row, so that the tiles running on it at one time share A and B panels in its L2
        const int cpx = tiles_n / 8, xcd = blockIdx.x % 8, j = blockIdx.x / 8;
        tile_n = xcd * cpx + j % cpx;
        tile_m = j / cpx;
    } else {
        tile_m = blockIdx.x / tiles_n;
        tile_n = blockIdx.x % tiles_n;
    }
    const int64_t m0 = static_cast<int64_t>(tile_m) * TM;
    const int n0 = tile_n * TN;
    const int wm = (wave / 4) * 128, wn = (wave % 4) * 64;

    v16i acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = v16i{0};

    // DMA sources: wave w fills LDS kilobytes 4w .. 4w+3 of both operand tiles = rows 32w .. 32w+31; lane l of a load
    // lands in (row l/8 of the kilobyte, slot l%8) and therefore fetches chunk (l%8) ^ ((row >> 1) & 7) of that row.
    const int8_t *gA = a.A + m0 * a.lda;
    const int8_t *gB = a.BT + static_cast<int64_t>(n0) * a.ldb;
    unsigned offA[4], offB[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = (wave * 4 + j) * 8 + lane / 8;
        const int kc = (lane % 8) ^ ((row >> 1) & 7);
        const int64_t ra = m0 + row, rb = static_cast<int64_t>(n0) + row;
        offA[j] = static_cast<unsigned>(((ra < a.M ? ra : a.M - 1) - m0) * a.lda + kc * 16);  // < 256 * lda < 2^32
        offB[j] = static_cast<unsigned>(((rb < a.N ? rb : a.N - 1) - n0) * a.ldb + kc * 16);
    }
    const int ntiles = a.K / EK;
    auto issue = [&](int t) {
        const int k = (t < ntiles ? t : ntiles - 1) * EK;  // past the end: the last tile once more, into the free stage
        int8_t *st = dlds + (t & 1) * ESTB + wave * 4096;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            dma16(gA + (offA[j] + static_cast<unsigned>(k)), st + j * 1024);
            dma16(gB + (offB[j] + static_cast<unsigned>(k)), st + EOPB + j * 1024);
        }
    };
    const int r32 = lane % 32, kh = lane / 32;
    const int aoff = (wm + r32) * EK + ((kh ^ (((wm + r32) >> 1) & 7)) * 16);
    const int boff = EOPB + (wn + r32) * EK + ((kh ^ (((wn + r32) >> 1) & 7)) * 16);

#define TANGO_FENCE() __builtin_amdgcn_sched_barrier(0)
#define TANGO_MF(i, j) \
    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0); \
    TANGO_FENCE()
#define TANGO_RA(i) \
    if (rd) na[i] = *reinterpret_cast<const v4i *>(base + ((aoff ^ (q * 32)) + i * 32 * EK)); \
    TANGO_FENCE()
#define TANGO_RB(j) \
    if (rd) nb[j] = *reinterpret_cast<const v4i *>(base + ((boff ^ (q * 32)) + j * 32 * EK)); \
    TANGO_FENCE()
    // eight MFMAs on (fa, fb); meanwhile (rd) the fragments (na, nb) of quarter q of the tile at `base` are requested, one
    // behind each MFMA and at least six MFMAs ahead of their first use, and (dma_tile >= 0) that tile's loads are issued
    auto half_step = [&](const v4i(&fa)[4], const v4i(&fb)[2], v4i(&na)[4], v4i(&nb)[2], const int8_t *base, int q,
                         auto read, int dma_tile) {
        constexpr bool rd = decltype(read)::value;
        TANGO_FENCE();
        TANGO_MF(0, 0);
        if (dma_tile >= 0) {
            issue(dma_tile);
            TANGO_FENCE();
        }
        TANGO_RA(0);
        TANGO_MF(0, 1);
        TANGO_RB(0);
        TANGO_MF(1, 0);
        TANGO_RB(1);
        TANGO_MF(1, 1);
        TANGO_RA(1);
        TANGO_MF(2, 0);
        TANGO_RA(2);
        TANGO_MF(2, 1);
        TANGO_RA(3);
        TANGO_MF(3, 0);
        TANGO_MF(3, 1);
    };
#undef TANGO_RB
#undef TANGO_RA
#undef TANGO_MF
#undef TANGO_FENCE
    constexpr std::true_type RD{};
    constexpr std::false_type NORD{};

    v4i fa0[4], fb0[2], fa1[4], fb1[2];
    issue(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): my part of tile 0 has landed
    __builtin_amdgcn_s_barrier();
    issue(1);
    {
        const int8_t *base = dlds;
#pragma unroll
        for (int i = 0; i < 4; ++i) fa0[i] = *reinterpret_cast<const v4i *>(base + (aoff + i * 32 * EK));
#pragma unroll
        for (int j = 0; j < 2; ++j) fb0[j] = *reinterpret_cast<const v4i *>(base + (boff + j * 32 * EK));
        half_step(fa0, fb0, fa1, fb1, base, 1, RD, -1);
        half_step(fa1, fb1, fa0, fb0, base, 2, RD, -1);
        half_step(fa0, fb0, fa1, fb1, base, 3, RD, -1);
    }
    for (int s = 1; s < ntiles; ++s) {
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): my part of tile s has landed
        __builtin_amdgcn_s_barrier();
        const int8_t *base = dlds + (s & 1) * ESTB;
        half_step(fa1, fb1, fa0, fb0, base, 0, RD, s + 1);  // (s-1, last quarter), held in registers across the barrier
        half_step(fa0, fb0, fa1, fb1, base, 1, RD, -1);
        half_step(fa1, fb1, fa0, fb0, base, 2, RD, -1);
        half_step(fa0, fb0, fa1, fb1, base, 3, RD, -1);
    }
    half_step(fa1, fb1, fa0, fb0, dlds, 0, NORD, -1);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // (the last, redundant load must not outlive the workgroup's LDS)

    // epilogue: dequantize, store, abs-max (element r of a 32x32 tile: column lane%32, row 8*(r/4) + 4*(lane/32) + r%4)
    const float sc = (*a.s_A) * (*a.s_B);
    int maxabs = 0;
    if (m0 + TM <= a.M && n0 + TN <= a.N && a.N < (1 << 22)) {
        float *ct = a.C + (m0 + wm) * a.N + (n0 + wn);
        const unsigned lane_off = static_cast<unsigned>((lane / 32) * 4 * a.N + lane % 32);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float *cu = ct + static_cast<int64_t>(i * 32 + (r / 4) * 8 + (r % 4)) * a.N + j * 32;
                    cu[lane_off] = static_cast<float>(acc[i][j][r]) * sc;
                    maxabs = max(maxabs, abs(acc[i][j][r]));
                }
    } else {
        const int col0 = n0 + wn + lane % 32;
        const int64_t row0 = m0 + wm + (lane / 32) * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int col = col0 + j * 32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t row = row0 + i * 32 + (r / 4) * 8 + (r % 4);
                    if (row < a.M && col < a.N) {
                        a.C[row * a.N + col] = static_cast<float>(acc[i][j][r]) * sc;
                        maxabs = max(maxabs, abs(acc[i][j][r]));
                    }
                }
            }
    }
    if (a.absmax_C) {
        float m = static_cast<float>(maxabs) * sc;
        m = tango_wave_max(m);
        if (lane == 0 && m > 0.0f) tango_atomic_max_nonneg(a.absmax_C, m);
    }
}

}  // namespace

// The product for operands with row strides (bytes) lda, ldb >= K, both multiples of 16; used by the quantizing GEMM
// entry points when the reduction is too long for their panel kernel.
int tango_gemm_i8_async(int64_t M, int64_t N, int64_t K, const int8_t *A_q, int64_t lda, const float *s_A, const int8_t *BT_q,
                        int64_t ldb, const float *s_B, float *C, float *absmax_C, hipStream_t st)
{
    TANGO_REQUIRE(K % 16 == 0 && lda % 16 == 0 && ldb % 16 == 0 && lda >= K && ldb >= K && lda < (int64_t(1) << 24) &&
                      ldb < (int64_t(1) << 24),
                  TANGO_ERR_UNSUPPORTED);
    if (absmax_C) {
        int rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(absmax_C), 0u, 1, st);
        if (rc != TANGO_OK) return rc;
    }
    i8gemm_args a;
    a.M = M; a.N = static_cast<int>(N); a.K = static_cast<int>(K);
    a.lda = static_cast<int>(lda); a.ldb = static_cast<int>(ldb);
    a.A = A_q; a.BT = BT_q; a.s_A = s_A; a.s_B = s_B; a.C = C; a.absmax_C = absmax_C;
    const int64_t tiles = ((M + TM - 1) / TM) * ((N + TN - 1) / TN);
    TANGO_REQUIRE(tiles < (int64_t(1) << 31), TANGO_ERR_BAD_SHAPE);
    if (K % EK == 0) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_i8_dma128), hipFuncAttributeMaxDynamicSharedMemorySize, ELDS) !=
            hipSuccess)
            return TANGO_ERR_LAUNCH;
        k_gemm_i8_dma128<<<static_cast<unsigned>(tiles), 512, ELDS, st>>>(a);
    } else {
        k_gemm_i8<<<static_cast<unsigned>(tiles), 256, 0, st>>>(a);
    }
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

extern "C" {

int tango_qgemm_i8(int64_t M, int64_t N, int64_t K, const int8_t *A_q, const float *s_A, const int8_t *BT_q,
                   const float *s_B, float *C, float *absmax_C, void *stream)
{
    TANGO_REQUIRE(M >= 1 && N >= 1 && K >= 1 && M < (int64_t(1) << 31) && N < (int64_t(1) << 24) && K < (int64_t(1) << 24),
                  TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(K % 16 == 0, TANGO_ERR_UNSUPPORTED);
    TANGO_REQUIRE(A_q && s_A && BT_q && s_B && C, TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(A_q, 16) && tango_aligned(BT_q, 16) && tango_aligned(C, 4), TANGO_ERR_BAD_SHAPE);
    return tango_gemm_i8_async(M, N, K, A_q, K, s_A, BT_q, K, s_B, C, absmax_C, tango_stream(stream));
}

}  // extern "C"
