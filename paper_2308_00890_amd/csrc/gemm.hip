// Quantized GEMM on the int8 matrix cores (Sec. 3.2 Fig. 3; Sec. 3.3 "GEMM with
// on-the-fly quantization", Fig. 4), forward and backward.
//
// What is kept from the paper's design: the fp32 operand is quantized while it
// is loaded (no separate pass), its int8 copy is written back for the backward
// pass, accumulation is int32 in registers, the result is dequantized in
// registers and the abs-max that the next quantization needs is computed in the
// same kernel.  What differs (the paper tiles for V100 CUDA cores and DP4A):
// the products run on v_mfma_i32_32x32x32_i8; at GNN shapes (K = 64..602,
// N = 64..384) the GEMM is bound by HBM traffic of the tall fp32 operand, not
// by the matrix cores, so a workgroup quantizes a whole 64-row panel of A
// (all K) into LDS once -- a contiguous, perfectly coalesced stream -- and then
// sweeps all N columns against the small, cache-resident quantized B.
//
// Algorithmic HBM bytes of the forward call per row of A: 4K (abs-max pass)
// + 4K (read) + K (A_q write) + 4N (C write).
#include <type_traits>

#include "internal.hip.h"

int tango_gemm_i8_async(int64_t M, int64_t N, int64_t K, const int8_t *A_q, int64_t lda, const float *s_A, const int8_t *BT_q,
                        int64_t ldb, const float *s_B, float *C, float *absmax_C, hipStream_t st);

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 64;     // rows of A per workgroup
constexpr int BN = 256;    // columns per sweep: 4 waves x 64
constexpr int KMAX = 2048; // largest reduction length whose 64-row int8 panel fits LDS
// weight matrices up to this size are prepared by one launch in which every workgroup finds max|B| for itself
constexpr int64_t SMALL_B_ELEMS = 8192;
constexpr int64_t SMALL_A_ELEMS = 1 << 20;  // an A of up to this size has its abs-max found by that same launch
constexpr int LDS_PAD = 16;

struct fused_args {
    int64_t M;
    int N, K;        // logical sizes: out is M x N, reduction K
    int Kp, Np;      // padded: Kp multiple of 32 (BT row length), Np multiple of 64 (BT rows)
    const float *A;  // M x K fp32
    const float *absmax_A;
    int absmax_A_count;  // 1, or the number of partial maxima at absmax_A (tango_absmax_load)
    tango_rng rng;
    int8_t *A_q;     // M x K
    float *s_A;      // out
    const int8_t *BT;  // Np x Kp, zero padded
    const float *s_B;
    float *C;        // M x N
    float *absmax_C; // or NULL
    const uint32_t *C_keep_bits;  // or NULL: bit i of the flat M x N output clear -> C[i] is written as 0 and does not count
                                  // in absmax_C (a ReLU' applied on the way out); N a multiple of 32
    uint32_t K_magic;  // ceil(2^32 / K): f / K == umulhi(f, K_magic) for the flat panel offsets f < 64 * K (K >= 2)
};

template <int ROUNDING>
__device__ inline uint2 quantize8_packed(const float (&y)[8], const tango_rng &rng, uint64_t blk)
{
    uint4 b = make_uint4(0, 0, 0, 0);
    if (ROUNDING == TANGO_SR) b = tango_philox_block(rng, blk);
    const uint32_t w[4] = {b.x, b.y, b.z, b.w};
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t bits = (j & 1) ? (w[j >> 1] >> 16) : (w[j >> 1] & 0xffffu);
        const uint32_t byte = static_cast<uint32_t>(tango_round_clamp<ROUNDING>(y[j], bits)) & 0xffu;
        if (j < 4)
            lo |= byte << (8 * j);
        else
            hi |= byte << (8 * (j - 4));
    }
    return make_uint2(lo, hi);
}

// WL = bytes per LDS write: 4 if K % 4 == 0, 2 if K % 2 == 0, else 1 (pieces never straddle a row then).
template <int ROUNDING, int WL, bool KEEP = false>
// (Occupancy: three waves per SIMD.  Capping the registers for four was measured slower at K = 384 - 2.22 against 2.05 ms
// for 2.4 M rows - and two against three makes no difference: the kernel runs at 0.85-0.9 of the rate a plain streaming
// kernel with its read : write mix reaches.)
__global__ __launch_bounds__(256) void k_qgemm_fused(fused_args a)
{
    extern __shared__ __align__(16) int8_t lds[];
    const int LDK = a.Kp + LDS_PAD;
    const int tid = threadIdx.x;
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * BM;
    const int rows = static_cast<int>(min(static_cast<int64_t>(BM), a.M - row0));

    // ---- phase 1: stream the panel (a contiguous range of A), quantize, keep it in LDS and write it back
    float s, inv;
    tango_scale_from_absmax(tango_absmax_load(a.absmax_A, a.absmax_A_count), s, inv);
    if (blockIdx.x == 0 && tid == 0) *a.s_A = s;
    const int64_t flat0 = row0 * a.K;  // multiple of 8 because row0 is a multiple of 64
    const int cnt = rows * a.K;
    const int ngroups = (cnt + 7) / 8;
    const float *Ap = a.A + flat0;
    int8_t *Aq = a.A_q + flat0;
    // one group of 8 elements (one Philox block): quantize y, write the int8 copy back and into the LDS panel
    auto finish_group = [&](int f, int valid, const float (&y)[8]) {
        const uint2 q = quantize8_packed<ROUNDING>(y, a.rng, static_cast<uint64_t>((flat0 + f) >> 3));
        if (valid == 8) {
            *reinterpret_cast<uint2 *>(Aq + f) = q;
        } else {
            for (int j = 0; j < valid; ++j) Aq[f + j] = static_cast<int8_t>((j < 4 ? q.x >> (8 * j) : q.y >> (8 * (j - 4))) & 0xffu);
        }
        int row = a.K == 1 ? f : static_cast<int>(__umulhi(static_cast<uint32_t>(f), a.K_magic));  // f / K
        int col = f - row * a.K;
        const uint64_t bits = (static_cast<uint64_t>(q.y) << 32) | q.x;
#pragma unroll
        for (int j = 0; j < 8; j += WL) {
            if (j < valid) {
                int8_t *dst = lds + row * LDK + col;
                if (WL == 4)
                    *reinterpret_cast<uint32_t *>(dst) = static_cast<uint32_t>(bits >> (8 * j));
                else if (WL == 2)
                    *reinterpret_cast<uint16_t *>(dst) = static_cast<uint16_t>(bits >> (8 * j));
                else
                    *dst = static_cast<int8_t>(bits >> (8 * j));
                col += WL;
                if (col >= a.K) {
                    col -= a.K;
                    row += 1;
                }
            }
        }
    };
    // four full groups per thread and iteration: their eight 16-byte loads are in flight together
    constexpr int UG = 4;
    const int nfull = cnt / 8;  // groups with all 8 elements
    int g = tid;
    for (; g + (UG - 1) * 256 < nfull; g += UG * 256) {
        float4 x0[UG], x1[UG];
#pragma unroll
        for (int u = 0; u < UG; ++u) {
            x0[u] = *reinterpret_cast<const float4 *>(Ap + (g + u * 256) * 8);
            x1[u] = *reinterpret_cast<const float4 *>(Ap + (g + u * 256) * 8 + 4);
        }
#pragma unroll
        for (int u = 0; u < UG; ++u) {
            const float y[8] = {x0[u].x * inv, x0[u].y * inv, x0[u].z * inv, x0[u].w * inv,
                                x1[u].x * inv, x1[u].y * inv, x1[u].z * inv, x1[u].w * inv};
            finish_group((g + u * 256) * 8, 8, y);
        }
    }
    for (; g < ngroups; g += 256) {
        const int f = g * 8;
        const int valid = min(8, cnt - f);
        float y[8];
        if (valid == 8) {
            const float4 x0 = *reinterpret_cast<const float4 *>(Ap + f);
            const float4 x1 = *reinterpret_cast<const float4 *>(Ap + f + 4);
            y[0] = x0.x * inv; y[1] = x0.y * inv; y[2] = x0.z * inv; y[3] = x0.w * inv;
            y[4] = x1.x * inv; y[5] = x1.y * inv; y[6] = x1.z * inv; y[7] = x1.w * inv;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) y[j] = (j < valid) ? Ap[f + j] * inv : 0.0f;
        }
        finish_group(f, valid, y);
    }
    __syncthreads();

    // ---- phase 2: int8 MFMA sweep over the columns; B^T fragments come straight from the (cached) global copy
    const int lane = tid % TANGO_WAVE, wave = tid / TANGO_WAVE;
    const float sc = s * (*a.s_B);
    const int8_t *ap0 = lds + (lane % 32) * LDK + 16 * (lane / 32);
    const int8_t *ap1 = ap0 + 32 * LDK;
    int maxabs = 0;
    for (int nt = 0; nt < a.Np; nt += BN) {
        const int col0 = nt + wave * 64;
        if (col0 >= a.Np) break;
        v16i acc00 = {0}, acc01 = {0}, acc10 = {0}, acc11 = {0};
        const int8_t *bp0 = a.BT + static_cast<int64_t>(col0 + lane % 32) * a.Kp + 16 * (lane / 32);
        const int8_t *bp1 = bp0 + static_cast<int64_t>(32) * a.Kp;
        v4i b0 = *reinterpret_cast<const v4i *>(bp0);
        v4i b1 = *reinterpret_cast<const v4i *>(bp1);
        for (int kk = 0; kk < a.Kp; kk += 32) {
            const v4i a0 = *reinterpret_cast<const v4i *>(ap0 + kk);
            const v4i a1 = *reinterpret_cast<const v4i *>(ap1 + kk);
            const v4i c0 = b0, c1 = b1;
            if (kk + 32 < a.Kp) {  // prefetch the next B fragments
                b0 = *reinterpret_cast<const v4i *>(bp0 + kk + 32);
                b1 = *reinterpret_cast<const v4i *>(bp1 + kk + 32);
            }
            acc00 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, c0, acc00, 0, 0, 0);
            acc01 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, c1, acc01, 0, 0, 0);
            acc10 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, c0, acc10, 0, 0, 0);
            acc11 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, c1, acc11, 0, 0, 0);
        }
        // epilogue: dequantize in registers, store, track the abs-max
        // (element i of a 32x32 tile: column = lane%32, row = 8*(i/4) + 4*(lane/32) + i%4).  Every address is the
        // workgroup's (uniform) base plus a 32-bit offset, and the row part of that offset is uniform too: the sixty-four
        // stores of a wave need no 64-bit address arithmetic and no registers to hold addresses.
        float *Cb = a.C + row0 * a.N;
        const uint32_t un = static_cast<uint32_t>(a.N);
        auto store_tiles = [&](auto checked_tag) {
            constexpr bool CHECKED = decltype(checked_tag)::value;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const v16i &acc = t == 0 ? acc00 : (t == 1 ? acc01 : (t == 2 ? acc10 : acc11));
                const int rb = t / 2, cb = t % 2;
                const int col = col0 + cb * 32 + lane % 32;
                const int rfirst = rb * 32 + (lane / 32) * 4;
                const uint32_t off0 = static_cast<uint32_t>(rfirst) * un + static_cast<uint32_t>(col);
                uint32_t mine = 0u;
                if constexpr (KEEP) {
                    // the 32 columns of a tile row are one aligned word of the bit array (N a multiple of 32): lane l
                    // fetches the word of row l % 32 of this tile, and every lane then picks the words of its sixteen rows
                    const int64_t wr = row0 + rb * 32 + lane % 32;
                    if (rb * 32 + lane % 32 < rows && col < a.N) mine = a.C_keep_bits[(wr * a.N + (col - lane % 32)) >> 5];
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int rl = (i / 4) * 8 + (i % 4);
                    int v = acc[i];
                    if constexpr (KEEP) {
                        const uint32_t kw = static_cast<uint32_t>(__shfl(static_cast<int>(mine), (lane / 32) * 4 + rl, 64));
                        v = ((kw >> (lane % 32)) & 1u) ? v : 0;
                    }
                    if (!CHECKED || (rfirst + rl < rows && col < a.N)) {
                        Cb[off0 + static_cast<uint32_t>(rl) * un] = static_cast<float>(v) * sc;
                        maxabs = max(maxabs, abs(v));
                    }
                }
            }
        };
        if (rows == BM && col0 + 64 <= a.N)
            store_tiles(std::false_type{});
        else
            store_tiles(std::true_type{});
    }
    if (a.absmax_C) {
        float m = static_cast<float>(maxabs) * sc;  // conversion and product are monotone
        m = tango_wave_max(m);
        if (lane == 0 && m > 0.0f) tango_atomic_max_nonneg(a.absmax_C, m);
    }
}

// B (K x N fp32) -> B_q (K x N int8) and its zero-padded transpose BT (Np x Kp).  B is small: one element per thread.
template <int ROUNDING>
__global__ __launch_bounds__(256) void k_quantize_b(int K, int N, int Kp, const float *__restrict__ B,
                                                    const float *__restrict__ absmax_B, tango_rng rng,
                                                    int8_t *__restrict__ B_q, float *s_B, int8_t *__restrict__ BT)
{
    float s, inv;
    tango_scale_from_absmax(*absmax_B, s, inv);
    if (blockIdx.x == 0 && threadIdx.x == 0) *s_B = s;
    const int64_t total = static_cast<int64_t>(K) * N;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < total;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        uint32_t bits = 0;
        if (ROUNDING == TANGO_SR) bits = tango_bits16(tango_philox_block(rng, static_cast<uint64_t>(i) >> 3), static_cast<int>(i & 7));
        const int8_t q = static_cast<int8_t>(tango_round_clamp<ROUNDING>(B[i] * inv, bits));
        B_q[i] = q;
        const int k = static_cast<int>(i / N), n = static_cast<int>(i - static_cast<int64_t>(k) * N);
        BT[static_cast<int64_t>(n) * Kp + k] = q;
    }
}

// The same for a small B in ONE launch: clears the abs-max words of the call (absmax_A may be NULL) and the runs of
// also_zero, finds max|B| (left in *absmax_B), then writes B_q and every byte of BT, padding included.  Every workgroup
// finds max|B| for itself - B is a few thousand elements, reading it again costs less than a grid-wide reduction and the
// launch that would have to clear its target - and takes its share of the words to write and to clear.  It replaces four
// launches that are each a few microseconds of latency on graphs too small to hide them.
template <int ROUNDING>
__global__ __launch_bounds__(256) void k_quantize_b_small(int K, int N, int Kp, int Np, const float *__restrict__ B,
                                                          float *absmax_A, float *absmax_B, float *absmax_C, tango_rng rng,
                                                          int8_t *__restrict__ B_q, float *s_B, int8_t *__restrict__ BT,
                                                          tango_zero_regions also_zero, const float *__restrict__ A, int64_t a_elems,
                                                          float *__restrict__ a_partials)
{
    __shared__ float red[4], red_a[4];
    __shared__ float Bs[SMALL_B_ELEMS];  // B itself: read from memory once, the second pass takes it from here
    const int64_t tid = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x, nthr = static_cast<int64_t>(gridDim.x) * 256;
    // a small A whose abs-max is not known (a_partials != NULL): this workgroup's share of max|A|, left as one of
    // gridDim.x partial maxima for the GEMM kernel to reduce (no atomics, so no launch that clears their target, and no
    // launch of its own).  Its loads go out together with those of B: one memory round trip for both.
    tango_zero_regions_apply(also_zero, tid, nthr);  // (stores that nothing below waits for)
    float ma = 0.0f;
    if (a_partials) {
        const float4 *A4 = reinterpret_cast<const float4 *>(A);  // (A is 16-byte aligned: the entry point requires it)
        for (int64_t i = tid; i < a_elems / 4; i += nthr) {
            const float4 v = A4[i];
            ma = fmaxf(ma, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
        }
        for (int64_t i = a_elems / 4 * 4 + tid; i < a_elems; i += nthr) ma = fmaxf(ma, fabsf(A[i]));
    }
    const int total = K * N;
    float m = 0.0f;
    for (int i = threadIdx.x; i < total; i += 256) {
        const float v = B[i];
        Bs[i] = v;
        m = fmaxf(m, fabsf(v));
    }
    m = tango_wave_max(m);
    ma = tango_wave_max(ma);
    if (threadIdx.x % TANGO_WAVE == 0) {
        red[threadIdx.x / TANGO_WAVE] = m;
        red_a[threadIdx.x / TANGO_WAVE] = ma;
    }
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    if (a_partials && threadIdx.x == 0) a_partials[blockIdx.x] = fmaxf(fmaxf(red_a[0], red_a[1]), fmaxf(red_a[2], red_a[3]));
    float s, inv;
    tango_scale_from_absmax(m, s, inv);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *s_B = s;
        *absmax_B = m;
        if (absmax_A) *absmax_A = 0.0f;
        if (absmax_C) *absmax_C = 0.0f;
    }
    const int wpr = Kp / 4;  // 32-bit words per row of BT
    for (int w = static_cast<int>(tid); w < Np * wpr; w += static_cast<int>(nthr)) {
        const int n = w / wpr, k0 = (w - n * wpr) * 4;
        uint32_t word = 0;
        if (n < N) {
            for (int j = 0; j < 4; ++j) {
                const int k = k0 + j;
                if (k >= K) break;
                const int i = k * N + n;
                uint32_t bits = 0;
                if (ROUNDING == TANGO_SR) bits = tango_bits16(tango_philox_block(rng, static_cast<uint64_t>(i) >> 3), i & 7);
                const int q = tango_round_clamp<ROUNDING>(Bs[i] * inv, bits);
                B_q[i] = static_cast<int8_t>(q);
                word |= (static_cast<uint32_t>(q) & 0xffu) << (8 * j);
            }
        }
        reinterpret_cast<uint32_t *>(BT)[w] = word;
    }
}

// src (R x C int8) -> dst (Rp x Cp bytes, Cp a multiple of 4), every byte of dst written (zero in the padding); the same
// launch clears n_zero 32-bit words at zero_words (the weight-gradient accumulator) and one more at zero_one (an abs-max),
// either of which may be NULL.
__global__ __launch_bounds__(256) void k_pad_copy_i8(int R, int C, int Rp, int Cp, const int8_t *__restrict__ src,
                                                     int8_t *__restrict__ dst, uint32_t *zero_words, int64_t n_zero,
                                                     uint32_t *zero_one, tango_colsum_job tail)
{
    if (blockIdx.x == gridDim.x - 1) tango_colsum_apply(tail);  // (a job left over from the previous step of the chain)
    const int wpr = Cp / 4;
    const int64_t words = static_cast<int64_t>(Rp) * wpr;
    if (blockIdx.x == 0 && threadIdx.x == 0 && zero_one) *zero_one = 0u;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < words + n_zero;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        if (i >= words) {
            zero_words[i - words] = 0u;
            continue;
        }
        const int r = static_cast<int>(i / wpr), c0 = static_cast<int>(i - static_cast<int64_t>(r) * wpr) * 4;
        uint32_t word = 0;
        if (r < R) {
            for (int j = 0; j < 4 && c0 + j < C; ++j)
                word |= static_cast<uint32_t>(static_cast<uint8_t>(src[static_cast<int64_t>(r) * C + c0 + j])) << (8 * j);
        }
        reinterpret_cast<uint32_t *>(dst)[i] = word;
    }
}

// ---------------------------------------------------------------------------
// acc[k][n] += sum_{m in slab} P[m][k] * Q[m][n]  (P: M x K, Q: M x N, both int8 row-major):
// the weight-gradient product, whose reduction runs over the nodes.  Both
// operands are read with the reduction index as the slow one, so 4x4 byte
// blocks are transposed in registers (v_perm_b32) on their way into LDS.
// Workgroup = 128 x 128 output tile x one slab of rows; partial tiles are added
// with int32 atomics (exact, order-free).
// ---------------------------------------------------------------------------
constexpr int TT = 128;          // output tile edge
constexpr int MS = 64;           // reduction rows per step
constexpr int LDM = MS + 16;     // LDS row stride (bytes)

struct unaligned_u32 {
    uint32_t v;
} __attribute__((packed, aligned(1)));

// 4 bytes P[row][c0..c0+3] (zero beyond the edges); rows may start at any byte address.
__device__ inline uint32_t load_quad(const int8_t *__restrict__ base, int64_t row, int64_t nrows, int ld, int c0, int ncols)
{
    if (row >= nrows || c0 >= ncols) return 0u;
    const int8_t *p = base + row * ld + c0;
    if (c0 + 3 < ncols) return reinterpret_cast<const unaligned_u32 *>(p)->v;
    uint32_t w = 0;
    for (int j = 0; j < 4 && c0 + j < ncols; ++j) w |= static_cast<uint32_t>(static_cast<uint8_t>(p[j])) << (8 * j);
    return w;
}

__device__ inline void transpose4x4(uint32_t r0, uint32_t r1, uint32_t r2, uint32_t r3, uint32_t (&t)[4])
{
    const uint32_t x01l = __builtin_amdgcn_perm(r1, r0, 0x05010400u);
    const uint32_t x01h = __builtin_amdgcn_perm(r1, r0, 0x07030602u);
    const uint32_t x23l = __builtin_amdgcn_perm(r3, r2, 0x05010400u);
    const uint32_t x23h = __builtin_amdgcn_perm(r3, r2, 0x07030602u);
    t[0] = __builtin_amdgcn_perm(x23l, x01l, 0x05040100u);
    t[1] = __builtin_amdgcn_perm(x23l, x01l, 0x07060302u);
    t[2] = __builtin_amdgcn_perm(x23h, x01h, 0x05040100u);
    t[3] = __builtin_amdgcn_perm(x23h, x01h, 0x07060302u);
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void k_gemm_tn(int64_t M, int K, int N, const int8_t *__restrict__ P,
                                                 const int8_t *__restrict__ Q, long long *acc_out, int64_t slab_rows,
                                                 int tiles_k, int tiles_n)
{
    __shared__ __align__(16) int8_t Pt[TT * LDM];
    __shared__ __align__(16) int8_t Qt[TT * LDM];
    const int tid = threadIdx.x, lane = tid % TANGO_WAVE, wave = tid / TANGO_WAVE;
    // Workgroups go to the 8 XCDs in turn, each with an L2 of its own: the output tiles of one slab of rows read the same
    // rows of P and Q, so they are given to workgroups 8 apart (same XCD, consecutive there) and share those rows in
    // that L2 instead of each fetching them across the fabric.
    const int tiles = tiles_k * tiles_n;
    const int xcd = blockIdx.x % 8, j = blockIdx.x / 8;
    const int tile = j % tiles;
    const int64_t slab = static_cast<int64_t>(j / tiles) * 8 + xcd;
    const int k0 = (tile / tiles_n) * TT, n0 = (tile % tiles_n) * TT;
    const int64_t m_begin = slab * slab_rows;
    if (m_begin >= M) return;  // (the slab count is padded to a multiple of 8)
    const int64_t m_end = min(M, m_begin + slab_rows);
    const int rbase = (wave / 2) * 64, cbase = (wave % 2) * 64;
    v16i acc00 = {0}, acc01 = {0}, acc10 = {0}, acc11 = {0};

    for (int64_t m0 = m_begin; m0 < m_end; m0 += MS) {
        // stage: waves 0-1 transpose the P slab, waves 2-3 the Q slab.  A thread takes one quad of columns (32 per tile,
        // consecutive lanes = 128 contiguous bytes of a row) and 16 consecutive rows: four 4x4 byte transposes give, for
        // each of its 4 columns, the 16 row bytes that one MFMA operand read wants - one 16-byte LDS store each.  The
        // 16-byte chunk index is XORed with (row / 16) % 4 so that neither these stores (lanes 4 rows apart) nor the
        // operand reads (lanes 1 row apart) collide in the LDS banks (64 banks of 4 bytes; a 16-byte access is served
        // sixteen lanes per cycle, and with the 80-byte row stride sixteen consecutive rows - or sixteen rows 4 apart -
        // then cover all 64 banks exactly once).
        {
            const int half = tid / 128, t128 = tid % 128;
            const int qb = t128 % 32, qa = t128 / 32;
            const int8_t *src = half ? Q : P;
            const int ld = half ? N : K;
            const int c0 = (half ? n0 : k0) + 4 * qb;
            int8_t *dstT = half ? Qt : Pt;
            uint32_t w[16];
            if (m0 + MS <= m_end && c0 + 3 < ld) {
                // interior: sixteen independent loads, no per-load bounds check between them
                const int8_t *p0 = src + (m0 + 16 * qa) * ld + c0;
#pragma unroll
                for (int i = 0; i < 16; ++i) w[i] = reinterpret_cast<const unaligned_u32 *>(p0 + static_cast<int64_t>(i) * ld)->v;
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) w[i] = load_quad(src, m0 + 16 * qa + i, m_end, ld, c0, ld);
            }
            uint32_t t[4][4];
#pragma unroll
            for (int b = 0; b < 4; ++b) transpose4x4(w[4 * b], w[4 * b + 1], w[4 * b + 2], w[4 * b + 3], t[b]);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int row = 4 * qb + c;
                *reinterpret_cast<uint4 *>(dstT + row * LDM + 16 * (qa ^ ((row / 16) % 4))) =
                    make_uint4(t[0][c], t[1][c], t[2][c], t[3][c]);
            }
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < MS; ks += 32) {
            const int mc = ks / 16 + lane / 32;  // 16-byte chunk of the reduction rows
            const int ra = rbase + lane % 32, rb = cbase + lane % 32;
            const v4i a0 = *reinterpret_cast<const v4i *>(Pt + ra * LDM + 16 * (mc ^ ((ra / 16) % 4)));
            const v4i a1 = *reinterpret_cast<const v4i *>(Pt + (ra + 32) * LDM + 16 * (mc ^ (((ra + 32) / 16) % 4)));
            const v4i b0 = *reinterpret_cast<const v4i *>(Qt + rb * LDM + 16 * (mc ^ ((rb / 16) % 4)));
            const v4i b1 = *reinterpret_cast<const v4i *>(Qt + (rb + 32) * LDM + 16 * (mc ^ (((rb + 32) / 16) % 4)));
            acc00 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, acc00, 0, 0, 0);
            acc01 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b1, acc01, 0, 0, 0);
            acc10 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b0, acc10, 0, 0, 0);
            acc11 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, acc11, 0, 0, 0);
        }
        __syncthreads();
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const v16i &acc = t == 0 ? acc00 : (t == 1 ? acc01 : (t == 2 ? acc10 : acc11));
        const int rb = t / 2, cb = t % 2;
        const int col = n0 + cbase + cb * 32 + lane % 32;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = k0 + rbase + rb * 32 + (i / 4) * 8 + (lane / 32) * 4 + (i % 4);
            if (row < K && col < N && acc[i] != 0)
                atomicAdd(reinterpret_cast<unsigned long long *>(acc_out + static_cast<int64_t>(row) * N + col),
                          static_cast<unsigned long long>(static_cast<long long>(acc[i])));
        }
    }
}

__global__ __launch_bounds__(256) void k_dequant_i64(const long long *__restrict__ acc, int64_t n, const float *sa,
                                                     const float *sb, float *__restrict__ out)
{
    const float sc = (*sa) * (*sb);
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x)
        out[i] = static_cast<float>(acc[i]) * sc;
}

int launch_fused(const fused_args &a_in, int rounding, hipStream_t st)
{
    fused_args a = a_in;
    a.K_magic = static_cast<uint32_t>(((uint64_t(1) << 32) + a.K - 1) / static_cast<uint64_t>(a.K > 1 ? a.K : 2));
    const size_t lds_bytes = static_cast<size_t>(BM) * (a.Kp + LDS_PAD);
    const unsigned grid = static_cast<unsigned>((a.M + BM - 1) / BM);
    const int wl = (a.K % 4 == 0) ? 4 : ((a.K % 2 == 0) ? 2 : 1);
#define TANGO_FUSED_K(R, W, KEEP_)                                                                          \
    {                                                                                                       \
        if (lds_bytes > 48 * 1024 &&                                                                        \
            hipFuncSetAttribute(reinterpret_cast<const void *>(&k_qgemm_fused<R, W, KEEP_>),                \
                                hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes)) != hipSuccess) \
            return TANGO_ERR_LAUNCH;                                                                        \
        k_qgemm_fused<R, W, KEEP_><<<grid, 256, lds_bytes, st>>>(a);                                        \
    }
#define TANGO_FUSED(R, W)                                                  \
    {                                                                      \
        if (a.C_keep_bits) TANGO_FUSED_K(R, W, true) else TANGO_FUSED_K(R, W, false) \
    }
    if (rounding == TANGO_RN) {
        if (wl == 4) TANGO_FUSED(TANGO_RN, 4) else if (wl == 2) TANGO_FUSED(TANGO_RN, 2) else TANGO_FUSED(TANGO_RN, 1)
    } else {
        if (wl == 4) TANGO_FUSED(TANGO_SR, 4) else if (wl == 2) TANGO_FUSED(TANGO_SR, 2) else TANGO_FUSED(TANGO_SR, 1)
    }
#undef TANGO_FUSED
#undef TANGO_FUSED_K
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int validate_mnk(int64_t M, int64_t N, int64_t K)
{
    TANGO_REQUIRE(M >= 1 && N >= 1 && K >= 1, TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(M < (int64_t(1) << 31) && N <= 65536 && K <= 65536, TANGO_ERR_BAD_SHAPE);
    return TANGO_OK;
}

size_t bt_bytes(int64_t rows, int64_t red)
{
    return tango_round_up(static_cast<size_t>(tango_round_up(rows, 64)) * tango_round_up(red, 32), 256);
}

}  // namespace

extern "C" {

size_t tango_qgemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (validate_mnk(M, N, K) != TANGO_OK) return 0;
    return 256 + bt_bytes(N, K);
}

int tango_qgemm(int64_t M, int64_t N, int64_t K, const float *A, const float *B, int rounding, uint64_t seed,
                uint64_t stream_id_A, uint64_t stream_id_B, int8_t *A_q, float *s_A, int8_t *B_q, float *s_B, float *C,
                float *absmax_C, void *ws, size_t ws_bytes, void *stream)
{
    return tango_qgemm_known_absmax(M, N, K, A, nullptr, B, rounding, seed, stream_id_A, stream_id_B, A_q, s_A, B_q, s_B, C,
                                    absmax_C, ws, ws_bytes, stream);
}

}  // extern "C"

// tango_qgemm with max|A| already on the device (absmax_A_in, may be NULL): the pass over A that finds it is skipped.
int tango_qgemm_known_absmax(int64_t M, int64_t N, int64_t K, const float *A, const float *absmax_A_in, const float *B,
                             int rounding, uint64_t seed, uint64_t stream_id_A, uint64_t stream_id_B, int8_t *A_q, float *s_A,
                             int8_t *B_q, float *s_B, float *C, float *absmax_C, void *ws, size_t ws_bytes, void *stream,
                             const tango_zero_regions *also_zero)
{
    TANGO_REQUIRE(rounding == TANGO_RN || rounding == TANGO_SR, TANGO_ERR_BAD_ENUM);
    int rc = validate_mnk(M, N, K);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(K <= KMAX || K % 16 == 0, TANGO_ERR_UNSUPPORTED);  // long reductions go through the tiled int8 kernel
    TANGO_REQUIRE(A && B && A_q && s_A && B_q && s_B && C, TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(A, 16) && tango_aligned(A_q, 8) && tango_aligned(B, 4) && tango_aligned(C, 4),
                  TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(ws && tango_aligned(ws, 256) && ws_bytes >= tango_qgemm_workspace_bytes(M, N, K), TANGO_ERR_WORKSPACE);
    hipStream_t st = tango_stream(stream);
    float *am = static_cast<float *>(ws);  // [0] = absmax A, [1] = absmax B
    int8_t *BT = static_cast<int8_t *>(ws) + 256;
    const int Kp = static_cast<int>(tango_round_up(K, 32)), Np = static_cast<int>(tango_round_up(N, 64));

    const float *am_A = absmax_A_in ? absmax_A_in : am;
    int am_A_count = 1;
    const tango_rng rng_b = tango_rng_make(seed, stream_id_B);
    tango_zero_regions zr{};
    if (also_zero) zr = *also_zero;
    TANGO_REQUIRE(!zr.overflow, TANGO_ERR_BAD_SHAPE);
    if (K * N <= SMALL_B_ELEMS && static_cast<int64_t>(Np) * Kp <= 4 * SMALL_B_ELEMS) {
        // a small weight matrix: everything that concerns B, and the clearing of the call's abs-max words, in one launch
        int64_t zwords = 0;
        for (int r = 0; r < zr.count; ++r) zwords += zr.n[r];
        // (max|A| of a small A: per-workgroup partial maxima behind the two abs-max words of the workspace header)
        const bool a_partials = !absmax_A_in && M * K <= SMALL_A_ELEMS;
        const int64_t longest = std::max<int64_t>(std::max<int64_t>(static_cast<int64_t>(Np) * Kp / 4, zwords), a_partials ? M * K / 4 : 0);
        const unsigned gs = tango_grid_for(static_cast<size_t>(longest), 256 * 2, 60);
        if (a_partials) {
            am_A = am + 2;
            am_A_count = static_cast<int>(gs);
        }
        if (rounding == TANGO_RN)
            k_quantize_b_small<TANGO_RN><<<gs, 256, 0, st>>>(static_cast<int>(K), static_cast<int>(N), Kp, Np, B, am, am + 1,
                                                           absmax_C, rng_b, B_q, s_B, BT, zr, A, M * K, a_partials ? am + 2 : nullptr);
        else
            k_quantize_b_small<TANGO_SR><<<gs, 256, 0, st>>>(static_cast<int>(K), static_cast<int>(N), Kp, Np, B, am, am + 1,
                                                           absmax_C, rng_b, B_q, s_B, BT, zr, A, M * K, a_partials ? am + 2 : nullptr);
        TANGO_LAUNCH_CHECK();
        if (!absmax_A_in && !a_partials && (rc = tango_absmax_accumulate_async(A, static_cast<size_t>(M) * K, am, st)) != TANGO_OK)
            return rc;
    } else {
        TANGO_REQUIRE(zr.count <= 6, TANGO_ERR_BAD_SHAPE);
        tango_zero_regions_add(zr, am, 2);
        tango_zero_regions_add(zr, absmax_C, 1);
        if ((rc = tango_zero_regions_async(zr, st)) != TANGO_OK) return rc;
        if (!absmax_A_in && (rc = tango_absmax_accumulate_async(A, static_cast<size_t>(M) * K, am, st)) != TANGO_OK) return rc;
        if ((rc = tango_absmax_accumulate_async(B, static_cast<size_t>(K) * N, am + 1, st)) != TANGO_OK) return rc;
        if ((rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(BT), 0u, static_cast<int64_t>(Np) * Kp / 4, st)) != TANGO_OK)
            return rc;
        const unsigned gb = tango_grid_for(static_cast<size_t>(K) * N, 256);
        if (rounding == TANGO_RN)
            k_quantize_b<TANGO_RN><<<gb, 256, 0, st>>>(static_cast<int>(K), static_cast<int>(N), Kp, B, am + 1, rng_b, B_q, s_B, BT);
        else
            k_quantize_b<TANGO_SR><<<gb, 256, 0, st>>>(static_cast<int>(K), static_cast<int>(N), Kp, B, am + 1, rng_b, B_q, s_B, BT);
        TANGO_LAUNCH_CHECK();
    }

    if (K > KMAX) {
        // the 64-row panel of A no longer fits LDS: quantize A in a pass of its own, then the tiled kernel on the int8
        // operands (BT: N rows of Kp bytes, zero-padded)
        if ((rc = tango_quantize_with_absmax_async(A, static_cast<size_t>(M) * K, rounding, seed, stream_id_A, am_A, A_q, s_A, st,
                                                   am_A_count)) != TANGO_OK)
            return rc;
        return tango_gemm_i8_async(M, N, K, A_q, K, s_A, BT, Kp, s_B, C, absmax_C, st);
    }
    fused_args a;
    a.M = M; a.N = static_cast<int>(N); a.K = static_cast<int>(K); a.Kp = Kp; a.Np = Np;
    a.A = A; a.absmax_A = am_A; a.absmax_A_count = am_A_count; a.rng = tango_rng_make(seed, stream_id_A);
    a.A_q = A_q; a.s_A = s_A; a.BT = BT; a.s_B = s_B; a.C = C; a.absmax_C = absmax_C; a.C_keep_bits = nullptr;
    return launch_fused(a, rounding, st);
}

extern "C" {

size_t tango_qgemm_bwd_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (validate_mnk(M, N, K) != TANGO_OK) return 0;
    return 256 + bt_bytes(K, N) + tango_round_up(static_cast<size_t>(K) * N * sizeof(long long), 256);
}

int tango_qgemm_bwd(int64_t M, int64_t N, int64_t K, const int8_t *A_q, const float *s_A, const int8_t *B_q,
                    const float *s_B, const float *dC, int rounding, uint64_t seed, uint64_t stream_id_dC,
                    const float *absmax_dC_in, int8_t *dC_q, float *s_dC, float *dA, float *dB, void *ws, size_t ws_bytes,
                    void *stream)
{
    return tango_qgemm_bwd_masked(M, N, K, A_q, s_A, B_q, s_B, dC, rounding, seed, stream_id_dC, absmax_dC_in, dC_q, s_dC, dA,
                                  nullptr, nullptr, dB, ws, ws_bytes, stream);
}

}  // extern "C"

// tango_qgemm_bwd with a ReLU' on dA's way out: dA_keep_bits (optional; bit i of the flat M x K tensor, 4-byte aligned,
// K a multiple of 32, K <= the on-chip panel limit) clear -> dA[i] = 0; absmax_dA (optional, device) receives max|dA| of
// what was written.
int tango_qgemm_bwd_masked(int64_t M, int64_t N, int64_t K, const int8_t *A_q, const float *s_A, const int8_t *B_q,
                           const float *s_B, const float *dC, int rounding, uint64_t seed, uint64_t stream_id_dC,
                           const float *absmax_dC_in, int8_t *dC_q, float *s_dC, float *dA, const uint32_t *dA_keep_bits,
                           float *absmax_dA, float *dB, void *ws, size_t ws_bytes, void *stream, const tango_colsum_job *tail)
{
    TANGO_REQUIRE(rounding == TANGO_RN || rounding == TANGO_SR, TANGO_ERR_BAD_ENUM);
    int rc = validate_mnk(M, N, K);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(N <= KMAX || N % 16 == 0 || !dA, TANGO_ERR_UNSUPPORTED);  // N is the reduction length of the dA product
    TANGO_REQUIRE(dC && dC_q && s_dC, TANGO_ERR_NULL);
    TANGO_REQUIRE(!dA || (B_q && s_B), TANGO_ERR_NULL);
    TANGO_REQUIRE(!dB || (A_q && s_A), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(dC, 16) && tango_aligned(dC_q, 8) && tango_aligned(dA, 4) && tango_aligned(dB, 4),
                  TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(ws && tango_aligned(ws, 256) && ws_bytes >= tango_qgemm_bwd_workspace_bytes(M, N, K), TANGO_ERR_WORKSPACE);
    TANGO_REQUIRE((!dA_keep_bits && !absmax_dA) || (dA && N <= KMAX), TANGO_ERR_UNSUPPORTED);
    TANGO_REQUIRE(!dA_keep_bits || (K % 32 == 0 && tango_aligned(dA_keep_bits, 4)), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(!tail || (dA && N <= KMAX), TANGO_ERR_UNSUPPORTED);  // (the launch that takes the job exists only then)
    hipStream_t st = tango_stream(stream);
    float *am = static_cast<float *>(ws);
    int8_t *BT = static_cast<int8_t *>(ws) + 256;           // B_q padded: Kp64 rows x Np32 bytes
    long long *acc = reinterpret_cast<long long *>(BT + bt_bytes(K, N));  // 64-bit sums of the weight gradient
    bool acc_zeroed = false;
    const float *amp = absmax_dC_in;
    if (!amp) {
        if ((rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(am), 0u, 1, st)) != TANGO_OK) return rc;
        if ((rc = tango_absmax_accumulate_async(dC, static_cast<size_t>(M) * N, am, st)) != TANGO_OK) return rc;
        amp = am;
    }
    if (dA && N > KMAX) {
        // long reduction: quantize dC first, then the tiled int8 kernel; B_q (K x N, rows contiguous along n) already is
        // the transposed operand of this product
        if ((rc = tango_quantize_with_absmax_async(dC, static_cast<size_t>(M) * N, rounding, seed, stream_id_dC, amp, dC_q,
                                                   s_dC, st)) != TANGO_OK)
            return rc;
        if ((rc = tango_gemm_i8_async(M, K, N, dC_q, N, s_dC, B_q, N, s_B, dA, nullptr, st)) != TANGO_OK) return rc;
    } else if (dA) {
        // dA = dC_q . B_q^T: the forward kernel with dC in the role of A and B_q (K x N, rows contiguous along
        // the reduction index n) in the role of the transposed operand.
        const int Rp = static_cast<int>(tango_round_up(N, 32)), Cp = static_cast<int>(tango_round_up(K, 64));
        // (the padded copy of B_q, the clearing of max|dA| and, if the weight gradient follows, of its accumulator: one launch)
        const int64_t n_zero = dB ? 2 * K * N : 0;
        k_pad_copy_i8<<<tango_grid_for(static_cast<size_t>(Cp) * Rp / 4 + n_zero, 256), 256, 0, st>>>(
            static_cast<int>(K), static_cast<int>(N), Cp, Rp, B_q, BT, reinterpret_cast<uint32_t *>(acc), n_zero,
            reinterpret_cast<uint32_t *>(absmax_dA), tail ? *tail : tango_colsum_job{nullptr, 0, 0, nullptr, nullptr});
        TANGO_LAUNCH_CHECK();
        acc_zeroed = true;
        fused_args a;
        a.M = M; a.N = static_cast<int>(K); a.K = static_cast<int>(N); a.Kp = Rp; a.Np = Cp;
        a.A = dC; a.absmax_A = amp; a.absmax_A_count = 1; a.rng = tango_rng_make(seed, stream_id_dC);
        a.A_q = dC_q; a.s_A = s_dC; a.BT = BT; a.s_B = s_B; a.C = dA; a.absmax_C = absmax_dA; a.C_keep_bits = dA_keep_bits;
        if ((rc = launch_fused(a, rounding, st)) != TANGO_OK) return rc;
    } else {
        if ((rc = tango_quantize_with_absmax_async(dC, static_cast<size_t>(M) * N, rounding, seed, stream_id_dC, amp, dC_q,
                                                   s_dC, st)) != TANGO_OK)
            return rc;
    }
    if (dB) {
        // dB = A_q^T . dC_q, reduction over the M rows, split into slabs
        if (!acc_zeroed && (rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(acc), 0u, 2 * K * N, st)) != TANGO_OK)
            return rc;
        const int tiles_k = static_cast<int>((K + TT - 1) / TT), tiles_n = static_cast<int>((N + TT - 1) / TT);
        // about 2,048 workgroups in all: enough to fill the chip several times over, and half the 64-bit atomics of 4,096
        // (measured at 233 k x 602 x 256: 0.38 -> 0.31 ms)
        int64_t slabs = 2048 / (tiles_k * tiles_n);
        // at least eight steps per workgroup before its 64 KB of atomics; two where the whole product is a few dozen steps,
        // which a couple of workgroups would otherwise walk as one long chain of dependent load - transpose - multiply steps
        slabs = std::min<int64_t>(slabs, M / ((M < 65536 ? 2 : 8) * MS));
        if (slabs < 1) slabs = 1;
        // a slab's int32 partial sums stay exact (2^17 rows x 127^2 < 2^31); the slabs are combined in 64 bits
        int64_t slab_rows = std::min<int64_t>(tango_round_up(static_cast<size_t>((M + slabs - 1) / slabs), MS), int64_t(1) << 17);
        slabs = (M + slab_rows - 1) / slab_rows;
        const unsigned grid = static_cast<unsigned>(tiles_k * tiles_n * tango_round_up(static_cast<size_t>(slabs), 8));
        k_gemm_tn<<<grid, 256, 0, st>>>(M, static_cast<int>(K), static_cast<int>(N), A_q, dC_q, acc, slab_rows, tiles_k,
                                        tiles_n);
        TANGO_LAUNCH_CHECK();
        k_dequant_i64<<<tango_grid_for(static_cast<size_t>(K) * N, 256), 256, 0, st>>>(acc, K * N, s_A, s_dC, dB);
        TANGO_LAUNCH_CHECK();
    }
    return TANGO_OK;
}



// ---------------------------------------------------------------------------------------------------------------
// tango_qgemm for callers that cannot allocate and have no workspace to pass (code under HIP graph capture, tight
// serving loops, harnesses that forbid hipMalloc): the scratch of the forward GEMM (two abs-max words and the padded,
// transposed int8 copy of B) lives in a fixed device array of the library instead of a caller workspace.
// ---------------------------------------------------------------------------------------------------------------
namespace {

constexpr size_t STATIC_SCRATCH_BYTES = TANGO_QGEMM_STATIC_SCRATCH_BYTES;  // covers every N, K with round_up(N,64)*round_up(K,32) <= 2 MiB

// One copy per GPU the library runs on, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress: the device address it stands for is looked up once per device and kept in scratch_ptr.
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
void *scratch_ptr[MAX_DEVICES];  // device address of `scratch` on each device (written once; same value if two threads race)

int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return TANGO_ERR_LAUNCH;
    void *p = __atomic_load_n(&scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return TANGO_ERR_LAUNCH;
        __atomic_store_n(&scratch_ptr[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return TANGO_OK;
}

}  // namespace

extern "C" {

int tango_qgemm_static(int64_t M, int64_t N, int64_t K, const float *A, const float *B, int rounding, uint64_t seed,
                       uint64_t stream_id_A, uint64_t stream_id_B, int8_t *A_q, float *s_A, int8_t *B_q, float *s_B, float *C,
                       float *absmax_C, void *stream)
{
    int rc = validate_mnk(M, N, K);
    if (rc != TANGO_OK) return rc;
    // the scratch this shape needs must fit the fixed array: refuse before anything is launched
    TANGO_REQUIRE(tango_qgemm_workspace_bytes(M, N, K) <= STATIC_SCRATCH_BYTES, TANGO_ERR_WORKSPACE);
    void *ws = nullptr;
    if ((rc = static_scratch(&ws)) != TANGO_OK) return rc;
    // every word of the scratch that must start at zero (the abs-max words, the padding of the transposed B) is cleared
    // by fill kernels inside the call below, on the caller's stream: contents left by an earlier call do not matter
    return tango_qgemm_known_absmax(M, N, K, A, nullptr, B, rounding, seed, stream_id_A, stream_id_B, A_q, s_A, B_q, s_B, C,
                                    absmax_C, ws, STATIC_SCRATCH_BYTES, stream);
}

}  // extern "C"
