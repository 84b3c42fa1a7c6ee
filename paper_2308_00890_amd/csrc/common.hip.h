// Device and host helpers shared by the kernels of the library (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tango.h"

#define TANGO_WAVE 64

#define TANGO_REQUIRE(cond, err) \
    do {                         \
        if (!(cond)) return (err); \
    } while (0)

// Launch check: never synchronises; reports a refused launch only.
#define TANGO_LAUNCH_CHECK()                                   \
    do {                                                       \
        if (hipGetLastError() != hipSuccess) return TANGO_ERR_LAUNCH; \
    } while (0)

static inline hipStream_t tango_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

static inline bool tango_aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

static inline size_t tango_round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Grid size for a grid-stride kernel: enough workgroups to fill 256 CUs several times over.
static inline unsigned tango_grid_for(size_t work_items, unsigned per_block, unsigned max_blocks = 256 * 16)
{
    size_t b = (work_items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > max_blocks) b = max_blocks;
    return static_cast<unsigned>(b);
}

// Up to eight runs of 32-bit words to clear (accumulators and abs-max words that a later kernel of the same chain adds
// to): passed by value to the one kernel that clears them, so that several clears cost one launch.
struct tango_zero_regions {
    uint32_t *p[8];
    int64_t n[8];  // words in each run; unused entries hold 0
    int count;
    int overflow;  // set when a ninth run was asked for: the launch that would clear the list is refused
};

static inline void tango_zero_regions_add(tango_zero_regions &z, void *p, int64_t words)
{
    if (!p || words <= 0) return;
    if (z.count >= 8) {
        z.overflow = 1;
        return;
    }
    z.p[z.count] = static_cast<uint32_t *>(p);
    z.n[z.count] = words;
    ++z.count;
}

// Thread `tid` of `nthreads` takes its share of every run.
__device__ static inline void tango_zero_regions_apply(const tango_zero_regions &z, int64_t tid, int64_t nthreads)
{
    for (int r = 0; r < z.count; ++r)
        for (int64_t i = tid; i < z.n[r]; i += nthreads) z.p[r][i] = 0u;
}

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): counter-based random
// bits for stochastic rounding (Sec. 3.2 "GPU-accelerated stochastic
// rounding" asks for a register-resident generator; a counter-based one adds
// independence from the thread mapping).
// ---------------------------------------------------------------------------
struct tango_rng {
    uint32_t k0, k1;  // key = 64-bit seed
    uint32_t s0, s1;  // stream id -> counter words 2, 3
};

__host__ __device__ static inline tango_rng tango_rng_make(uint64_t seed, uint64_t stream_id)
{
    tango_rng r;
    r.k0 = static_cast<uint32_t>(seed);
    r.k1 = static_cast<uint32_t>(seed >> 32);
    r.s0 = static_cast<uint32_t>(stream_id);
    r.s1 = static_cast<uint32_t>(stream_id >> 32);
    return r;
}

// The 128-bit block that serves flat elements 8*blk .. 8*blk+7 (16 bits each).
__device__ static inline uint4 tango_philox_block(const tango_rng &r, uint64_t blk)
{
    uint32_t c0 = static_cast<uint32_t>(blk), c1 = static_cast<uint32_t>(blk >> 32), c2 = r.s0, c3 = r.s1;
    uint32_t k0 = r.k0, k1 = r.k1;
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c0;
        const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c2;
        const uint32_t n0 = static_cast<uint32_t>(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = static_cast<uint32_t>(p0 >> 32) ^ c3 ^ k1;
        c1 = static_cast<uint32_t>(p1);
        c3 = static_cast<uint32_t>(p0);
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return make_uint4(c0, c1, c2, c3);
}

// 16 random bits of element `lane8` (0..7) of a block.
__device__ static inline uint32_t tango_bits16(const uint4 b, int lane8)
{
    // two selects and one 64-bit shift (written without any indexing so that the block stays in registers)
    const uint32_t lo = (lane8 & 4) ? b.z : b.x;
    const uint32_t hi = (lane8 & 4) ? b.w : b.y;
    const uint64_t half = (static_cast<uint64_t>(hi) << 32) | lo;
    return static_cast<uint32_t>(half >> (16 * (lane8 & 3))) & 0xffffu;
}

// Scale rule (Sec. 2.3, symmetric per-tensor, B = 8): s = absmax/127, inv = 127/absmax.
__device__ static inline void tango_scale_from_absmax(float absmax, float &s, float &inv)
{
    if (absmax > 0.0f) {
        s = absmax / 127.0f;
        inv = 127.0f / absmax;
    } else {
        s = 1.0f;
        inv = 0.0f;
    }
}

// One element: y = x*inv already formed.  Nearest-even or Eq. 3 with u = bits*2^-16.
template <int ROUNDING>
__device__ static inline int tango_round_clamp(float y, uint32_t bits16)
{
    int v;
    if (ROUNDING == TANGO_RN) {
        v = static_cast<int>(rintf(y));
    } else {
        const float f = floorf(y);
        const float frac = y - f;
        const float u = static_cast<float>(bits16) * (1.0f / 65536.0f);
        v = static_cast<int>(f) + (u < frac ? 1 : 0);
    }
    return min(127, max(-127, v));
}

// Quantize 8 consecutive elements (one Philox block) held in y[8] = x*inv.
template <int ROUNDING>
__device__ static inline uint2 tango_quantize8(const float (&y)[8], const tango_rng &rng, uint64_t blk)
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

// ---------------------------------------------------------------------------
// Wave-level reductions (wave64) via cross-lane shuffles.
// ---------------------------------------------------------------------------
// Sum over aligned groups of n adjacent lanes (n a power of two), result in every lane of the group.  Up to 16
// lanes the partner values come through DPP modifiers of VALU moves (quad permutes, then mirrored halves and rows -
// after the earlier steps all lanes of a half hold the same value, so a mirror is as good as an xor); only wider
// groups use LDS-pipe shuffles.  Must be called by all 64 lanes.
__device__ static inline int tango_group_sum(int d, int n)
{
    if (n >= 2) d += __builtin_amdgcn_update_dpp(0, d, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
    if (n >= 4) d += __builtin_amdgcn_update_dpp(0, d, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
    if (n >= 8) d += __builtin_amdgcn_update_dpp(0, d, 0x141, 0xF, 0xF, true);   // row_half_mirror
    if (n >= 16) d += __builtin_amdgcn_update_dpp(0, d, 0x140, 0xF, 0xF, true);  // row_mirror
    for (int off = 16; off < n; off <<= 1) d += __shfl_xor(d, off, 64);
    return d;
}

// The same with the group size known at compile time (N = 0: not known, use n): no branches in the caller's loop.
template <int N>
__device__ static inline int tango_group_sum_c(int d, int n)
{
    if (N == 0) return tango_group_sum(d, n);
    if (N >= 2) d += __builtin_amdgcn_update_dpp(0, d, 0xB1, 0xF, 0xF, true);
    if (N >= 4) d += __builtin_amdgcn_update_dpp(0, d, 0x4E, 0xF, 0xF, true);
    if (N >= 8) d += __builtin_amdgcn_update_dpp(0, d, 0x141, 0xF, 0xF, true);
    if (N >= 16) d += __builtin_amdgcn_update_dpp(0, d, 0x140, 0xF, 0xF, true);
#pragma unroll
    for (int off = 16; off < N; off <<= 1) d += __shfl_xor(d, off, 64);
    return d;
}

// Sum of a double over aligned groups of n adjacent lanes (n a power of two), result in every lane of the group: the
// same additions as an xor-shuffle tree (the mirrored partners hold the value the xor partner holds), but up to 16
// lanes through DPP moves of the two halves instead of LDS-pipe shuffles.  Must be called by all 64 lanes.
__device__ static inline double tango_group_sum_f64(double v, int n)
{
#define TANGO_DPP_ADD_F64(CTRL)                                                                           \
    {                                                                                                     \
        const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, true);           \
        const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, true);           \
        v += __hiloint2double(hi, lo);                                                                    \
    }
    if (n >= 2) TANGO_DPP_ADD_F64(0xB1)    // quad_perm [1,0,3,2]
    if (n >= 4) TANGO_DPP_ADD_F64(0x4E)    // quad_perm [2,3,0,1]
    if (n >= 8) TANGO_DPP_ADD_F64(0x141)   // row_half_mirror
    if (n >= 16) TANGO_DPP_ADD_F64(0x140)  // row_mirror
#undef TANGO_DPP_ADD_F64
    for (int off = 16; off < n; off <<= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Sum of a double over the lanes of a wave that share lane % stride (stride a power of two, wave-uniform), result in
// every lane: rotations inside the rows of 16 lanes through DPP moves of the two halves, then two xor shuffles.
// Must be called by all 64 lanes.
__device__ static inline double tango_stride_sum_f64(double v, int stride)
{
#define TANGO_DPP_ROR_ADD_F64(CTRL)                                                                       \
    {                                                                                                     \
        const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, true);           \
        const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, true);           \
        v += __hiloint2double(hi, lo);                                                                    \
    }
    if (stride <= 1) TANGO_DPP_ROR_ADD_F64(0x121)  // row_ror:1
    if (stride <= 2) TANGO_DPP_ROR_ADD_F64(0x122)  // row_ror:2
    if (stride <= 4) TANGO_DPP_ROR_ADD_F64(0x124)  // row_ror:4
    if (stride <= 8) TANGO_DPP_ROR_ADD_F64(0x128)  // row_ror:8
#undef TANGO_DPP_ROR_ADD_F64
    if (stride <= 16) v += __shfl_xor(v, 16, 64);
    if (stride <= 32) v += __shfl_xor(v, 32, 64);
    return v;
}

__device__ static inline float tango_wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

__device__ static inline float tango_wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ static inline double tango_wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// The last step of the head-projection backward (step 2'): da_src[c], da_dst[c] = the sums over `copies` partial
// accumulators of 2F doubles.  A few hundred additions: done by one workgroup of whatever launch follows in the chain
// instead of in a launch of its own.
struct tango_colsum_job {
    const double *acc;  // NULL: nothing to do
    int F, copies;
    float *da_src, *da_dst;
};

__device__ static inline void tango_colsum_apply(const tango_colsum_job &j)
{
    if (!j.acc) return;
    for (int c = threadIdx.x; c < j.F; c += blockDim.x) {
        double ts = 0.0, td = 0.0;
        for (int k = 0; k < j.copies; ++k) {
            ts += j.acc[static_cast<size_t>(k) * 2 * j.F + c];
            td += j.acc[static_cast<size_t>(k) * 2 * j.F + j.F + c];
        }
        j.da_src[c] = static_cast<float>(ts);
        j.da_dst[c] = static_cast<float>(td);
    }
}

// An abs-max handed from one kernel to the next is either one word (count == 1) or `count` partial maxima, one per
// workgroup of the producing launch (no atomics, and so no launch that clears their target first); every lane returns
// the maximum.  count <= 64.
__device__ static inline float tango_absmax_load(const float *p, int count)
{
    if (count == 1) return *p;
    const int lane = threadIdx.x % TANGO_WAVE;
    return tango_wave_max(lane < count ? p[lane] : 0.0f);
}

// max over non-negative floats through their bit patterns (monotone for x >= 0).
// The running maximum only grows, so a value that is not above what a plain load already sees cannot change it and
// needs no atomic: thousands of waves ending with an atomic on one address would otherwise queue up behind each other
// (about 10 ns each, measured).  The load is a device-scope atomic load so that it sees the other XCDs' updates.
__device__ static inline void tango_atomic_max_nonneg(float *addr, float v)
{
    const unsigned int bits = __float_as_uint(v);
    if (bits > __hip_atomic_load(reinterpret_cast<const unsigned int *>(addr), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        atomicMax(reinterpret_cast<unsigned int *>(addr), bits);
}

// *addr = max(*addr, max of m over the workgroup): one update per workgroup.  (Per-wave updates all read the scalar with
// device scope first; when the waves of a launch finish together those reads queue at one L2 channel.)  Must be
// reached by every thread of the workgroup; blockDim.x a multiple of 64, at most 1024.
__device__ static inline void tango_block_max_update(float m, float *addr)
{
    __shared__ float tango_block_max_part[16];
    m = tango_wave_max(m);
    if (threadIdx.x % TANGO_WAVE == 0) tango_block_max_part[threadIdx.x / TANGO_WAVE] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (unsigned w = 1; w < blockDim.x / TANGO_WAVE; ++w) m = fmaxf(m, tango_block_max_part[w]);
        if (m > 0.0f) tango_atomic_max_nonneg(addr, m);
    }
    __syncthreads();
}

