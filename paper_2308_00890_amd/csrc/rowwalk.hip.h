// Row-walking skeleton shared by the streaming edge kernels: rows (nodes) are handed out in blocks of 64
// consecutive rows per wavefront; short rows are processed by groups of GROUP lanes (GROUP ~ the mean
// degree), rows longer than 16*GROUP by the whole wave, one lane per edge with all heads of that edge.
#pragma once

#include "internal.hip.h"

namespace {

template <int H>
__device__ inline void load_h(const float *p, float (&v)[H])
{
    if constexpr (H == 4) {
        const float4 t = *reinterpret_cast<const float4 *>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else if constexpr (H == 2) {
        const float2 t = *reinterpret_cast<const float2 *>(p);
        v[0] = t.x; v[1] = t.y;
    } else {
#pragma unroll
        for (int h = 0; h < H; ++h) v[h] = p[h];
    }
}

template <int H>
__device__ inline void store_h(float *p, const float (&v)[H])
{
    if constexpr (H == 4) {
        *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    } else if constexpr (H == 2) {
        *reinterpret_cast<float2 *>(p) = make_float2(v[0], v[1]);
    } else {
#pragma unroll
        for (int h = 0; h < H; ++h) p[h] = v[h];
    }
}

// A team = the lanes (or threads) that share one row.  lane_team<GS>: GS consecutive lanes of a wave,
// reductions by cross-lane shuffles.  block_team: every thread of the workgroup, reductions through LDS
// (deterministic: partial results are combined in wave order).
template <int GS>
struct lane_team {
    int rank;
    __device__ int size() const { return GS; }
    __device__ float max(float v) const
    {
#pragma unroll
        for (int o = GS / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
        return v;
    }
    __device__ float sum(float v) const
    {
#pragma unroll
        for (int o = GS / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
        return v;
    }
    __device__ double sum(double v) const
    {
#pragma unroll
        for (int o = GS / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
        return v;
    }
    // combine online-softmax states (maximum m, sum s of exp(x - m))
    __device__ void merge_ms(float &m, float &s) const
    {
#pragma unroll
        for (int o = GS / 2; o > 0; o >>= 1) {
            const float m2 = __shfl_xor(m, o, 64), s2 = __shfl_xor(s, o, 64);
            const float M = fmaxf(m, m2);
            const float f1 = (m == M) ? 1.0f : __expf(m - M);
            const float f2 = (m2 == M) ? 1.0f : __expf(m2 - M);
            s = s * f1 + s2 * f2;
            m = M;
        }
    }
};

constexpr int TEAM_BLOCK_THREADS = 1024;

struct block_team {
    int rank;
    double *scratch;  // 2 * (blockDim.x / 64) doubles of LDS
    __device__ int size() const { return blockDim.x; }
    __device__ double sum(double v) const
    {
        const lane_team<64> w{0};
        v = w.sum(v);
        const int nw = blockDim.x / 64;
        if (threadIdx.x % 64 == 0) scratch[threadIdx.x / 64] = v;
        __syncthreads();
        double t = 0.0;
        for (int i = 0; i < nw; ++i) t += scratch[i];
        __syncthreads();
        return t;
    }
    __device__ float sum(float v) const { return static_cast<float>(sum(static_cast<double>(v))); }
    __device__ float max(float v) const
    {
        const lane_team<64> w{0};
        v = w.max(v);
        const int nw = blockDim.x / 64;
        if (threadIdx.x % 64 == 0) scratch[threadIdx.x / 64] = static_cast<double>(v);
        __syncthreads();
        float t = static_cast<float>(scratch[0]);
        for (int i = 1; i < nw; ++i) t = fmaxf(t, static_cast<float>(scratch[i]));
        __syncthreads();
        return t;
    }
    __device__ void merge_ms(float &m, float &s) const
    {
        const lane_team<64> w{0};
        w.merge_ms(m, s);
        const int nw = blockDim.x / 64;
        if (threadIdx.x % 64 == 0) {
            scratch[2 * (threadIdx.x / 64)] = static_cast<double>(m);
            scratch[2 * (threadIdx.x / 64) + 1] = static_cast<double>(s);
        }
        __syncthreads();
        float M = static_cast<float>(scratch[0]), S = static_cast<float>(scratch[1]);
        for (int i = 1; i < nw; ++i) {
            const float m2 = static_cast<float>(scratch[2 * i]), s2 = static_cast<float>(scratch[2 * i + 1]);
            const float MM = fmaxf(M, m2);
            const float f1 = (M == MM) ? 1.0f : __expf(M - MM);
            const float f2 = (m2 == MM) ? 1.0f : __expf(m2 - MM);
            S = S * f1 + s2 * f2;
            M = MM;
        }
        __syncthreads();
        m = M;
        s = S;
    }
};

// Rows longer than this are not processed by one wave but appended to a list and handled by whole
// workgroups in a second kernel (hub rows would otherwise serialise the tail of the launch).
constexpr int HUGE_ROW = 4096;

inline size_t huge_list_bytes(int64_t nnz) { return tango_round_up(static_cast<size_t>(nnz / HUGE_ROW + 2) * sizeof(int), 256); }

// Hand rows to lane teams: op.run(row, begin, end, team) is called by all lanes of the team.
// huge: NULL, or a list (huge[0] = count, zero-initialised; huge[1..] = rows) that receives rows longer than
// HUGE_ROW instead of processing them here.
// first_block, skip_huge: the launch's workgroups below first_block do something else (walk_huge_rows_strided) and the
// rows longer than HUGE_ROW are theirs: skipped here, no list.
// rows_per_wave (groups of fewer than 64 lanes only; a power of two, 64 / GROUP <= rows_per_wave <= 64): the rows a wave
// takes per outer iteration - fewer on small graphs, so that more waves share them.
template <int GROUP, class Op>
__device__ inline void walk_rows(const int32_t *__restrict__ ptr, int n, Op &op, int *huge = nullptr, int first_block = 0,
                                 bool skip_huge = false, int rows_per_wave = 64)
{
    const int lane = threadIdx.x % TANGO_WAVE;
    // readfirstlane / readlane: the wave index and the bounds of a row taken by the whole wave are wave-uniform, and
    // saying so keeps them (and the loops over a row's edges) in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(
        static_cast<int>(((blockIdx.x - first_block) * blockDim.x + threadIdx.x) / TANGO_WAVE));
    const int nwaves = (gridDim.x - first_block) * blockDim.x / TANGO_WAVE;
    constexpr int RPI = 64 / GROUP;  // rows per wave-iteration
    // rows a wave takes per outer iteration: with a whole wave per row they are walked one after the other, each with
    // its own chain of dependent loads, so fewer rows per wave (more waves) hide more of that latency
    const int ROWS = GROUP == 64 ? 4 : rows_per_wave;
    for (int64_t base = static_cast<int64_t>(wave) * ROWS; base < n; base += static_cast<int64_t>(nwaves) * ROWS) {
        const int r = (lane < ROWS) ? static_cast<int>(base) + lane : n;
        int b = 0, t = 0;
        if (r < n) {
            b = ptr[r];
            t = ptr[r + 1];
        }
        int is_long = (GROUP == 64) ? 1 : ((t - b) > 16 * GROUP ? 1 : 0);
        if ((huge || skip_huge) && r < n && (t - b) > HUGE_ROW) {
            if (huge) huge[1 + atomicAdd(huge, 1)] = r;
            is_long = 2;  // neither a group nor this wave processes it
        }
        if (GROUP < 64) {
            for (int k = 0; k * RPI < ROWS; ++k) {
                const int src = k * RPI + lane / GROUP;
                const int rb = __shfl(b, src, 64), rt = __shfl(t, src, 64), lg = __shfl(is_long, src, 64);
                const int row = static_cast<int>(base) + src;
                if (row < n && !lg) op.run(row, rb, rt, lane_team<GROUP>{lane % GROUP});
            }
        }
        unsigned long long mask = __ballot(r < n && is_long == 1);
        while (mask) {
            const int k = __ffsll(static_cast<long long>(mask)) - 1;
            mask &= mask - 1;
            const int rb = __builtin_amdgcn_readlane(b, k), rt = __builtin_amdgcn_readlane(t, k);
            op.run(static_cast<int>(base) + k, rb, rt, lane_team<64>{lane});
        }
    }
}

// Second kernel body: one workgroup per listed row.
template <class Op>
__device__ inline void walk_huge_rows(const int32_t *__restrict__ ptr, const int *huge, Op &op, double *scratch)
{
    const int count = huge[0];
    for (int i = blockIdx.x; i < count; i += gridDim.x) {
        const int row = huge[1 + i];
        op.run(row, ptr[row], ptr[row + 1], block_team{static_cast<int>(threadIdx.x), scratch});
    }
}

// The same without a list, inside the launch that walks the other rows: workgroup j of nblocks looks at the rows
// j, j + nblocks, ... (strided, so that hubs clustered at neighbouring ids spread over the workgroups), collects those
// longer than HUGE_ROW, up to one per thread and round, in LDS (list: blockDim.x + 1 ints) and takes them one by one.
template <class Op>
__device__ inline void walk_huge_rows_strided(const int32_t *__restrict__ ptr, int n, int j, int nblocks, Op &op,
                                              double *scratch, int *list)
{
    for (int64_t r0 = j; r0 < n; r0 += static_cast<int64_t>(nblocks) * blockDim.x) {
        if (threadIdx.x == 0) list[0] = 0;
        __syncthreads();
        const int64_t r = r0 + static_cast<int64_t>(threadIdx.x) * nblocks;
        if (r < n && ptr[r + 1] - ptr[r] > HUGE_ROW) list[1 + atomicAdd(&list[0], 1)] = static_cast<int>(r);
        __syncthreads();
        const int count = list[0];
        for (int i = 0; i < count; ++i) {
            const int row = list[1 + i];
            op.run(row, ptr[row], ptr[row + 1], block_team{static_cast<int>(threadIdx.x), scratch});
        }
        __syncthreads();
    }
}

constexpr unsigned HUGE_GRID = 2048;

// Rows per wave for walk_rows with groups of `group` lanes: 64, or fewer (down to one per group) while the graph has
// fewer than 2,048 waves' worth of rows.
inline int pick_rows_per_wave(int n, int group)
{
    if (group >= 64) return 64;
    int rows = 64;
    while (rows > 64 / group && static_cast<int64_t>(n) / rows < 2048) rows /= 2;
    return rows;
}

inline int pick_group(int n, int64_t nnz)
{
    const double avg = n > 0 ? static_cast<double>(nnz) / n : 0.0;
    // (measured on the softmax statistics pass: with rows of 17-26 edges groups of 8 lanes beat 16 and 32 - more rows in
    // flight per wave matter more than one pass per row)
    if (avg <= 32.0) return 8;
    if (avg <= 64.0) return 16;
    if (avg <= 128.0) return 32;
    return 64;
}

// group = lanes per row as picked by pick_group (walk_rows hands a wave 16 rows per iteration when a row takes the
// whole wave, else 64)
inline unsigned row_grid(int n, int group = 0, int rows_per_wave = 64)
{
    const size_t rows = group == 64 ? 4 : rows_per_wave;
    return tango_grid_for((static_cast<size_t>(n) + rows - 1) / rows, 4, 256 * 16);
}

// Dispatch a kernel template K<H, GROUP> over the supported head counts and group sizes.
#define TANGO_DISPATCH_HG(H_, G_, CALL)                         \
    switch (G_) {                                               \
        case 8: { constexpr int GROUP = 8; CALL(H_); } break;   \
        case 16: { constexpr int GROUP = 16; CALL(H_); } break; \
        case 32: { constexpr int GROUP = 32; CALL(H_); } break; \
        default: { constexpr int GROUP = 64; CALL(H_); } break; \
    }

#define TANGO_DISPATCH_H(heads, G_, CALL)                      \
    switch (heads) {                                           \
        case 1: TANGO_DISPATCH_HG(1, G_, CALL) break;          \
        case 2: TANGO_DISPATCH_HG(2, G_, CALL) break;          \
        case 3: TANGO_DISPATCH_HG(3, G_, CALL) break;          \
        case 4: TANGO_DISPATCH_HG(4, G_, CALL) break;          \
        case 8: TANGO_DISPATCH_HG(8, G_, CALL) break;          \
        default: return TANGO_ERR_UNSUPPORTED;                 \
    }

inline bool heads_supported(int heads) { return heads == 1 || heads == 2 || heads == 3 || heads == 4 || heads == 8; }


}  // namespace
