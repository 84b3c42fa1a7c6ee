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

template <int GS>
__device__ inline float group_max(float v)
{
#pragma unroll
    for (int o = GS / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
template <int GS>
__device__ inline float group_sum(float v)
{
#pragma unroll
    for (int o = GS / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
template <int GS>
__device__ inline double group_sum(double v)
{
#pragma unroll
    for (int o = GS / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Hand rows to lane groups: op.run<GS>(row, begin, end, lane_in_group) is called by all GS lanes of a group.
template <int GROUP, class Op>
__device__ inline void walk_rows(const int32_t *__restrict__ ptr, int n, Op &op)
{
    const int lane = threadIdx.x % TANGO_WAVE;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) / TANGO_WAVE;
    const int nwaves = gridDim.x * blockDim.x / TANGO_WAVE;
    constexpr int RPI = 64 / GROUP;  // rows per wave-iteration
    for (int64_t base = static_cast<int64_t>(wave) * 64; base < n; base += static_cast<int64_t>(nwaves) * 64) {
        const int r = static_cast<int>(base) + lane;
        int b = 0, t = 0;
        if (r < n) {
            b = ptr[r];
            t = ptr[r + 1];
        }
        const int is_long = (GROUP == 64) ? 1 : ((t - b) > 16 * GROUP ? 1 : 0);
        if (GROUP < 64) {
            for (int k = 0; k < GROUP; ++k) {
                const int src = k * RPI + lane / GROUP;
                const int rb = __shfl(b, src, 64), rt = __shfl(t, src, 64), lg = __shfl(is_long, src, 64);
                const int row = static_cast<int>(base) + src;
                if (row < n && !lg) op.template run<GROUP>(row, rb, rt, lane % GROUP);
            }
        }
        unsigned long long mask = __ballot(r < n && is_long);
        while (mask) {
            const int k = __ffsll(static_cast<long long>(mask)) - 1;
            mask &= mask - 1;
            const int rb = __shfl(b, k, 64), rt = __shfl(t, k, 64);
            op.template run<64>(static_cast<int>(base) + k, rb, rt, lane);
        }
    }
}

inline int pick_group(int n, int64_t nnz)
{
    const double avg = n > 0 ? static_cast<double>(nnz) / n : 0.0;
    if (avg <= 12.0) return 8;
    if (avg <= 24.0) return 16;
    if (avg <= 48.0) return 32;
    return 64;
}

inline unsigned row_grid(int n) { return tango_grid_for((static_cast<size_t>(n) + 63) / 64, 4, 256 * 8); }

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
