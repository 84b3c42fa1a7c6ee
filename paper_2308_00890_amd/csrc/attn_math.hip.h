// The attention arithmetic shared by every kernel of the fused path, so that the forward pass, the
// statistics pass and both backward passes form bit-identical fp32 values (Sec. 2.1 steps 3 and 4):
//   t     = s_S*S_q[u][h] + s_D*D_q[v][h]          (two fp32 products, one fp32 sum)
//   E     = t > 0 ? t : slope*t                    (LeakyReLU)
//   alpha = exp(E - row_lse)                       (row_lse = log of the row's sum of exp(E): max + log(sum exp(E - max)))
// exp is the hardware exponential (v_exp_f32 on x*log2(e)); its relative error, about 1e-7*(1+|x|), is far
// inside the fp32 tolerance of the softmax.
#pragma once

#include "internal.hip.h"

__device__ static inline float tango_attn_exp(float x) { return __expf(x); }

__device__ static inline float tango_attn_score(float ts, float td, float slope, bool &positive)
{
    const float x = ts + td;
    positive = x > 0.0f;
    return positive ? x : slope * x;
}

__device__ static inline float tango_attn_alpha(float ev, float row_lse) { return tango_attn_exp(ev - row_lse); }

// The `heads` int8 values of one node (heads <= 8) as sign-extended ints; one vector load when heads is 2, 4 or 8
// (the table must then be aligned to `heads` bytes).
template <int H>
__device__ static inline void tango_load_heads(const int8_t *__restrict__ table, int64_t node, int (&v)[H])
{
    const int8_t *p = table + node * H;
    if constexpr (H == 4) {
        const uint32_t w = *reinterpret_cast<const uint32_t *>(p);
#pragma unroll
        for (int h = 0; h < 4; ++h) v[h] = static_cast<int>(static_cast<int8_t>(w >> (8 * h)));
    } else if constexpr (H == 2) {
        const uint16_t w = *reinterpret_cast<const uint16_t *>(p);
        v[0] = static_cast<int>(static_cast<int8_t>(w & 0xff));
        v[1] = static_cast<int>(static_cast<int8_t>(w >> 8));
    } else if constexpr (H == 8) {
        const uint2 w = *reinterpret_cast<const uint2 *>(p);
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            v[h] = static_cast<int>(static_cast<int8_t>(w.x >> (8 * h)));
            v[4 + h] = static_cast<int>(static_cast<int8_t>(w.y >> (8 * h)));
        }
    } else {
#pragma unroll
        for (int h = 0; h < H; ++h) v[h] = static_cast<int>(p[h]);
    }
}

// The reverse: the H codes in v become entry `node` of a table (aligned like the table of tango_load_heads).
template <int H>
__device__ static inline void tango_store_heads(int8_t *__restrict__ table, int64_t node, const int (&v)[H])
{
    int8_t *p = table + node * H;
    if constexpr (H == 4 || H == 8) {
        uint32_t w[H / 4];
#pragma unroll
        for (int q = 0; q < H / 4; ++q) {
            w[q] = 0;
#pragma unroll
            for (int h = 0; h < 4; ++h) w[q] |= (static_cast<uint32_t>(v[4 * q + h]) & 0xffu) << (8 * h);
        }
        if constexpr (H == 4)
            *reinterpret_cast<uint32_t *>(p) = w[0];
        else
            *reinterpret_cast<uint2 *>(p) = make_uint2(w[0], w[1]);
    } else if constexpr (H == 2) {
        *reinterpret_cast<uint16_t *>(p) = static_cast<uint16_t>((static_cast<uint32_t>(v[0]) & 0xffu) | ((static_cast<uint32_t>(v[1]) & 0xffu) << 8));
    } else {
#pragma unroll
        for (int h = 0; h < H; ++h) p[h] = static_cast<int8_t>(v[h]);
    }
}

// Heads h0 .. h0+3 of a node (run-time head count; entries at or beyond `heads` are left zero).
__device__ static inline void tango_load_heads4(const int8_t *__restrict__ table, int64_t node, int heads, int h0, int (&v)[4])
{
    const int8_t *p = table + node * heads + h0;
    if ((heads & 3) == 0) {
        const uint32_t w = *reinterpret_cast<const uint32_t *>(p);
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = static_cast<int>(static_cast<int8_t>(w >> (8 * j)));
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (h0 + j < heads) ? static_cast<int>(p[j]) : 0;
    }
}

// Per (destination, head) record gathered by the source-side backward pass: everything that pass needs of the
// destination in 16 bytes.  The table has tango_rec_heads(heads) records per node (heads rounded up to a power of two),
// so the records of one node are one aligned run of 16, 32, 64 or 128 bytes: lanes that fetch one record each, with the
// heads of an edge in adjacent lanes, touch one such run per edge.
struct __attribute__((aligned(16))) tango_attn_rec {
    double P;        // sum over the in-edges of dalpha*alpha
    float row_lse;   // log-sum-exp of the destination's scores
    int32_t dq;      // the destination's quantized projection D_q[v][h]
};
__host__ __device__ static inline int tango_rec_heads(int heads) { return heads <= 1 ? 1 : heads <= 2 ? 2 : heads <= 4 ? 4 : 8; }
