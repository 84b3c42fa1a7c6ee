// Stochastic-rounding quantizer whose random bits come from xoshiro256++ generators with their state in registers
// (Sec. 3.2 "GPU-accelerated stochastic rounding"), as an alternative to the counter-based bits of tango_quantize.
// A generator with state cannot be addressed per element, so the mapping is part of the definition: 65,536
// generators = 65,536 threads; generator g is seeded with four splitmix64 outputs from
// x0 = seed + stream_id*0xD1342543DE82EF95 + g*0x9E3779B97F4A7C15; its j-th 64-bit output serves elements
// 4v .. 4v+3 (16 bits each, lowest first) of group v = j*65536 + g.  A thread therefore reads one float4 and
// writes 4 bytes per output: coalesced, HBM stream of 4 + 1 bytes per element.
#include "internal.hip.h"

namespace {

constexpr unsigned XO_GENERATORS = 65536;

__device__ inline uint64_t rotl64(uint64_t x, int k) { return (x << k) | (x >> (64 - k)); }

__device__ inline uint64_t splitmix64(uint64_t &x)
{
    uint64_t z = (x += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ __launch_bounds__(256) void k_quantize_xoshiro(const float *__restrict__ x, size_t n, const float *__restrict__ absmax,
                                                          uint64_t seed, uint64_t stream_id, int8_t *__restrict__ q,
                                                          float *scale_out)
{
    float s, inv;
    tango_scale_from_absmax(*absmax, s, inv);
    if (blockIdx.x == 0 && threadIdx.x == 0 && scale_out) *scale_out = s;
    const uint64_t g = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;  // the grid is exactly 65,536 threads
    uint64_t x0 = seed + stream_id * 0xD1342543DE82EF95ull + g * 0x9E3779B97F4A7C15ull;
    uint64_t s0 = splitmix64(x0), s1 = splitmix64(x0), s2 = splitmix64(x0), s3 = splitmix64(x0);
    const uint64_t groups = (static_cast<uint64_t>(n) + 3) / 4;
    auto next = [&]() {
        const uint64_t r = rotl64(s0 + s3, 23) + s0;
        const uint64_t t = s1 << 17;
        s2 ^= s0;
        s3 ^= s1;
        s1 ^= s2;
        s0 ^= s3;
        s2 ^= t;
        s3 = rotl64(s3, 45);
        return r;
    };
    auto code = [&](float xv, uint64_t r, int j) {
        return static_cast<uint32_t>(tango_round_clamp<TANGO_SR>(xv * inv, static_cast<uint32_t>(r >> (16 * j)) & 0xffffu)) & 0xffu;
    };
    // a thread owns only every 65,536-th group, so it keeps UNR independent loads in flight to cover the memory latency
    constexpr int UNR = 8;
    uint64_t v = g;
    for (; v + static_cast<uint64_t>(UNR - 1) * XO_GENERATORS < groups && 4 * (v + static_cast<uint64_t>(UNR - 1) * XO_GENERATORS) + 4 <= n;
         v += static_cast<uint64_t>(UNR) * XO_GENERATORS) {
        float4 a[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) a[u] = *reinterpret_cast<const float4 *>(x + 4 * (v + static_cast<uint64_t>(u) * XO_GENERATORS));
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const uint64_t r = next();
            *reinterpret_cast<uint32_t *>(q + 4 * (v + static_cast<uint64_t>(u) * XO_GENERATORS)) =
                code(a[u].x, r, 0) | (code(a[u].y, r, 1) << 8) | (code(a[u].z, r, 2) << 16) | (code(a[u].w, r, 3) << 24);
        }
    }
    for (; v < groups; v += XO_GENERATORS) {
        const uint64_t r = next();
        const uint64_t i = 4 * v;
        if (i + 4 <= n) {
            const float4 a = *reinterpret_cast<const float4 *>(x + i);
            *reinterpret_cast<uint32_t *>(q + i) = code(a.x, r, 0) | (code(a.y, r, 1) << 8) | (code(a.z, r, 2) << 16) | (code(a.w, r, 3) << 24);
        } else {
            for (int j = 0; j < 4 && i + j < n; ++j) q[i + j] = static_cast<int8_t>(static_cast<int>(code(x[i + j], r, j) << 24) >> 24);
        }
    }
}

}  // namespace

extern "C" {

int tango_quantize_xoshiro(const float *x, size_t n, uint64_t seed, uint64_t stream_id, const float *absmax_in, int8_t *q,
                           float *scale_out, void *ws, size_t ws_bytes, void *stream)
{
    TANGO_REQUIRE(n == 0 || (x != nullptr && q != nullptr), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(x, 16) && tango_aligned(q, 4), TANGO_ERR_BAD_SHAPE);
    hipStream_t st = tango_stream(stream);
    const float *am = absmax_in;
    if (am == nullptr) {
        TANGO_REQUIRE(ws != nullptr && ws_bytes >= 256 && tango_aligned(ws, 256), TANGO_ERR_WORKSPACE);
        float *wam = static_cast<float *>(ws);
        int rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(wam), 0u, 1, st);
        if (rc != TANGO_OK) return rc;
        rc = tango_absmax_accumulate_async(x, n, wam, st);
        if (rc != TANGO_OK) return rc;
        am = wam;
    }
    k_quantize_xoshiro<<<XO_GENERATORS / 256, 256, 0, st>>>(x, n, am, seed, stream_id, q, scale_out);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

}  // extern "C"
