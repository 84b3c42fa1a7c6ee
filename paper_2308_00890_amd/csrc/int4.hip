// 4-bit operands (Sec. 4 "Speed impact for # of quantization bits"): the same symmetric per-tensor quantizer with
// codes in [-7, 7] (s = absmax/7, inv = 7/absmax), stored two per byte - element 2j in the low nibble, 2j+1 in the
// high nibble, each a 4-bit two's-complement number.  Rounding rules and random bits per element are those of the
// 8-bit quantizer (one Philox block per 8 consecutive elements), so one thread-iteration turns 8 floats into 4 bytes.
// HBM stream: 4 bytes read + 0.5 byte written per element.
#include "internal.hip.h"

namespace {

template <int ROUNDING>
__device__ inline int round_clamp7(float y, uint32_t bits16)
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
    return min(7, max(-7, v));
}

template <int ROUNDING>
__global__ __launch_bounds__(256) void k_quantize_i4(const float *__restrict__ x, size_t n, const float *__restrict__ absmax,
                                                     tango_rng rng, uint8_t *__restrict__ q4, float *scale_out)
{
    const float am = *absmax;
    float s = 1.0f, inv = 0.0f;
    if (am > 0.0f) {
        s = am / 7.0f;
        inv = 7.0f / am;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0 && scale_out) *scale_out = s;
    const size_t n8 = n / 8;
    const size_t tid = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const size_t nthr = static_cast<size_t>(gridDim.x) * blockDim.x;
    const float4 *x4 = reinterpret_cast<const float4 *>(x);
    uint32_t *out = reinterpret_cast<uint32_t *>(q4);
    for (size_t i = tid; i < n8; i += nthr) {
        const float4 a = x4[2 * i];
        const float4 b = x4[2 * i + 1];
        const float y[8] = {a.x * inv, a.y * inv, a.z * inv, a.w * inv, b.x * inv, b.y * inv, b.z * inv, b.w * inv};
        uint4 blk = make_uint4(0, 0, 0, 0);
        if (ROUNDING == TANGO_SR) blk = tango_philox_block(rng, i);
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            word |= (static_cast<uint32_t>(round_clamp7<ROUNDING>(y[j], tango_bits16(blk, j))) & 0xfu) << (4 * j);
        out[i] = word;
    }
    // ragged tail: an even number (< 8) of elements, one thread
    if (tid == 0 && n8 * 8 < n) {
        uint4 blk = make_uint4(0, 0, 0, 0);
        if (ROUNDING == TANGO_SR) blk = tango_philox_block(rng, n8);
        for (size_t j = n8 * 8; j < n; j += 2) {
            const uint32_t lo = static_cast<uint32_t>(round_clamp7<ROUNDING>(x[j] * inv, tango_bits16(blk, static_cast<int>(j & 7)))) & 0xfu;
            const uint32_t hi = static_cast<uint32_t>(round_clamp7<ROUNDING>(x[j + 1] * inv, tango_bits16(blk, static_cast<int>((j + 1) & 7)))) & 0xfu;
            q4[j / 2] = static_cast<uint8_t>(lo | (hi << 4));
        }
    }
}

}  // namespace

extern "C" {

int tango_quantize_i4(const float *x, size_t n, int rounding, uint64_t seed, uint64_t stream_id, const float *absmax_in,
                      uint8_t *q4, float *scale_out, void *ws, size_t ws_bytes, void *stream)
{
    TANGO_REQUIRE(rounding == TANGO_RN || rounding == TANGO_SR, TANGO_ERR_BAD_ENUM);
    TANGO_REQUIRE(n % 2 == 0, TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(n == 0 || (x != nullptr && q4 != nullptr), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(x, 16) && tango_aligned(q4, 4), TANGO_ERR_BAD_SHAPE);
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
    if (n == 0) return TANGO_OK;
    const tango_rng rng = tango_rng_make(seed, stream_id);
    const unsigned grid = tango_grid_for(n / 8 + 1, 256 * 2);
    if (rounding == TANGO_RN)
        k_quantize_i4<TANGO_RN><<<grid, 256, 0, st>>>(x, n, am, rng, q4, scale_out);
    else
        k_quantize_i4<TANGO_SR><<<grid, 256, 0, st>>>(x, n, am, rng, q4, scale_out);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

}  // extern "C"
