// Per-tensor symmetric int8 quantization (Sec. 2.3 Eq. 1-2 with zero point 0;
// Sec. 3.2 Eq. 3 for stochastic rounding): abs-max reduction, quantize,
// dequantize.  All three are pure streaming kernels bound by HBM bandwidth:
// abs-max reads 4 B/element, quantize reads 4 B and writes 1 B per element.
#include "internal.hip.h"

namespace {

__global__ void k_fill_u32(uint32_t *p, uint32_t v, int64_t n)
{
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x)
        p[i] = v;
}

__device__ inline float4 tango_mask4(const float4 a, const float4 k)
{
    return make_float4(k.x > 0.0f ? a.x : 0.0f, k.y > 0.0f ? a.y : 0.0f, k.z > 0.0f ? a.z : 0.0f, k.w > 0.0f ? a.w : 0.0f);
}

// the same with one bit per element (bit j of `bits` for component j) instead of a float
__device__ inline float4 tango_mask4b(const float4 a, const uint32_t bits)
{
    return make_float4((bits & 1u) ? a.x : 0.0f, (bits & 2u) ? a.y : 0.0f, (bits & 4u) ? a.z : 0.0f, (bits & 8u) ? a.w : 0.0f);
}

// max|x| over n floats into *out (as the bit pattern of a non-negative float; *out must start at 0).
// VEC = 4: x is 16-byte aligned and float4 loads are used for the body.
// MASKED = 1: element i counts as 0 where mask[i] <= 0 (the gradient behind a ReLU whose output is `mask`).
// MASKED = 2: the same with mask_bits, bit i set where the ReLU's output is positive (n a multiple of 8).
template <int VEC, int MASKED = 0>
__global__ __launch_bounds__(256) void k_absmax(const float *__restrict__ x, size_t n, float *out,
                                                const float *__restrict__ mask = nullptr,
                                                const uint8_t *__restrict__ mask_bits = nullptr)
{
    float m = 0.0f;
    const size_t tid = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const size_t nthr = static_cast<size_t>(gridDim.x) * blockDim.x;
    if (VEC == 4) {
        const size_t n4 = n / 4;
        const float4 *x4 = reinterpret_cast<const float4 *>(x);
        size_t i = tid;
        // eight independent loads per iteration keep enough bytes in flight to cover the memory latency
        const float4 *k4 = reinterpret_cast<const float4 *>(mask);
        constexpr int UA = MASKED ? 4 : 8;
        for (; i + (UA - 1) * nthr < n4; i += UA * nthr) {
            float4 a[UA], k[UA];
#pragma unroll
            for (int u = 0; u < UA; ++u) {
                a[u] = x4[i + u * nthr];
                if (MASKED == 1) k[u] = k4[i + u * nthr];
                if (MASKED == 2) k[u].x = __uint_as_float(mask_bits[(i + u * nthr) >> 1]);
            }
#pragma unroll
            for (int u = 0; u < UA; ++u) {
                if (MASKED == 1) a[u] = tango_mask4(a[u], k[u]);
                if (MASKED == 2) a[u] = tango_mask4b(a[u], __float_as_uint(k[u].x) >> (4 * ((i + u * nthr) & 1)));
                m = fmaxf(m, fmaxf(fmaxf(fabsf(a[u].x), fabsf(a[u].y)), fmaxf(fabsf(a[u].z), fabsf(a[u].w))));
            }
        }
        for (; i < n4; i += nthr) {
            float4 a = x4[i];
            if (MASKED == 1) a = tango_mask4(a, k4[i]);
            if (MASKED == 2) a = tango_mask4b(a, static_cast<uint32_t>(mask_bits[i >> 1]) >> (4 * (i & 1)));
            m = fmaxf(m, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
        }
        for (size_t j = n4 * 4 + tid; j < n; j += nthr) m = fmaxf(m, (MASKED != 1 || mask[j] > 0.0f) ? fabsf(x[j]) : 0.0f);
    } else {
        for (size_t j = tid; j < n; j += nthr) m = fmaxf(m, (MASKED != 1 || mask[j] > 0.0f) ? fabsf(x[j]) : 0.0f);
    }
    m = tango_wave_max(m);
    __shared__ float part[4];
    const int wave = threadIdx.x / TANGO_WAVE, lane = threadIdx.x % TANGO_WAVE;
    if (lane == 0) part[wave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
        if (m > 0.0f) tango_atomic_max_nonneg(out, m);
    }
}

// Vector path: x 16-byte aligned, q 8-byte aligned.  One thread-iteration = 8 elements.
// (bid, nblocks: this workgroup's index among those that share the tensor - the launch may hold two tensors)
template <int ROUNDING, int MASKED = 0>
__device__ __forceinline__ void quantize_vec_body(const float *__restrict__ x, size_t n, const float *__restrict__ absmax,
                                                  const tango_rng &rng, int8_t *__restrict__ q, float *scale_out,
                                                  const float *__restrict__ mask, const uint8_t *__restrict__ mask_bits,
                                                  unsigned bid, unsigned nblocks, int absmax_count = 1)
{
    float s, inv;
    tango_scale_from_absmax(tango_absmax_load(absmax, absmax_count), s, inv);
    if (bid == 0 && threadIdx.x == 0 && scale_out) *scale_out = s;
    const size_t n8 = n / 8;
    const size_t tid = static_cast<size_t>(bid) * blockDim.x + threadIdx.x;
    const size_t nthr = static_cast<size_t>(nblocks) * blockDim.x;
    const float4 *x4 = reinterpret_cast<const float4 *>(x);
    uint2 *q8 = reinterpret_cast<uint2 *>(q);
    // four independent 32-byte pieces per iteration keep enough loads in flight to cover the memory latency
    constexpr int UNR = 4;
    size_t i = tid;
    const float4 *k4 = reinterpret_cast<const float4 *>(mask);
    for (; i + (UNR - 1) * nthr < n8; i += UNR * nthr) {
        float4 a[UNR], b[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            a[u] = x4[2 * (i + u * nthr)];
            b[u] = x4[2 * (i + u * nthr) + 1];
            if (MASKED == 1) {
                a[u] = tango_mask4(a[u], k4[2 * (i + u * nthr)]);
                b[u] = tango_mask4(b[u], k4[2 * (i + u * nthr) + 1]);
            }
            if (MASKED == 2) {
                const uint32_t kb = mask_bits[i + u * nthr];
                a[u] = tango_mask4b(a[u], kb);
                b[u] = tango_mask4b(b[u], kb >> 4);
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const float y[8] = {a[u].x * inv, a[u].y * inv, a[u].z * inv, a[u].w * inv,
                                b[u].x * inv, b[u].y * inv, b[u].z * inv, b[u].w * inv};
            q8[i + u * nthr] = tango_quantize8<ROUNDING>(y, rng, i + u * nthr);
        }
    }
    for (; i < n8; i += nthr) {
        float4 a = x4[2 * i];
        float4 b = x4[2 * i + 1];
        if (MASKED == 1) {
            a = tango_mask4(a, k4[2 * i]);
            b = tango_mask4(b, k4[2 * i + 1]);
        }
        if (MASKED == 2) {
            const uint32_t kb = mask_bits[i];
            a = tango_mask4b(a, kb);
            b = tango_mask4b(b, kb >> 4);
        }
        const float y[8] = {a.x * inv, a.y * inv, a.z * inv, a.w * inv, b.x * inv, b.y * inv, b.z * inv, b.w * inv};
        q8[i] = tango_quantize8<ROUNDING>(y, rng, i);
    }
    // ragged tail: fewer than 8 elements, one thread
    if (tid == 0 && n8 * 8 < n) {
        uint4 b = make_uint4(0, 0, 0, 0);
        if (ROUNDING == TANGO_SR) b = tango_philox_block(rng, n8);
        for (size_t j = n8 * 8; j < n; ++j) {
            const float xv = (MASKED != 1 || mask[j] > 0.0f) ? x[j] : 0.0f;
            q[j] = static_cast<int8_t>(tango_round_clamp<ROUNDING>(xv * inv, tango_bits16(b, static_cast<int>(j & 7))));
        }
    }
}

template <int ROUNDING, int MASKED = 0>
__global__ __launch_bounds__(256) void k_quantize_vec(const float *__restrict__ x, size_t n,
                                                      const float *__restrict__ absmax, tango_rng rng,
                                                      int8_t *__restrict__ q, float *scale_out,
                                                      const float *__restrict__ mask = nullptr,
                                                      const uint8_t *__restrict__ mask_bits = nullptr, int absmax_count = 1)
{
    quantize_vec_body<ROUNDING, MASKED>(x, n, absmax, rng, q, scale_out, mask, mask_bits, blockIdx.x, gridDim.x, absmax_count);
}

// partials[b] = max|x| over workgroup b's share (b < gridDim.x <= 64); the same launch clears the runs of z.
__global__ __launch_bounds__(256) void k_absmax_partials(const float *__restrict__ x, size_t n, float *__restrict__ partials,
                                                         tango_zero_regions z)
{
    __shared__ float red[4];
    const size_t tid = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x, nthr = static_cast<size_t>(gridDim.x) * 256;
    tango_zero_regions_apply(z, static_cast<int64_t>(tid), static_cast<int64_t>(nthr));
    float m = 0.0f;
    const float4 *x4 = reinterpret_cast<const float4 *>(x);
    for (size_t i = tid; i < n / 4; i += nthr) {
        const float4 v = x4[i];
        m = fmaxf(m, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
    }
    for (size_t i = n / 4 * 4 + tid; i < n; i += nthr) m = fmaxf(m, fabsf(x[i]));
    m = tango_wave_max(m);
    if (threadIdx.x % TANGO_WAVE == 0) red[threadIdx.x / TANGO_WAVE] = m;
    __syncthreads();
    if (threadIdx.x == 0) partials[blockIdx.x] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// Two tensors in one launch (the first g1 workgroups take the first): for the small tensors of a layer, whose
// quantizations would otherwise be two dependent launches of a few microseconds each.
struct quantize_job {
    const float *x;
    size_t n;
    const float *absmax;
    tango_rng rng;
    int8_t *q;
    float *scale_out;
};
template <int ROUNDING>
__global__ __launch_bounds__(256) void k_quantize_pair(quantize_job j1, quantize_job j2, unsigned g1)
{
    if (blockIdx.x < g1)
        quantize_vec_body<ROUNDING, 0>(j1.x, j1.n, j1.absmax, j1.rng, j1.q, j1.scale_out, nullptr, nullptr, blockIdx.x, g1);
    else
        quantize_vec_body<ROUNDING, 0>(j2.x, j2.n, j2.absmax, j2.rng, j2.q, j2.scale_out, nullptr, nullptr, blockIdx.x - g1,
                                       gridDim.x - g1);
}

// Scalar path for unaligned pointers: one element per thread-iteration (same results, slower).
template <int ROUNDING>
__global__ __launch_bounds__(256) void k_quantize_scalar(const float *__restrict__ x, size_t n,
                                                         const float *__restrict__ absmax, tango_rng rng,
                                                         int8_t *__restrict__ q, float *scale_out)
{
    float s, inv;
    tango_scale_from_absmax(*absmax, s, inv);
    if (blockIdx.x == 0 && threadIdx.x == 0 && scale_out) *scale_out = s;
    const size_t tid = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const size_t nthr = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t j = tid; j < n; j += nthr) {
        uint32_t bits = 0;
        if (ROUNDING == TANGO_SR) bits = tango_bits16(tango_philox_block(rng, j >> 3), static_cast<int>(j & 7));
        q[j] = static_cast<int8_t>(tango_round_clamp<ROUNDING>(x[j] * inv, bits));
    }
}

__global__ __launch_bounds__(256) void k_dequantize(const int8_t *__restrict__ q, size_t n,
                                                    const float *__restrict__ scale, float *__restrict__ x)
{
    const float s = *scale;
    const size_t tid = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const size_t nthr = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t j = tid; j < n; j += nthr) x[j] = s * static_cast<float>(q[j]);
}

// y = max(x, 0) and, optionally, max|y| (the abs-max the next layer's quantization needs)
__global__ __launch_bounds__(256) void k_relu(const float *__restrict__ x, size_t n, float *__restrict__ y, float *absmax)
{
    const size_t tid = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const size_t nthr = static_cast<size_t>(gridDim.x) * blockDim.x;
    float m = 0.0f;
    for (size_t i = tid; i < n; i += nthr) {
        const float v = fmaxf(x[i], 0.0f);
        y[i] = v;
        m = fmaxf(m, v);
    }
    if (absmax) {
        m = tango_wave_max(m);
        if (threadIdx.x % TANGO_WAVE == 0 && m > 0.0f) tango_atomic_max_nonneg(absmax, m);
    }
}

// dx = x > 0 ? dy : 0
__global__ __launch_bounds__(256) void k_relu_bwd(const float *__restrict__ x, const float *__restrict__ dy, size_t n,
                                                  float *__restrict__ dx)
{
    const size_t tid = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const size_t nthr = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t i = tid; i < n; i += nthr) dx[i] = x[i] > 0.0f ? dy[i] : 0.0f;
}

// Error_X (Sec. 3.2 Eq. 4) of up to MAX_CAND bit counts in one pass: sums[c] += |x - xq| / |x + xq + eps| with xq
// the grid point of a bits[c]-bit symmetric quantizer.  One element per thread-iteration; fp64 sums.
constexpr int MAX_CAND = 4;
struct error_x_cands {
    int n;
    int bits[MAX_CAND];
};

template <int ROUNDING>
__global__ __launch_bounds__(256) void k_error_x(const float *__restrict__ x, size_t n, const float *__restrict__ absmax,
                                                 tango_rng rng, error_x_cands cands, double *sums)
{
    const float am = *absmax;
    float s[MAX_CAND], inv[MAX_CAND], qmax[MAX_CAND];
    double acc[MAX_CAND];
#pragma unroll
    for (int c = 0; c < MAX_CAND; ++c) {
        qmax[c] = static_cast<float>((1 << ((c < cands.n ? cands.bits[c] : 8) - 1)) - 1);
        s[c] = am > 0.0f ? am / qmax[c] : 1.0f;
        inv[c] = am > 0.0f ? qmax[c] / am : 0.0f;
        acc[c] = 0.0;
    }
    const size_t tid = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const size_t nthr = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t i = tid; i < n; i += nthr) {
        const float xv = x[i];
        float u = 0.0f;
        if (ROUNDING == TANGO_SR)
            u = static_cast<float>(tango_bits16(tango_philox_block(rng, static_cast<uint64_t>(i) >> 3), static_cast<int>(i & 7))) *
                (1.0f / 65536.0f);
#pragma unroll
        for (int c = 0; c < MAX_CAND; ++c) {
            if (c < cands.n) {
                const float y = xv * inv[c];
                float v;
                if (ROUNDING == TANGO_RN) {
                    v = rintf(y);
                } else {
                    const float f = floorf(y);
                    v = f + (u < (y - f) ? 1.0f : 0.0f);
                }
                v = fminf(qmax[c], fmaxf(-qmax[c], v));
                const float xq = s[c] * v;
                acc[c] += fabs((static_cast<double>(xv) - static_cast<double>(xq)) /
                               (static_cast<double>(xv) + static_cast<double>(xq) + 0.0005));
            }
        }
    }
#pragma unroll
    for (int c = 0; c < MAX_CAND; ++c) {
        if (c < cands.n) {
            const double t = tango_wave_sum(acc[c]);
            if (threadIdx.x % TANGO_WAVE == 0 && t != 0.0) atomicAdd(sums + c, t);
        }
    }
}

// error[c] = sums[c]/n; *chosen = the first candidate below the threshold, else the last one
__global__ void k_error_x_finish(error_x_cands cands, size_t n, float threshold, const double *sums, double *error,
                                 int *chosen)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    int pick = cands.bits[cands.n - 1];
    bool found = false;
    for (int c = 0; c < cands.n; ++c) {
        const double e = n ? sums[c] / static_cast<double>(n) : 0.0;
        error[c] = e;
        if (!found && e < static_cast<double>(threshold)) {
            pick = cands.bits[c];
            found = true;
        }
    }
    if (chosen) *chosen = pick;
}

}  // namespace

// Internal (not part of the ABI): used by the other translation units.
static __global__ void k_zero2_u32(uint32_t *p1, int64_t n1, uint32_t *p2, int64_t n2)
{
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n1 + n2;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        if (i < n1)
            p1[i] = 0u;
        else
            p2[i - n1] = 0u;
    }
}

// p1[0..n1) = 0 and p2[0..n2) = 0 in one launch (either pointer may be NULL with its count ignored).
int tango_zero2_u32_async(uint32_t *p1, int64_t n1, uint32_t *p2, int64_t n2, hipStream_t st)
{
    if (!p1 || n1 < 0) n1 = 0;
    if (!p2 || n2 < 0) n2 = 0;
    if (n1 + n2 == 0) return TANGO_OK;
    k_zero2_u32<<<tango_grid_for(static_cast<size_t>(n1 + n2), 256, 256 * 64), 256, 0, st>>>(p1, n1, p2, n2);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

static __global__ void k_zero_regions(tango_zero_regions z)
{
    tango_zero_regions_apply(z, static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x,
                             static_cast<int64_t>(gridDim.x) * blockDim.x);
}

// Every run of z in one launch.
int tango_zero_regions_async(const tango_zero_regions &z, hipStream_t st)
{
    TANGO_REQUIRE(!z.overflow, TANGO_ERR_BAD_SHAPE);
    int64_t longest = 0;
    for (int r = 0; r < z.count; ++r) longest = z.n[r] > longest ? z.n[r] : longest;
    if (longest == 0) return TANGO_OK;
    k_zero_regions<<<tango_grid_for(static_cast<size_t>(longest), 256, 256 * 64), 256, 0, st>>>(z);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_fill_u32_async(uint32_t *p, uint32_t v, int64_t n, hipStream_t st)
{
    if (n <= 0) return TANGO_OK;
    k_fill_u32<<<tango_grid_for(static_cast<size_t>(n), 256, 256 * 64), 256, 0, st>>>(p, v, n);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_absmax_accumulate_async(const float *x, size_t n, float *out, hipStream_t st)
{
    if (n == 0) return TANGO_OK;
    if (tango_aligned(x, 16))
        k_absmax<4><<<tango_grid_for(n / 4 + 1, 256 * 2), 256, 0, st>>>(x, n, out);
    else
        k_absmax<1><<<tango_grid_for(n, 256 * 4), 256, 0, st>>>(x, n, out);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

// For a small tensor: per-workgroup maxima of |x| into partials[0 .. *count) (x 16-byte aligned, *count <= 64), and the
// runs of z cleared, in one launch; tango_quantize_with_absmax_async takes (partials, *count) in place of an abs-max word.
int tango_absmax_partials_async(const float *x, size_t n, float *partials, int *count, const tango_zero_regions &z, hipStream_t st)
{
    TANGO_REQUIRE(!z.overflow && tango_aligned(x, 16), TANGO_ERR_BAD_SHAPE);
    int64_t longest = static_cast<int64_t>(n / 4);
    for (int r = 0; r < z.count; ++r) longest = z.n[r] > longest ? z.n[r] : longest;
    const unsigned nb = tango_grid_for(static_cast<size_t>(longest), 256 * 2, 64);
    k_absmax_partials<<<nb, 256, 0, st>>>(x, n, partials, z);
    TANGO_LAUNCH_CHECK();
    *count = static_cast<int>(nb);
    return TANGO_OK;
}

int tango_quantize_with_absmax_async(const float *x, size_t n, int rounding, uint64_t seed, uint64_t stream_id,
                                     const float *absmax, int8_t *q, float *scale_out, hipStream_t st, int absmax_count)
{
    const tango_rng rng = tango_rng_make(seed, stream_id);
    TANGO_REQUIRE(absmax_count >= 1 && absmax_count <= 64, TANGO_ERR_BAD_SHAPE);
    if (tango_aligned(x, 16) && tango_aligned(q, 8)) {
        const unsigned grid = tango_grid_for(n / 8 + 1, 256 * 2);
        if (rounding == TANGO_RN)
            k_quantize_vec<TANGO_RN><<<grid, 256, 0, st>>>(x, n, absmax, rng, q, scale_out, nullptr, nullptr, absmax_count);
        else
            k_quantize_vec<TANGO_SR><<<grid, 256, 0, st>>>(x, n, absmax, rng, q, scale_out, nullptr, nullptr, absmax_count);
    } else {
        TANGO_REQUIRE(absmax_count == 1, TANGO_ERR_BAD_SHAPE);  // (partial maxima are only handed to the vector path)
        const unsigned grid = tango_grid_for(n + 1, 256 * 8);
        if (rounding == TANGO_RN)
            k_quantize_scalar<TANGO_RN><<<grid, 256, 0, st>>>(x, n, absmax, rng, q, scale_out);
        else
            k_quantize_scalar<TANGO_SR><<<grid, 256, 0, st>>>(x, n, absmax, rng, q, scale_out);
    }
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

// Two quantizations with known abs-max values in one launch (falls back to two launches for unaligned tensors).
int tango_quantize_pair_with_absmax_async(const float *x1, size_t n1, uint64_t stream_id1, const float *absmax1, int8_t *q1,
                                          float *scale1, const float *x2, size_t n2, uint64_t stream_id2, const float *absmax2,
                                          int8_t *q2, float *scale2, int rounding, uint64_t seed, hipStream_t st)
{
    if (!(tango_aligned(x1, 16) && tango_aligned(q1, 8) && tango_aligned(x2, 16) && tango_aligned(q2, 8))) {
        int rc = tango_quantize_with_absmax_async(x1, n1, rounding, seed, stream_id1, absmax1, q1, scale1, st);
        if (rc != TANGO_OK) return rc;
        return tango_quantize_with_absmax_async(x2, n2, rounding, seed, stream_id2, absmax2, q2, scale2, st);
    }
    const quantize_job j1{x1, n1, absmax1, tango_rng_make(seed, stream_id1), q1, scale1};
    const quantize_job j2{x2, n2, absmax2, tango_rng_make(seed, stream_id2), q2, scale2};
    const unsigned g1 = tango_grid_for(n1 / 8 + 1, 256 * 2), g2 = tango_grid_for(n2 / 8 + 1, 256 * 2);
    if (rounding == TANGO_RN)
        k_quantize_pair<TANGO_RN><<<g1 + g2, 256, 0, st>>>(j1, j2, g1);
    else
        k_quantize_pair<TANGO_SR><<<g1 + g2, 256, 0, st>>>(j1, j2, g1);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

// q = quantize(x where mask > 0, else 0) with its own abs-max (found here into ws[0]); x, mask 16-byte and q 8-byte aligned.
int tango_quantize_masked_async(const float *x, const float *mask, size_t n, int rounding, uint64_t seed, uint64_t stream_id,
                                int8_t *q, float *scale_out, float *absmax_ws, hipStream_t st)
{
    int rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(absmax_ws), 0u, 1, st);
    if (rc != TANGO_OK) return rc;
    if (n == 0) return tango_quantize_with_absmax_async(x, n, rounding, seed, stream_id, absmax_ws, q, scale_out, st);
    k_absmax<4, 1><<<tango_grid_for(n / 4 + 1, 256 * 2), 256, 0, st>>>(x, n, absmax_ws, mask);
    TANGO_LAUNCH_CHECK();
    const tango_rng rng = tango_rng_make(seed, stream_id);
    const unsigned grid = tango_grid_for(n / 8 + 1, 256 * 2);
    if (rounding == TANGO_RN)
        k_quantize_vec<TANGO_RN, 1><<<grid, 256, 0, st>>>(x, n, absmax_ws, rng, q, scale_out, mask);
    else
        k_quantize_vec<TANGO_SR, 1><<<grid, 256, 0, st>>>(x, n, absmax_ws, rng, q, scale_out, mask);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

// The same with the ReLU's sign bits (bit i set where output i is positive) in place of the output; n a multiple of 8.
int tango_quantize_bitmasked_async(const float *x, const uint8_t *mask_bits, size_t n, int rounding, uint64_t seed,
                                   uint64_t stream_id, int8_t *q, float *scale_out, float *absmax_ws, hipStream_t st)
{
    TANGO_REQUIRE(n % 8 == 0, TANGO_ERR_BAD_SHAPE);
    int rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(absmax_ws), 0u, 1, st);
    if (rc != TANGO_OK) return rc;
    if (n == 0) return tango_quantize_with_absmax_async(x, n, rounding, seed, stream_id, absmax_ws, q, scale_out, st);
    k_absmax<4, 2><<<tango_grid_for(n / 4 + 1, 256 * 2), 256, 0, st>>>(x, n, absmax_ws, nullptr, mask_bits);
    TANGO_LAUNCH_CHECK();
    const tango_rng rng = tango_rng_make(seed, stream_id);
    const unsigned grid = tango_grid_for(n / 8 + 1, 256 * 2);
    if (rounding == TANGO_RN)
        k_quantize_vec<TANGO_RN, 2><<<grid, 256, 0, st>>>(x, n, absmax_ws, rng, q, scale_out, nullptr, mask_bits);
    else
        k_quantize_vec<TANGO_SR, 2><<<grid, 256, 0, st>>>(x, n, absmax_ws, rng, q, scale_out, nullptr, mask_bits);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

extern "C" {

int tango_version(void) { return 100; }

const char *tango_status_string(int status)
{
    switch (status) {
        case TANGO_OK: return "ok";
        case TANGO_ERR_NULL: return "a required pointer is NULL";
        case TANGO_ERR_BAD_SHAPE: return "bad shape, size or alignment";
        case TANGO_ERR_BAD_ENUM: return "unknown enum value";
        case TANGO_ERR_UNSUPPORTED: return "unsupported configuration";
        case TANGO_ERR_WORKSPACE: return "workspace missing, misaligned or too small (or, for an entry point without one, the shape needs more scratch than the library holds)";
        case TANGO_ERR_LAUNCH: return "kernel launch refused by the HIP runtime";
        default: return "unknown status";
    }
}

int tango_absmax(const float *x, size_t n, float *absmax_out, void *stream)
{
    TANGO_REQUIRE(absmax_out != nullptr, TANGO_ERR_NULL);
    TANGO_REQUIRE(n == 0 || x != nullptr, TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(x, 4) && tango_aligned(absmax_out, 4), TANGO_ERR_BAD_SHAPE);
    hipStream_t st = tango_stream(stream);
    int rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(absmax_out), 0u, 1, st);
    if (rc != TANGO_OK) return rc;
    return tango_absmax_accumulate_async(x, n, absmax_out, st);
}

size_t tango_quantize_workspace_bytes(size_t) { return 256; }

int tango_quantize(const float *x, size_t n, int rounding, uint64_t seed, uint64_t stream_id,
                   const float *absmax_in, int8_t *q, float *scale_out, void *ws, size_t ws_bytes, void *stream)
{
    TANGO_REQUIRE(rounding == TANGO_RN || rounding == TANGO_SR, TANGO_ERR_BAD_ENUM);
    TANGO_REQUIRE(n == 0 || (x != nullptr && q != nullptr), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(x, 4), TANGO_ERR_BAD_SHAPE);
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
    return tango_quantize_with_absmax_async(x, n, rounding, seed, stream_id, am, q, scale_out, st);
}

int tango_quantize_relu_bwd(const float *x, const float *y, size_t n, int rounding, uint64_t seed, uint64_t stream_id,
                            int8_t *q, float *scale_out, void *ws, size_t ws_bytes, void *stream)
{
    TANGO_REQUIRE(rounding == TANGO_RN || rounding == TANGO_SR, TANGO_ERR_BAD_ENUM);
    TANGO_REQUIRE(n == 0 || (x != nullptr && y != nullptr && q != nullptr), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(x, 16) && tango_aligned(y, 16) && tango_aligned(q, 8), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(ws != nullptr && ws_bytes >= 256 && tango_aligned(ws, 256), TANGO_ERR_WORKSPACE);
    return tango_quantize_masked_async(x, y, n, rounding, seed, stream_id, q, scale_out, static_cast<float *>(ws),
                                       tango_stream(stream));
}

size_t tango_error_x_workspace_bytes(void) { return 512; }

int tango_error_x(const float *x, size_t n, const int *candidate_bits, int n_candidates, float threshold, int rounding,
                  uint64_t seed, uint64_t stream_id, const float *absmax_in, double *error_out, int *bits_out, void *ws,
                  size_t ws_bytes, void *stream)
{
    TANGO_REQUIRE(rounding == TANGO_RN || rounding == TANGO_SR, TANGO_ERR_BAD_ENUM);
    TANGO_REQUIRE(candidate_bits && error_out && (n == 0 || x), TANGO_ERR_NULL);
    TANGO_REQUIRE(n_candidates >= 1 && n_candidates <= MAX_CAND, TANGO_ERR_BAD_SHAPE);
    error_x_cands cands;
    cands.n = n_candidates;
    for (int c = 0; c < MAX_CAND; ++c) cands.bits[c] = 8;
    for (int c = 0; c < n_candidates; ++c) {
        TANGO_REQUIRE(candidate_bits[c] >= 2 && candidate_bits[c] <= 8, TANGO_ERR_BAD_SHAPE);
        cands.bits[c] = candidate_bits[c];
    }
    TANGO_REQUIRE(ws && tango_aligned(ws, 256) && ws_bytes >= tango_error_x_workspace_bytes(), TANGO_ERR_WORKSPACE);
    hipStream_t st = tango_stream(stream);
    double *sums = static_cast<double *>(ws);               // MAX_CAND doubles
    float *wam = reinterpret_cast<float *>(static_cast<char *>(ws) + 256);
    int rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(sums), 0u, 2 * MAX_CAND, st);
    if (rc != TANGO_OK) return rc;
    const float *am = absmax_in;
    if (!am) {
        if ((rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(wam), 0u, 1, st)) != TANGO_OK) return rc;
        if ((rc = tango_absmax_accumulate_async(x, n, wam, st)) != TANGO_OK) return rc;
        am = wam;
    }
    const tango_rng rng = tango_rng_make(seed, stream_id);
    if (n > 0) {
        const unsigned grid = tango_grid_for(n, 256 * 4);
        if (rounding == TANGO_RN)
            k_error_x<TANGO_RN><<<grid, 256, 0, st>>>(x, n, am, rng, cands, sums);
        else
            k_error_x<TANGO_SR><<<grid, 256, 0, st>>>(x, n, am, rng, cands, sums);
        TANGO_LAUNCH_CHECK();
    }
    k_error_x_finish<<<1, 64, 0, st>>>(cands, n, threshold, sums, error_out, bits_out);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_relu(const float *x, size_t n, float *y, float *absmax_y, void *stream)
{
    TANGO_REQUIRE(n == 0 || (x != nullptr && y != nullptr), TANGO_ERR_NULL);
    hipStream_t st = tango_stream(stream);
    if (absmax_y) {
        int rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(absmax_y), 0u, 1, st);
        if (rc != TANGO_OK) return rc;
    }
    if (n == 0) return TANGO_OK;
    k_relu<<<tango_grid_for(n, 256 * 4), 256, 0, st>>>(x, n, y, absmax_y);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_relu_bwd(const float *x, const float *dy, size_t n, float *dx, void *stream)
{
    TANGO_REQUIRE(n == 0 || (x != nullptr && dy != nullptr && dx != nullptr), TANGO_ERR_NULL);
    if (n == 0) return TANGO_OK;
    k_relu_bwd<<<tango_grid_for(n, 256 * 4), 256, 0, tango_stream(stream)>>>(x, dy, n, dx);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_dequantize(const int8_t *q, size_t n, const float *scale, float *x, void *stream)
{
    TANGO_REQUIRE(scale != nullptr, TANGO_ERR_NULL);
    TANGO_REQUIRE(n == 0 || (q != nullptr && x != nullptr), TANGO_ERR_NULL);
    if (n == 0) return TANGO_OK;
    k_dequantize<<<tango_grid_for(n, 256 * 8), 256, 0, tango_stream(stream)>>>(q, n, scale, x);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

}  // extern "C"
