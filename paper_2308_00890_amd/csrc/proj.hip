// Attention projections in fp32 (Sec. 2.1 step 2 and step 2').  Both kernels
// stream an n x F matrix once and are bound by HBM bandwidth:
//   forward : 4F bytes read per node, 8*heads written;
//   backward: (4F + F) read and 4F written per node.
#include "internal.hip.h"

namespace {

// S[p] = X[p, :] . a_src[h, :], D[p] likewise, p = v*heads + h; LPP lanes per (node, head) pair.
__global__ __launch_bounds__(256) void k_head_proj(int64_t npairs, int heads, int dim, int lpp,
                                                   const float *__restrict__ X, const float *__restrict__ a_src,
                                                   const float *__restrict__ a_dst, float *__restrict__ S,
                                                   float *__restrict__ D, float *absmax_S, float *absmax_D)
{
    const int lane = threadIdx.x % TANGO_WAVE;
    const int lg = lane % lpp;
    const int ppw = 64 / lpp;  // pairs per wave-iteration
    const int64_t wave = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) / TANGO_WAVE;
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * blockDim.x / TANGO_WAVE;
    const int q = dim / 4;  // float4 per pair
    float ms = 0.0f, md = 0.0f;
    // UNR groups of pairs per wave-iteration: their first loads are issued together (with one float4 per lane and
    // pair - dim <= 256 - the loop is otherwise one dependent load per iteration)
    constexpr int UNR = 4;
    const bool small = npairs < (int64_t(1) << 32);
    for (int64_t p0 = wave * ppw * UNR; p0 < npairs; p0 += nwaves * ppw * UNR) {
        int64_t p[UNR];
        float4 x0[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            p[u] = p0 + u * ppw + lane / lpp;
            x0[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (p[u] < npairs && lg < q) x0[u] = reinterpret_cast<const float4 *>(X + p[u] * dim)[lg];
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            double accs = 0.0, accd = 0.0;
            if (p[u] < npairs) {
                // (a 64-bit remainder costs more instructions than the dot product itself)
                const int h = small ? static_cast<int>(static_cast<uint32_t>(p[u]) % static_cast<uint32_t>(heads))
                                    : static_cast<int>(p[u] % heads);
                const float4 *x4 = reinterpret_cast<const float4 *>(X + p[u] * dim);
                const float4 *as4 = reinterpret_cast<const float4 *>(a_src + static_cast<int64_t>(h) * dim);
                const float4 *ad4 = reinterpret_cast<const float4 *>(a_dst + static_cast<int64_t>(h) * dim);
                for (int k = lg; k < q; k += lpp) {
                    const float4 x = (k == lg) ? x0[u] : x4[k], s = as4[k], d = ad4[k];
                    accs += static_cast<double>(x.x) * s.x + static_cast<double>(x.y) * s.y + static_cast<double>(x.z) * s.z +
                            static_cast<double>(x.w) * s.w;
                    accd += static_cast<double>(x.x) * d.x + static_cast<double>(x.y) * d.y + static_cast<double>(x.z) * d.z +
                            static_cast<double>(x.w) * d.w;
                }
            }
            for (int o = lpp / 2; o > 0; o >>= 1) {
                accs += __shfl_xor(accs, o, 64);
                accd += __shfl_xor(accd, o, 64);
            }
            if (p[u] < npairs && lg == 0) {
                const float fs = static_cast<float>(accs), fd = static_cast<float>(accd);
                S[p[u]] = fs;
                D[p[u]] = fd;
                ms = fmaxf(ms, fabsf(fs));
                md = fmaxf(md, fabsf(fd));
            }
        }
    }
    if (absmax_S) tango_block_max_update(ms, absmax_S);
    if (absmax_D) tango_block_max_update(md, absmax_D);
}

// The same for the usual widths (dim/4 a power of two <= 64, F <= 1024): a wave takes whole node rows, lane l the
// float4 number 64*j + l of the row in pass j, so the slices of a_src / a_dst a lane needs never change (loaded once)
// and no index arithmetic is left in the loop; the loads of several rows are issued before the first is used.  The
// sums are formed in the same order as in k_head_proj (a lane's four products, then the xor tree over the head's lanes).
template <int PASSES>
__global__ __launch_bounds__(256) void k_head_proj_rows(int64_t n, int heads, int dim, const float *__restrict__ X,
                                                        const float *__restrict__ a_src, const float *__restrict__ a_dst,
                                                        float *__restrict__ S, float *__restrict__ D, float *absmax_S,
                                                        float *absmax_D)
{
    constexpr int UNR = PASSES == 4 ? 2 : 4;  // rows whose loads are in flight together
    const int lane = threadIdx.x % TANGO_WAVE;
    const int64_t wave = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) / TANGO_WAVE;
    const int64_t nwaves = static_cast<int64_t>(gridDim.x) * blockDim.x / TANGO_WAVE;
    const int F = heads * dim, q = F / 4, lph = dim / 4;
    // narrow rows (q < 64, one pass): a wave takes 64 / q rows side by side
    const int rpw = (PASSES == 1 && q < 64) ? 64 / q : 1;
    const int lane_row = (PASSES == 1 && q < 64) ? lane / q : 0;
    const int lane_idx = lane - lane_row * q;
    double as[PASSES][4], ad[PASSES][4];  // my slices of a_src / a_dst, widened once
    int hd[PASSES];
    bool on[PASSES], first[PASSES];
#pragma unroll
    for (int j = 0; j < PASSES; ++j) {
        const int idx = 64 * j + lane_idx;
        on[j] = idx < q && lane_row < rpw;
        hd[j] = idx / lph;
        first[j] = on[j] && (idx % lph) == 0;
        const float4 s4 = on[j] ? reinterpret_cast<const float4 *>(a_src)[idx] : make_float4(0.f, 0.f, 0.f, 0.f);
        const float4 d4 = on[j] ? reinterpret_cast<const float4 *>(a_dst)[idx] : make_float4(0.f, 0.f, 0.f, 0.f);
        as[j][0] = s4.x; as[j][1] = s4.y; as[j][2] = s4.z; as[j][3] = s4.w;
        ad[j][0] = d4.x; ad[j][1] = d4.y; ad[j][2] = d4.z; ad[j][3] = d4.w;
    }
    float ms = 0.0f, md = 0.0f;
    for (int64_t v0 = wave * UNR * rpw; v0 < n; v0 += nwaves * UNR * rpw) {
        float4 x[UNR][PASSES];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t v = v0 + u * rpw + lane_row;
#pragma unroll
            for (int j = 0; j < PASSES; ++j) {
                x[u][j] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (v < n && on[j]) x[u][j] = reinterpret_cast<const float4 *>(X + v * F)[64 * j + lane_idx];
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t v = v0 + u * rpw + lane_row;
#pragma unroll
            for (int j = 0; j < PASSES; ++j) {
                const float4 xv = x[u][j];
                const double x0 = xv.x, x1 = xv.y, x2 = xv.z, x3 = xv.w;
                double accs = 0.0, accd = 0.0;
                accs += x0 * as[j][0] + x1 * as[j][1] + x2 * as[j][2] + x3 * as[j][3];
                accd += x0 * ad[j][0] + x1 * ad[j][1] + x2 * ad[j][2] + x3 * ad[j][3];
                accs = tango_group_sum_f64(accs, lph);
                accd = tango_group_sum_f64(accd, lph);
                if (v < n && first[j]) {
                    const float fs = static_cast<float>(accs), fd = static_cast<float>(accd);
                    S[v * heads + hd[j]] = fs;
                    D[v * heads + hd[j]] = fd;
                    ms = fmaxf(ms, fabsf(fs));
                    md = fmaxf(md, fabsf(fd));
                }
            }
        }
    }
    if (absmax_S) tango_block_max_update(ms, absmax_S);
    if (absmax_D) tango_block_max_update(md, absmax_D);
}

// Head projections and the quantization of X in one pass over X (Sec. 3.3: the tensor the sparse primitives gather
// from is quantized once, sequentially; its abs-max is already known from the GEMM that wrote it).  The tensor is taken
// as a flat run of groups of 8 elements - one block of random bits each, like the stand-alone quantizer - lane l of a
// wave taking group base + l: with dim/8 a power of two the dim/8 lanes of one (node, head) pair are adjacent and
// aligned, every lane is busy whatever the row width, and a_src / a_dst are read from LDS by column.
template <int ROUNDING>
__global__ __launch_bounds__(256) void k_head_proj_quant(int64_t n, int heads, int dim, const float *__restrict__ X,
                                                         const float *__restrict__ a_src, const float *__restrict__ a_dst,
                                                         float *__restrict__ S, float *__restrict__ D, float *absmax_S,
                                                         float *absmax_D, const float *__restrict__ absmax_X, tango_rng rng,
                                                         int8_t *__restrict__ Xq, float *scale_out)
{
    __shared__ __attribute__((aligned(16))) float a_s[2][1024];
    const int F = heads * dim;
    for (int i = threadIdx.x; i < F; i += blockDim.x) {
        a_s[0][i] = a_src[i];
        a_s[1][i] = a_dst[i];
    }
    __syncthreads();
    float s, inv;
    tango_scale_from_absmax(*absmax_X, s, inv);
    if (blockIdx.x == 0 && threadIdx.x == 0 && scale_out) *scale_out = s;
    const uint32_t g8 = static_cast<uint32_t>(F / 8);    // groups per row
    const int lph = dim / 8;                             // lanes per head (power of two)
    const int log2lph = __ffs(lph) - 1;
    const int64_t ngroups = n * g8;
    const int lane = threadIdx.x % TANGO_WAVE;
    const int64_t tid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t nthr = static_cast<int64_t>(gridDim.x) * blockDim.x;
    const float4 *x4 = reinterpret_cast<const float4 *>(X);
    uint2 *q8 = reinterpret_cast<uint2 *>(Xq);
    constexpr int UNR = 4;
    float ms = 0.0f, md = 0.0f;
    // the loop bound is the wave's: all 64 lanes take part in the lane sums
    for (int64_t w0 = tid - lane; w0 < ngroups; w0 += UNR * nthr) {
        float4 xa[UNR], xb[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t i = w0 + lane + u * nthr;
            xa[u] = xb[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i < ngroups) {
                xa[u] = x4[2 * i];
                xb[u] = x4[2 * i + 1];
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t i = w0 + lane + u * nthr;
            const int64_t row = (ngroups >> 32) == 0 ? static_cast<int64_t>(static_cast<uint32_t>(i) / g8) : i / g8;
            const int c8 = static_cast<int>(i - row * g8);
            const int head = c8 >> log2lph;
            const float x[8] = {xa[u].x, xa[u].y, xa[u].z, xa[u].w, xb[u].x, xb[u].y, xb[u].z, xb[u].w};
            float as[8], ad[8];
            *reinterpret_cast<float4 *>(as) = *reinterpret_cast<const float4 *>(&a_s[0][8 * c8]);
            *reinterpret_cast<float4 *>(as + 4) = *reinterpret_cast<const float4 *>(&a_s[0][8 * c8 + 4]);
            *reinterpret_cast<float4 *>(ad) = *reinterpret_cast<const float4 *>(&a_s[1][8 * c8]);
            *reinterpret_cast<float4 *>(ad + 4) = *reinterpret_cast<const float4 *>(&a_s[1][8 * c8 + 4]);
            double accs = 0.0, accd = 0.0;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const double xd = static_cast<double>(x[k]);
                accs += xd * static_cast<double>(as[k]);
                accd += xd * static_cast<double>(ad[k]);
            }
            accs = tango_group_sum_f64(accs, lph);
            accd = tango_group_sum_f64(accd, lph);
            if (i < ngroups) {
                if ((c8 & (lph - 1)) == 0) {
                    const float fs = static_cast<float>(accs), fd = static_cast<float>(accd);
                    S[row * heads + head] = fs;
                    D[row * heads + head] = fd;
                    ms = fmaxf(ms, fabsf(fs));
                    md = fmaxf(md, fabsf(fd));
                }
                const float y[8] = {x[0] * inv, x[1] * inv, x[2] * inv, x[3] * inv, x[4] * inv, x[5] * inv, x[6] * inv, x[7] * inv};
                q8[i] = tango_quantize8<ROUNDING>(y, rng, static_cast<uint64_t>(i));
            }
        }
    }
    // one update per workgroup, not per wave: the device-scope reads of the two scalars queue up at one L2 channel
    if (absmax_S) tango_block_max_update(ms, absmax_S);
    if (absmax_D) tango_block_max_update(md, absmax_D);
}

constexpr int ACC_COPIES = 16;  // copies of the column-sum accumulator of k_head_proj_bwd

// dX = dX_agg + (dS*a_src + dD*a_dst); column sums of dS*(sX*Xq), dD*(sX*Xq) into acc[2F] (double, atomics).
// Thread <-> one quad of columns; 256/TPR rows per block-iteration.
__global__ __launch_bounds__(256) void k_head_proj_bwd(int64_t n, int heads, int dim, const float *__restrict__ dS,
                                                       const float *__restrict__ dD, const float *__restrict__ a_src,
                                                       const float *__restrict__ a_dst, const int8_t *__restrict__ Xq,
                                                       const float *__restrict__ sX_p, const float *dX_agg, float *dX,
                                                       float *absmax_dX, double *acc)
{
    const int F = heads * dim;
    const int tpr = F / 4;            // threads per row
    const int rpb = 256 / tpr;        // rows per block-iteration
    const int ro = threadIdx.x / tpr;  // my row offset
    const int c = (threadIdx.x - ro * tpr) * 4;
    const bool active = ro < rpb;
    const float sX = *sX_p;
    double ss[4] = {0, 0, 0, 0}, sd[4] = {0, 0, 0, 0};
    float m = 0.0f;
    if (active) {
        const int h = c / dim;
        const float4 as = *reinterpret_cast<const float4 *>(a_src + c);
        const float4 ad = *reinterpret_cast<const float4 *>(a_dst + c);
        for (int64_t v = static_cast<int64_t>(blockIdx.x) * rpb + ro; v < n; v += static_cast<int64_t>(gridDim.x) * rpb) {
            const float gs = dS[v * heads + h], gd = dD[v * heads + h];
            const float4 ag = *reinterpret_cast<const float4 *>(dX_agg + v * F + c);
            const uint32_t xw = *reinterpret_cast<const uint32_t *>(Xq + v * F + c);
            float4 o;
            o.x = ag.x + (gs * as.x + gd * ad.x);
            o.y = ag.y + (gs * as.y + gd * ad.y);
            o.z = ag.z + (gs * as.z + gd * ad.z);
            o.w = ag.w + (gs * as.w + gd * ad.w);
            *reinterpret_cast<float4 *>(dX + v * F + c) = o;
            m = fmaxf(m, fmaxf(fmaxf(fabsf(o.x), fabsf(o.y)), fmaxf(fabsf(o.z), fabsf(o.w))));
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float x = sX * static_cast<float>(static_cast<int8_t>(xw >> (8 * j)));
                ss[j] += static_cast<double>(gs) * static_cast<double>(x);
                sd[j] += static_cast<double>(gd) * static_cast<double>(x);
            }
        }
    }
    // column sums: first across the rows of this block in LDS, then one atomic per column and block (per-thread
    // atomics onto 2F addresses serialise: they took longer than the streaming part)
    __shared__ double red[8][256];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        red[j][threadIdx.x] = active ? ss[j] : 0.0;
        red[4 + j][threadIdx.x] = active ? sd[j] : 0.0;
    }
    __syncthreads();
    if (static_cast<int>(threadIdx.x) < tpr) {  // row offset 0: my quad of columns, all row offsets
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            double ts = 0.0, td = 0.0;
            for (int r = 0; r < rpb; ++r) {
                ts += red[j][r * tpr + threadIdx.x];
                td += red[4 + j][r * tpr + threadIdx.x];
            }
            // (the accumulator exists ACC_COPIES times; workgroup b adds to copy b % ACC_COPIES: sixteen times fewer
            // atomics per address, and neighbouring workgroups do not queue on the same cache lines)
            double *mine = acc + static_cast<size_t>(blockIdx.x % ACC_COPIES) * 2 * F;
            if (ts != 0.0) atomicAdd(mine + c + j, ts);
            if (td != 0.0) atomicAdd(mine + F + c + j, td);
        }
    }
    if (absmax_dX) tango_block_max_update(m, absmax_dX);
}

__global__ void k_head_proj_bwd_finish(tango_colsum_job job) { tango_colsum_apply(job); }

}  // namespace

int tango_head_proj_async(int64_t n, int heads, int dim, const float *X, const float *a_src, const float *a_dst,
                          float *S, float *D, float *absmax_S, float *absmax_D, hipStream_t st)
{
    int rc;
    if ((rc = tango_zero2_u32_async(reinterpret_cast<uint32_t *>(absmax_S), 1, reinterpret_cast<uint32_t *>(absmax_D), 1, st)) != TANGO_OK)
        return rc;
    const int lph = dim / 4, q = heads * dim / 4;
    if (lph >= 1 && lph <= 64 && (lph & (lph - 1)) == 0 && q <= 256) {
        const int rpw = q < 64 ? 64 / q : 1;  // rows a wave takes side by side
        const unsigned grid = tango_grid_for(static_cast<size_t>((n + rpw - 1) / rpw), 16, 256 * 8);
        if (q <= 64) k_head_proj_rows<1><<<grid, 256, 0, st>>>(n, heads, dim, X, a_src, a_dst, S, D, absmax_S, absmax_D);
        else if (q <= 128) k_head_proj_rows<2><<<grid, 256, 0, st>>>(n, heads, dim, X, a_src, a_dst, S, D, absmax_S, absmax_D);
        else k_head_proj_rows<4><<<grid, 256, 0, st>>>(n, heads, dim, X, a_src, a_dst, S, D, absmax_S, absmax_D);
        TANGO_LAUNCH_CHECK();
        return TANGO_OK;
    }
    int lpp = 1;
    while (lpp * 2 <= 64 && lpp * 2 <= dim / 4) lpp *= 2;
    const int64_t npairs = n * heads;
    const size_t waves_needed = static_cast<size_t>((npairs + 4 * (64 / lpp) - 1) / (4 * (64 / lpp)));
    k_head_proj<<<tango_grid_for(waves_needed, 4, 256 * 8), 256, 0, st>>>(npairs, heads, dim, lpp, X, a_src, a_dst, S, D,
                                                                         absmax_S, absmax_D);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

bool tango_head_proj_quantize_supported(int heads, int dim)
{
    const int lph = dim / 8;
    return heads >= 1 && dim % 8 == 0 && lph <= 64 && (lph & (lph - 1)) == 0 && static_cast<int64_t>(heads) * dim <= 1024;
}

// tango_head_proj and the quantization of X (abs-max known: absmax_X, device) in one pass over X; X 16-byte and X_q
// 8-byte aligned; only where tango_head_proj_quantize_supported.  The results are those of the two separate calls.
int tango_head_proj_quantize_async(int64_t n, int heads, int dim, const float *X, const float *a_src, const float *a_dst,
                                   float *S, float *D, float *absmax_S, float *absmax_D, const float *absmax_X, int rounding,
                                   uint64_t seed, uint64_t stream_id, int8_t *X_q, float *s_X, hipStream_t st, bool absmax_zeroed)
{
    TANGO_REQUIRE(tango_head_proj_quantize_supported(heads, dim), TANGO_ERR_UNSUPPORTED);
    TANGO_REQUIRE(rounding == TANGO_RN || rounding == TANGO_SR, TANGO_ERR_BAD_ENUM);
    TANGO_REQUIRE(n > 0 && X && a_src && a_dst && S && D && absmax_X && X_q, TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(X, 16) && tango_aligned(X_q, 8), TANGO_ERR_BAD_SHAPE);
    int rc;
    if (!absmax_zeroed &&
        (rc = tango_zero2_u32_async(reinterpret_cast<uint32_t *>(absmax_S), 1, reinterpret_cast<uint32_t *>(absmax_D), 1, st)) != TANGO_OK)
        return rc;
    const tango_rng rng = tango_rng_make(seed, stream_id);
    const size_t ngroups = static_cast<size_t>(n) * (heads * dim / 8);
    const unsigned grid = tango_grid_for(ngroups / 4 + 1, 256, 256 * 8);
    if (rounding == TANGO_RN)
        k_head_proj_quant<TANGO_RN><<<grid, 256, 0, st>>>(n, heads, dim, X, a_src, a_dst, S, D, absmax_S, absmax_D, absmax_X,
                                                         rng, X_q, s_X);
    else
        k_head_proj_quant<TANGO_SR><<<grid, 256, 0, st>>>(n, heads, dim, X, a_src, a_dst, S, D, absmax_S, absmax_D, absmax_X,
                                                         rng, X_q, s_X);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_head_proj_bwd_async(int64_t n, int heads, int dim, const float *dS, const float *dD, const float *a_src,
                              const float *a_dst, const int8_t *X_q, const float *s_X, const float *dX_agg, float *dX,
                              float *absmax_dX, float *da_src, float *da_dst, void *ws, hipStream_t st, bool zeroed,
                              tango_colsum_job *deferred)
{
    const int F = heads * dim;
    double *acc = static_cast<double *>(ws);
    if (!zeroed) {
        int rc = tango_zero2_u32_async(reinterpret_cast<uint32_t *>(acc), 4 * F * ACC_COPIES, reinterpret_cast<uint32_t *>(absmax_dX), 1, st);
        if (rc != TANGO_OK) return rc;
    }
    const int rpb = 256 / (F / 4);
    k_head_proj_bwd<<<tango_grid_for(static_cast<size_t>((n + rpb - 1) / rpb), 8, 256 * 4), 256, 0, st>>>(
        n, heads, dim, dS, dD, a_src, a_dst, X_q, s_X, dX_agg, dX, absmax_dX, acc);
    TANGO_LAUNCH_CHECK();
    const tango_colsum_job job{acc, F, ACC_COPIES, da_src, da_dst};
    if (deferred) {  // the caller hands the column sums to the next launch of its chain
        *deferred = job;
        return TANGO_OK;
    }
    k_head_proj_bwd_finish<<<1, 256, 0, st>>>(job);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

void tango_head_proj_bwd_zero_regions(int heads, int dim, void *ws, float *absmax_dX, tango_zero_regions &z)
{
    tango_zero_regions_add(z, ws, static_cast<int64_t>(4) * heads * dim * ACC_COPIES);
    tango_zero_regions_add(z, absmax_dX, 1);
}

extern "C" {

int tango_head_proj(int64_t n, int heads, int dim, const float *X, const float *a_src, const float *a_dst, float *S,
                    float *D, float *absmax_S, float *absmax_D, void *stream)
{
    TANGO_REQUIRE(n >= 0 && heads >= 1 && dim >= 4 && dim % 4 == 0, TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(a_src && a_dst && (n == 0 || (X && S && D)), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(X, 16) && tango_aligned(a_src, 16) && tango_aligned(a_dst, 16), TANGO_ERR_BAD_SHAPE);
    return tango_head_proj_async(n, heads, dim, X, a_src, a_dst, S, D, absmax_S, absmax_D, tango_stream(stream));
}

size_t tango_head_proj_bwd_workspace_bytes(int64_t, int heads, int dim)
{
    return tango_round_up(static_cast<size_t>(2) * heads * dim * sizeof(double) * ACC_COPIES, 256);
}

int tango_head_proj_bwd(int64_t n, int heads, int dim, const float *dS, const float *dD, const float *a_src,
                        const float *a_dst, const int8_t *X_q, const float *s_X, const float *dX_agg, float *dX,
                        float *absmax_dX, float *da_src, float *da_dst, void *ws, size_t ws_bytes, void *stream)
{
    TANGO_REQUIRE(n >= 0 && heads >= 1 && dim >= 4 && dim % 4 == 0, TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(static_cast<int64_t>(heads) * dim <= 1024, TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(a_src && a_dst && s_X && da_src && da_dst && (n == 0 || (dS && dD && X_q && dX_agg && dX)),
                  TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(dX_agg, 16) && tango_aligned(dX, 16) && tango_aligned(X_q, 4) &&
                      tango_aligned(a_src, 16) && tango_aligned(a_dst, 16),
                  TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(ws && tango_aligned(ws, 256) && ws_bytes >= tango_head_proj_bwd_workspace_bytes(n, heads, dim),
                  TANGO_ERR_WORKSPACE);
    return tango_head_proj_bwd_async(n, heads, dim, dS, dD, a_src, a_dst, X_q, s_X, dX_agg, dX, absmax_dX, da_src, da_dst,
                                     ws, tango_stream(stream));
}

}  // extern "C"
