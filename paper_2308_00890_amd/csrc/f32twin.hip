// Full-precision twins of the quantized SPMM and SDDMM-dot: the same work decomposition (edge-balanced chunks,
// block-wise index fetch, cross-lane distribution, shuffle reductions) on fp32 operands.  They exist so that the
// benefit of quantization (Sec. 3.3: random accesses hit a 4x smaller table) can be measured inside one library
// on the same graph; they are not part of the quantized path.
#include "internal.hip.h"

namespace {

constexpr int CHUNK_SHIFT = 10;
constexpr int WAVES_PER_BLOCK = 4;

__device__ inline int wave_find_row_f(const int32_t *__restrict__ ptr, int n, int e)
{
    const int lane = threadIdx.x % TANGO_WAVE;
    int lo = 0, hi = n;
    while (hi - lo > 1) {
        const int step = (hi - lo + 63) / 64;
        const int p = lo + (lane + 1) * step;
        const bool le = (p < hi) && (ptr[p] <= e);
        const int cnt = __popcll(__ballot(le));
        const int nlo = lo + cnt * step;
        const int nhi = min(hi, lo + (cnt + 1) * step);
        lo = nlo;
        hi = nhi;
    }
    return lo;
}

struct spmm_f32_args {
    int n;
    int64_t nnz;
    const int32_t *ptr, *idx, *eid;
    const float *w;   // nnz x heads
    const float *X;   // n x F
    float *out;       // n x F
    int heads, dim, F;
};

__device__ inline bool split_row(int b, int t) { return t > b && (b >> CHUNK_SHIFT) != ((t - 1) >> CHUNK_SHIFT); }

// rows cut by a chunk boundary (accumulated with float atomics) and empty rows start at zero
__global__ __launch_bounds__(256) void k_spmm_f32_prepare(spmm_f32_args a)
{
    const int lane = threadIdx.x % TANGO_WAVE;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) / TANGO_WAVE;
    const int nwaves = gridDim.x * blockDim.x / TANGO_WAVE;
    for (int64_t base = static_cast<int64_t>(wave) * 64; base < a.n; base += static_cast<int64_t>(nwaves) * 64) {
        const int r = static_cast<int>(base) + lane;
        bool flag = false;
        if (r < a.n) {
            const int b = a.ptr[r], t = a.ptr[r + 1];
            flag = (t == b) || split_row(b, t);
        }
        unsigned long long mask = __ballot(flag);
        while (mask) {
            const int k = __ffsll(static_cast<long long>(mask)) - 1;
            mask &= mask - 1;
            float *row = a.out + (base + k) * a.F;
            for (int c = lane; c < a.F; c += 64) row[c] = 0.0f;
        }
    }
}

// One wave per chunk of 1024 edges; a lane owns 4 consecutive columns of a 256-column tile.
template <bool HAS_EID>
__global__ __launch_bounds__(64 * WAVES_PER_BLOCK) void k_spmm_f32(spmm_f32_args a)
{
    const int lane = threadIdx.x % TANGO_WAVE;
    // readfirstlane: tells the compiler that the wave index, hence the chunk and the row walk, is wave-uniform
    const int64_t chunk = static_cast<int64_t>(blockIdx.x) * WAVES_PER_BLOCK + __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x / TANGO_WAVE));
    const int64_t c0 = chunk << CHUNK_SHIFT;
    if (c0 >= a.nnz) return;
    const int64_t c1 = min(c0 + (int64_t(1) << CHUNK_SHIFT), a.nnz);
    const int TF = min(a.F, 256);       // columns per tile
    const int LPR = TF / 4;             // lanes per (tile of a) row
    const int G = 64 / LPR;
    const int gi = lane / LPR, li = lane - gi * LPR;
    constexpr int U = 8;
    int r = wave_find_row_f(a.ptr, a.n, static_cast<int>(c0));
    for (; r < a.n; ++r) {
        const int rb = a.ptr[r], rt = a.ptr[r + 1];
        if (rb >= c1) break;
        const int sb = max(rb, static_cast<int>(c0)), se = min(rt, static_cast<int>(c1));
        if (sb >= se) continue;
        const bool whole = (rb >= c0) && (rt <= c1);
        for (int tile = 0; tile < a.F; tile += TF) {
            const int col = tile + li * 4;
            const int h = col / a.dim;
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int base = sb; base < se; base += 64) {
                const int cnt = min(64, se - base);
                int my_nb = 0, my_wp = 0;
                if (lane < cnt) {
                    my_nb = a.idx[base + lane];
                    my_wp = HAS_EID ? a.eid[base + lane] : base + lane;
                }
                const int steps = (cnt + G - 1) / G;
                for (int s0 = 0; s0 < steps; s0 += U) {
                    float wv[U];
                    float4 xv[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int k = (s0 + u) * G + gi;
                        const bool ok = k < cnt;
                        const int kk = ok ? k : 0;
                        const int nb = __shfl(my_nb, kk, 64);
                        const int wp = __shfl(my_wp, kk, 64);
                        wv[u] = ok ? a.w[static_cast<int64_t>(wp) * a.heads + h] : 0.0f;
                        xv[u] = *reinterpret_cast<const float4 *>(a.X + static_cast<int64_t>(nb) * a.F + col);
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        acc.x += wv[u] * xv[u].x;
                        acc.y += wv[u] * xv[u].y;
                        acc.z += wv[u] * xv[u].z;
                        acc.w += wv[u] * xv[u].w;
                    }
                }
            }
            for (int off = G / 2; off >= 1; off >>= 1) {
                acc.x += __shfl_down(acc.x, off * LPR, 64);
                acc.y += __shfl_down(acc.y, off * LPR, 64);
                acc.z += __shfl_down(acc.z, off * LPR, 64);
                acc.w += __shfl_down(acc.w, off * LPR, 64);
            }
            if (gi == 0) {
                float *o = a.out + static_cast<int64_t>(r) * a.F + col;
                if (whole) {
                    *reinterpret_cast<float4 *>(o) = acc;
                } else {
                    atomicAdd(o + 0, acc.x);
                    atomicAdd(o + 1, acc.y);
                    atomicAdd(o + 2, acc.z);
                    atomicAdd(o + 3, acc.w);
                }
            }
        }
    }
}

struct sddmm_f32_args {
    int n;
    int64_t nnz;
    const int32_t *ptr, *idx;
    const float *Xdst, *Xsrc;
    float *out;
    int heads, dim, F;
};

template <int DUMMY>
__global__ __launch_bounds__(64 * WAVES_PER_BLOCK) void k_sddmm_dot_f32(sddmm_f32_args a)
{
    const int lane = threadIdx.x % TANGO_WAVE;
    // readfirstlane: tells the compiler that the wave index, hence the chunk and the row walk, is wave-uniform
    const int64_t chunk = static_cast<int64_t>(blockIdx.x) * WAVES_PER_BLOCK + __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x / TANGO_WAVE));
    const int64_t c0 = chunk << CHUNK_SHIFT;
    if (c0 >= a.nnz) return;
    const int64_t c1 = min(c0 + (int64_t(1) << CHUNK_SHIFT), a.nnz);
    const int TF = min(a.F, 256);
    const int LPR = TF / 4;
    const int G = 64 / LPR;
    const int gi = lane / LPR, li = lane - gi * LPR;
    // lanes per head inside a tile (a head wider than a tile spans all of its lanes and several tiles)
    const int LPH = min(a.dim, TF) / 4;
    constexpr int U = 4;
    int r = wave_find_row_f(a.ptr, a.n, static_cast<int>(c0));
    for (; r < a.n; ++r) {
        const int rb = a.ptr[r], rt = a.ptr[r + 1];
        if (rb >= c1) break;
        const int sb = max(rb, static_cast<int>(c0)), se = min(rt, static_cast<int>(c1));
        if (sb >= se) continue;
        for (int base = sb; base < se; base += 64) {
            const int cnt = min(64, se - base);
            int my_nb = 0;
            if (lane < cnt) my_nb = a.idx[base + lane];
            const int steps = (cnt + G - 1) / G;
            for (int s0 = 0; s0 < steps; s0 += U) {
                float dot[U];
#pragma unroll
                for (int u = 0; u < U; ++u) dot[u] = 0.0f;
                for (int tile = 0; tile < a.F; tile += TF) {
                    const int col = tile + li * 4;
                    const float4 dv = *reinterpret_cast<const float4 *>(a.Xdst + static_cast<int64_t>(r) * a.F + col);
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int k = (s0 + u) * G + gi;
                        const int nb = __shfl(my_nb, k < cnt ? k : 0, 64);
                        const float4 xv = *reinterpret_cast<const float4 *>(a.Xsrc + static_cast<int64_t>(nb) * a.F + col);
                        dot[u] += dv.x * xv.x + dv.y * xv.y + dv.z * xv.z + dv.w * xv.w;
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    float d = dot[u];
                    for (int off = LPH / 2; off >= 1; off >>= 1) d += __shfl_xor(d, off, 64);
                    const int k = (s0 + u) * G + gi;
                    const int h = (li * 4) / min(a.dim, TF);  // head of my lanes inside the tile (dim <= 256), else 0
                    if (k < cnt && (li % LPH) == 0)
                        a.out[(static_cast<int64_t>(base) + k) * a.heads + (a.dim >= TF ? 0 : h)] = d;
                }
            }
        }
    }
}

bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

int check_shape(int heads, int dim)
{
    TANGO_REQUIRE(heads >= 1 && dim >= 4 && dim % 4 == 0, TANGO_ERR_BAD_SHAPE);
    const int64_t F = static_cast<int64_t>(heads) * dim;
    TANGO_REQUIRE(F <= 4096, TANGO_ERR_BAD_SHAPE);
    if (F <= 256) {
        TANGO_REQUIRE(pow2(static_cast<int>(F) / 4) && pow2(dim / 4), TANGO_ERR_UNSUPPORTED);
    } else {
        // wider rows are processed in 256-column tiles: one head only
        TANGO_REQUIRE(F % 256 == 0 && heads == 1, TANGO_ERR_UNSUPPORTED);
    }
    return TANGO_OK;
}

}  // namespace

extern "C" {

int tango_spmm_f32(const tango_graph *g, int direction, int heads, int dim, const float *w, const float *X, float *out,
                   void *stream)
{
    TANGO_REQUIRE(direction == TANGO_IN || direction == TANGO_OUT, TANGO_ERR_BAD_ENUM);
    TANGO_REQUIRE(g != nullptr, TANGO_ERR_NULL);
    TANGO_REQUIRE(g->n_nodes > 0 && g->n_edges >= 0 && g->n_edges < (int64_t(1) << 31), TANGO_ERR_BAD_SHAPE);
    if (direction == TANGO_IN)
        TANGO_REQUIRE(g->in_ptr && (g->n_edges == 0 || g->in_src), TANGO_ERR_NULL);
    else
        TANGO_REQUIRE(g->out_ptr && (g->n_edges == 0 || (g->out_dst && g->out_eid)), TANGO_ERR_NULL);
    int rc = check_shape(heads, dim);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(X && out && (g->n_edges == 0 || w), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(X, 16) && tango_aligned(out, 16), TANGO_ERR_BAD_SHAPE);
    hipStream_t st = tango_stream(stream);
    spmm_f32_args a;
    a.n = g->n_nodes; a.nnz = g->n_edges;
    a.ptr = direction == TANGO_IN ? g->in_ptr : g->out_ptr;
    a.idx = direction == TANGO_IN ? g->in_src : g->out_dst;
    a.eid = direction == TANGO_IN ? nullptr : g->out_eid;
    a.w = w; a.X = X; a.out = out; a.heads = heads; a.dim = dim; a.F = heads * dim;
    k_spmm_f32_prepare<<<tango_grid_for((static_cast<size_t>(a.n) + 63) / 64, 4, 256 * 8), 256, 0, st>>>(a);
    TANGO_LAUNCH_CHECK();
    if (a.nnz > 0) {
        const int64_t chunks = (a.nnz + (int64_t(1) << CHUNK_SHIFT) - 1) >> CHUNK_SHIFT;
        const unsigned blocks = static_cast<unsigned>((chunks + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
        if (a.eid)
            k_spmm_f32<true><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
        else
            k_spmm_f32<false><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
        TANGO_LAUNCH_CHECK();
    }
    return TANGO_OK;
}

int tango_sddmm_dot_f32(const tango_graph *g, int heads, int dim, const float *X_src, const float *X_dst, float *E,
                        void *stream)
{
    TANGO_REQUIRE(g != nullptr, TANGO_ERR_NULL);
    TANGO_REQUIRE(g->n_nodes > 0 && g->n_edges >= 0 && g->n_edges < (int64_t(1) << 31), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(g->in_ptr && (g->n_edges == 0 || g->in_src), TANGO_ERR_NULL);
    int rc = check_shape(heads, dim);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(X_src && X_dst && (g->n_edges == 0 || E), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(X_src, 16) && tango_aligned(X_dst, 16), TANGO_ERR_BAD_SHAPE);
    if (g->n_edges == 0) return TANGO_OK;
    sddmm_f32_args a;
    a.n = g->n_nodes; a.nnz = g->n_edges; a.ptr = g->in_ptr; a.idx = g->in_src;
    a.Xdst = X_dst; a.Xsrc = X_src; a.out = E; a.heads = heads; a.dim = dim; a.F = heads * dim;
    const int64_t chunks = (a.nnz + (int64_t(1) << CHUNK_SHIFT) - 1) >> CHUNK_SHIFT;
    const unsigned blocks = static_cast<unsigned>((chunks + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
    k_sddmm_dot_f32<0><<<blocks, 64 * WAVES_PER_BLOCK, 0, tango_stream(stream)>>>(a);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

}  // extern "C"
