// Quantized SPMM (Sec. 2.1 steps 5, 5'; Sec. 3.3 "Incidence matrix-based
// adaptive SPMM") and quantized SDDMM-dot (Sec. 2.1 step 5''; Sec. 3.3 "SDDMM
// with on-the-fly dequantization", multiplication case).
//
// Work decomposition (both kernels): the edge array of the chosen direction is
// cut into chunks of CHUNK consecutive edges, one wavefront per chunk, so the
// load is balanced in edges whatever the degree distribution.  A wave finds
// the row that holds its first edge by a 64-ary search over the row pointer
// and then walks the row segments inside its chunk.  A row that lies entirely
// in one chunk is finished by that wave; a row cut by a chunk boundary is
// accumulated with int32 atomics (integer addition is associative, so the
// result does not depend on the order) and dequantized by a small second
// kernel.
//
// Inside a wave, a feature row of F int8 is covered by LPR = F/VEC lanes that
// load VEC bytes each, so one wave-wide load instruction gathers G = 64/LPR
// neighbour rows; the G partial sums are combined with cross-lane shuffles.
//
// Roofline: both kernels gather F bytes per edge from the int8 node table;
// HBM-bound when the table exceeds the on-chip caches, else bound by the
// cache/fabric gather rate.  Algorithmic bytes per edge: 4 (index) + heads
// (weight) + F (row); per node: 4 (pointer) + 4F (fp32 result).
#include "internal.hip.h"
#include "attn_math.hip.h"

#include <cstdlib>
#include <type_traits>

namespace {

constexpr int CHUNK_SHIFT_DEFAULT = 8;  // SDDMM-dot: 256 edges per wavefront
constexpr int WAVES_PER_BLOCK = 4;

// Largest r in [0, n) with ptr[r] <= e (ptr non-decreasing, ptr[0] = 0 <= e < ptr[n]).
// All 64 lanes cooperate: each step probes 64 positions and narrows the range 64-fold.
__device__ inline int wave_find_row(const int32_t *__restrict__ ptr, int n, int e)
{
    const int lane = threadIdx.x % TANGO_WAVE;
    int lo = 0, hi = n;  // ptr[lo] <= e; hi == n or ptr[hi] > e
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

template <int VEC>
struct vec_bytes;
template <>
struct vec_bytes<4> {
    using type = uint32_t;
};
template <>
struct vec_bytes<8> {
    using type = uint2;
};
template <>
struct vec_bytes<16> {
    using type = uint4;
};

template <int VEC>
__device__ inline void unpack_words(const typename vec_bytes<VEC>::type &v, uint32_t (&w)[VEC / 4]);
template <>
__device__ inline void unpack_words<4>(const uint32_t &v, uint32_t (&w)[1])
{
    w[0] = v;
}
template <>
__device__ inline void unpack_words<8>(const uint2 &v, uint32_t (&w)[2])
{
    w[0] = v.x;
    w[1] = v.y;
}
template <>
__device__ inline void unpack_words<16>(const uint4 &v, uint32_t (&w)[4])
{
    w[0] = v.x;
    w[1] = v.y;
    w[2] = v.z;
    w[3] = v.w;
}

// Edge weights computed on the fly (fused attention, Sec. 2.1 steps 3-5): alpha of edge (u -> v), head h is
// exp(lrelu(s_S*S_q[u][h] + s_D*D_q[v][h]) - row_lse[v][h]), quantized with the abs-max found by the statistics
// pass; the random bits of stochastic rounding belong to the edge's destination-major position, so the forward
// pass (walking in-edges) and the backward pass (walking out-edges) form identical int8 codes.
struct attn_params {
    const int8_t *Sq, *Dq;
    const float *sS, *sD;
    float slope;
    const float *row_lse;  // n x heads, of the destination
    const float *absmax_alpha;
    tango_rng rng;
    int rounding;
    int8_t *alpha_q;     // forward: out, nnz x heads (or NULL)
    float *s_alpha;      // forward: out
    float *alpha_dump;   // forward: out or NULL, the fp32 alpha that was quantized
    // reverse pass fused with step 3' (DS instantiations): the gathered rows also give dalpha of every out-edge
    const int8_t *Xrow;            // n x F: the table of the row side (H'_q of the source)
    const float *s_Xrow;
    const void *rec;     // per destination: row_lse and P of every head
    double *dS_acc;                // n x heads, zero-initialised
    int relu_out;                  // forward: out = max(0, aggregate) (ReLU between stacked layers), absmax of that
    uint16_t *relu_bits;           // forward, optional: one bit per output element, set where the output is positive
    const int8_t *src_codes;       // forward, optional: S_q[src(e)] per in-edge, in edge order (read instead of gathered)
};

enum { W_LOAD = 0, W_ATT_FWD = 1, W_ATT_REV = 2 };

struct spmm_args {
    int n;                 // rows
    int64_t nnz;           // edges
    const int32_t *ptr;    // n+1, row pointer of the chosen direction
    const int32_t *idx;    // nnz, neighbour of each edge in that direction
    const int32_t *eid;    // nnz or NULL: position of the edge weight (NULL = the edge's own position)
    const int8_t *w;       // nnz x heads
    const int8_t *X;       // n x F
    const float *s_w, *s_X;
    float *out;            // n x F (fp32; int32 partial sums while the kernels run)
    float *absmax;         // or NULL
    int heads, dim, F;
    int chunk_shift;       // log2 of the edges per wavefront
    int short_rows;        // k_spmm_short: rows a wave takes per pass
    int short_max;         // rows with at most this many edges are left to k_spmm_short (0: none)
    attn_params att;       // used by the ATT instantiations only
    int relu;              // out = max(0, .)
    uint16_t *relu_bits;   // with relu, optional: bit i = (out[i] > 0) over the flat n x F output (F % 64 == 0, 16 columns per lane)
    int w_words;           // the head codes of an edge can be read as 32-bit words (heads 4 or 8, w 4-byte aligned)
    const double *cvt_src; // k_spmm_finalize also writes cvt_dst[i] = float(cvt_src[i]), i < cvt_n (the fused dS sums,
    float *cvt_dst;        // complete once the main kernel has ended); NULL: nothing to convert
    int64_t cvt_n;
    int fin_rows;          // rows a wave of k_spmm_prepare / k_spmm_finalize looks at per pass (64, or 8 on small graphs)
};

// True when row [b, t) is cut by a chunk boundary (it then goes through the atomic path).
__device__ inline bool row_is_split(int b, int t, int shift, int short_max)
{
    return t > b && (t - b) > short_max && (b >> shift) != ((t - 1) >> shift);
}

// Zero the rows that the main kernel reaches through atomics (split rows) or never writes (empty rows).
__global__ __launch_bounds__(256) void k_spmm_prepare(spmm_args a)
{
    if (blockIdx.x == 0 && threadIdx.x == 0 && a.absmax) *a.absmax = 0.0f;
    const int lane = threadIdx.x % TANGO_WAVE;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) / TANGO_WAVE;
    const int nwaves = gridDim.x * blockDim.x / TANGO_WAVE;
    for (int64_t base = static_cast<int64_t>(wave) * a.fin_rows; base < a.n; base += static_cast<int64_t>(nwaves) * a.fin_rows) {
        const int r = static_cast<int>(base) + lane;
        bool flag = false;
        if (lane < a.fin_rows && r < a.n) {
            const int b = a.ptr[r], t = a.ptr[r + 1];
            flag = (t == b) || row_is_split(b, t, a.chunk_shift, a.short_max);
        }
        unsigned long long mask = __ballot(flag);
        while (mask) {
            const int k = __ffsll(static_cast<long long>(mask)) - 1;
            mask &= mask - 1;
            float *row = a.out + (base + k) * a.F;
            for (int c = lane; c < a.F; c += 64) row[c] = 0.0f;
            if (a.relu_bits) {
                uint16_t *bits = a.relu_bits + (base + k) * (a.F / 16);
                for (int c = lane; c < a.F / 16; c += 64) bits[c] = 0;
            }
        }
    }
}

// Dequantize the split rows in place (int32 -> fp32) and fold them into the abs-max.
__global__ __launch_bounds__(256) void k_spmm_finalize(spmm_args a)
{
    const float sc = (*a.s_w) * (*a.s_X);
    const int lane = threadIdx.x % TANGO_WAVE;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) / TANGO_WAVE;
    const int nwaves = gridDim.x * blockDim.x / TANGO_WAVE;
    float m = 0.0f;
    for (int64_t base = static_cast<int64_t>(wave) * a.fin_rows; base < a.n; base += static_cast<int64_t>(nwaves) * a.fin_rows) {
        const int r = static_cast<int>(base) + lane;
        bool flag = false;
        if (lane < a.fin_rows && r < a.n) flag = row_is_split(a.ptr[r], a.ptr[r + 1], a.chunk_shift, a.short_max);
        unsigned long long mask = __ballot(flag);
        if (!a.relu_bits) {
            // several flagged rows at a time: a row is covered by F/4 lanes with four columns each, 64 / (F/4) rows side by
            // side (one row after the other left most lanes idle on narrow rows, and each row is a dependent
            // load - store round trip)
            const int lpr = min(64, a.F / 4), G = 64 / lpr;
            const int gi = lane / lpr, li = lane - gi * lpr;
            while (mask) {
                int myk = -1;
                for (int g2 = 0; g2 < G && mask; ++g2) {
                    const int k = __ffsll(static_cast<long long>(mask)) - 1;
                    mask &= mask - 1;
                    if (gi == g2) myk = k;
                }
                if (myk >= 0) {
                    float4 *row4 = reinterpret_cast<float4 *>(a.out + (base + myk) * a.F);
                    for (int c4 = li; c4 < a.F / 4; c4 += lpr) {
                        const float4 v = row4[c4];
                        int a0 = __float_as_int(v.x), a1 = __float_as_int(v.y), a2 = __float_as_int(v.z), a3 = __float_as_int(v.w);
                        if (a.relu) {
                            a0 = max(a0, 0); a1 = max(a1, 0); a2 = max(a2, 0); a3 = max(a3, 0);
                        }
                        float4 o;
                        o.x = static_cast<float>(a0) * sc; o.y = static_cast<float>(a1) * sc;
                        o.z = static_cast<float>(a2) * sc; o.w = static_cast<float>(a3) * sc;
                        row4[c4] = o;
                        m = fmaxf(m, fmaxf(fmaxf(fabsf(o.x), fabsf(o.y)), fmaxf(fabsf(o.z), fabsf(o.w))));
                    }
                }
            }
            continue;
        }
        while (mask) {
            const int k = __ffsll(static_cast<long long>(mask)) - 1;
            mask &= mask - 1;
            float *row = a.out + (base + k) * a.F;
            for (int c = lane; c < a.F; c += 64) {
                int acc = __float_as_int(row[c]);
                if (a.relu) acc = max(acc, 0);
                const float o = static_cast<float>(acc) * sc;
                row[c] = o;
                m = fmaxf(m, fabsf(o));
                if (a.relu_bits) {  // F is a multiple of 64 here: the 64 lanes' signs are one aligned 64-bit word
                    const unsigned long long w = __ballot(acc > 0);
                    if (lane == 0)
                        *reinterpret_cast<unsigned long long *>(a.relu_bits + ((base + k) * a.F + (c - lane)) / 16) = w;
                }
            }
        }
    }
    if (a.absmax) tango_block_max_update(m, a.absmax);
    if (a.cvt_src) {
        for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < a.cvt_n;
             i += static_cast<int64_t>(gridDim.x) * blockDim.x)
            a.cvt_dst[i] = static_cast<float>(a.cvt_src[i]);
    }
}

// t[c] = (r0.byte c, r1.byte c, r2.byte c, r3.byte c): 4x4 byte transpose with v_perm_b32.
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

// One wave per chunk of edges.  VEC = bytes of the feature row per lane; HAS_EID: the weight of edge j of
// this direction sits at position eid[j] (reversed graph) instead of j.
// X4: the feature table holds packed 4-bit codes (two columns per byte, even column in the low nibble); a.F and
// a.dim still count columns.  The nibbles are used in place as (code * 16) in an int8, so the int32 sums carry a
// factor 16 that is shifted out (exactly) when a row is finished: exact while |sum| < 2^27.
// DS (reverse attention mode only; Sec. 2.1 steps 5', 5'', 4', 3' in one walk over the out-edges of each source u):
// the row of dOut_q[v] gathered for 5' is also multiplied with the resident row X_q[u], which is dalpha of edge
// (u -> v); with alpha (already recomputed for the edge weight), P[v] and the sign of the pre-activation this gives
// dE, summed into dS_acc[u][h] - the second gather pass over the same rows that a separate SDDMM would need is gone.
// LPHC (DS only): lanes per head when known at compile time (0: computed from the arguments), so that the lane-group
// sums in the gather loop carry no branches.
template <int VEC, bool HAS_EID, int WMODE, bool X4 = false, bool DS = false, int LPHC = 0>
__global__ __launch_bounds__(64 * WAVES_PER_BLOCK) __attribute__((amdgpu_waves_per_eu(WMODE == 2 ? 4 : 5))) void k_spmm(spmm_args a)
{
    constexpr int CPL = X4 ? 2 * VEC : VEC;  // columns per lane
    static_assert(!DS || (WMODE == W_ATT_REV && !X4), "the fused dS path belongs to the reverse attention mode");
    // DS: per wave, the dot products and the fp32 alpha of the current block of 64 edges, [edge][head], heads <= 8
    __shared__ int dots_s[DS ? WAVES_PER_BLOCK : 1][DS ? 64 * 8 : 1];
    __shared__ float alf_s[DS ? WAVES_PER_BLOCK : 1][DS ? 64 * 8 : 1];
    // per wave, for the 64 edges of the current block: byte offset of the neighbour's row in the table (64 bit) and
    // the packed weight codes of heads 0-3 and 4-7
    __shared__ __align__(16) uint4 nbw_s[WAVES_PER_BLOCK][64];
    using V = typename vec_bytes<VEC>::type;
    __shared__ __align__(16) int stage[WAVES_PER_BLOCK][1024];  // one strip of F <= 1024 sums per wave
    const int lane = threadIdx.x % TANGO_WAVE;
    // the wave index goes through readfirstlane so that the compiler knows it (and everything derived from it: the
    // chunk, the row walk, the loop bounds) is wave-uniform and keeps it in scalar registers
    const int wv = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x / TANGO_WAVE));
    const int64_t chunk = static_cast<int64_t>(blockIdx.x) * WAVES_PER_BLOCK + wv;
    const int64_t c0 = chunk << a.chunk_shift;
    if (c0 >= a.nnz) return;
    const int64_t c1 = min(c0 + (int64_t(1) << a.chunk_shift), a.nnz);

    const int LPR = a.F / CPL;          // lanes per feature row
    const int G = 64 / LPR;             // neighbour rows gathered per wave-wide load (power of two)
    const int gi = lane / LPR;          // my group (>= G: idle lane)
    const int li = lane - gi * LPR;     // my position in the row
    const bool active = gi < G;
    const int col = li * CPL;           // first of my CPL columns
    const int h = col / a.dim;          // their head
    const int row_bytes = X4 ? a.F / 2 : a.F;
    constexpr bool ATT = WMODE != W_LOAD;
    float s_w, inv_w = 0.0f, att_sS = 0.0f, att_sD = 0.0f;
    if (ATT) {
        tango_scale_from_absmax(*a.att.absmax_alpha, s_w, inv_w);
        if (WMODE == W_ATT_FWD && blockIdx.x == 0 && threadIdx.x == 0) *a.att.s_alpha = s_w;
        att_sS = *a.att.sS;
        att_sD = *a.att.sD;
    } else {
        s_w = *a.s_w;
    }
    const float sc = s_w * (*a.s_X);
    const int8_t *Xcol = a.X + li * VEC;
    const int LPH = LPHC ? LPHC : a.dim / VEC;  // DS: lanes per head (a power of two)
    const int log2G = 31 - __clz(G);
    const int HP = DS ? tango_rec_heads(a.heads) : 1;  // DS: records per node in the table (heads rounded up to a power of two)
    const int log2HP = 31 - __clz(HP);
    // which weight word of an entry of nbw_s holds my head, and the v_perm selectors that put byte (h & 3) of two
    // weight words side by side (0x0c selects a zero byte)
    const bool upper_heads = h >= 4;
    const uint32_t hb = static_cast<uint32_t>(h & 3);
    const uint32_t sel01 = hb | ((4u + hb) << 8) | 0x0c0c0000u;
    const uint32_t sel23 = 0x00000c0cu | (hb << 16) | ((4u + hb) << 24);
    const bool leader = DS && (li % LPH) == 0;
    float sc_dot = 0.0f;
    if (DS) sc_dot = (*a.s_X) * (*a.att.s_Xrow);

    // The chunk is walked in blocks of 64 consecutive edges, whatever rows they belong to: lane l of a block first
    // fetches the neighbour index and the packed head weights of edge base+l (coalesced; in the attention modes it
    // computes them), so that these loads and the attention arithmetic are paid once per 64 edges even when rows
    // are short.  Then the row segments inside the block are processed one after the other: the groups pull
    // (index, weight) pairs out of those registers with cross-lane reads and issue the row gathers back to back.
    const int c0i = static_cast<int>(c0), c1i = static_cast<int>(c1);
    int maxabs = 0;
    constexpr int U = 8;  // independent row gathers in flight per lane
    constexpr int NO_END = 0x7fffffff;

    // rows: cur_r = the non-empty row that holds edge `pos`; cur_rt = its end; row ends of rows win_r0 .. win_r0+63
    // sit in the lanes of win_end
    int cur_r = wave_find_row(a.ptr, a.n, c0i);
    int open_rb = a.ptr[cur_r];  // start of the row being accumulated
    int win_r0 = cur_r;
    int win_end = (win_r0 + lane < a.n) ? a.ptr[win_r0 + lane + 1] : NO_END;
    int cur_rt = __builtin_amdgcn_readlane(win_end, 0);  // readlane: the result is wave-uniform (scalar registers)
    auto next_row = [&]() {  // advance cur_r to the next non-empty row (or to n)
        const int was = cur_rt;
        do {
            ++cur_r;
            if (cur_r - win_r0 >= 64) {
                win_r0 = cur_r;
                win_end = (win_r0 + lane < a.n) ? a.ptr[win_r0 + lane + 1] : NO_END;
            }
            cur_rt = __builtin_amdgcn_readlane(win_end, cur_r - win_r0);
        } while (cur_rt == was);
    };

    int acc[CPL];
#pragma unroll
    for (int j = 0; j < CPL; ++j) acc[j] = 0;
    bool pending = false;  // acc holds sums of the open row

    auto finish_row = [&](int r, bool whole) {
        // combine the G groups: afterwards group 0 holds the sums of this row segment
        for (int off = G / 2; off >= 1; off >>= 1) {
#pragma unroll
            for (int j = 0; j < CPL; ++j) acc[j] += __shfl_down(acc[j], off * LPR, 64);
        }
        if (X4) {
#pragma unroll
            for (int j = 0; j < CPL; ++j) acc[j] >>= 4;  // exact: every term is a multiple of 16
        }
        if (whole) {
            if (gi == 0) {
                float *orow = a.out + static_cast<int64_t>(r) * a.F + col;
                uint32_t bits = 0;
#pragma unroll
                for (int j = 0; j < CPL; j += 4) {
                    float4 o;
                    if (WMODE == W_ATT_FWD && a.relu) {  // sc > 0: the sign of the sum is the sign of the output
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) {
                            acc[j + jj] = max(acc[j + jj], 0);
                            if (CPL == 16) bits |= static_cast<uint32_t>(min(acc[j + jj], 1)) << (j + jj);
                        }
                    }
                    o.x = static_cast<float>(acc[j + 0]) * sc;
                    o.y = static_cast<float>(acc[j + 1]) * sc;
                    o.z = static_cast<float>(acc[j + 2]) * sc;
                    o.w = static_cast<float>(acc[j + 3]) * sc;
                    *reinterpret_cast<float4 *>(orow + j) = o;
                    maxabs = max(maxabs, max(max(abs(acc[j]), abs(acc[j + 1])), max(abs(acc[j + 2]), abs(acc[j + 3]))));
                }
                if (WMODE == W_ATT_FWD && CPL == 16 && a.relu_bits)  // 16 columns per lane: one halfword of sign bits
                    a.relu_bits[(static_cast<uint32_t>(r) * static_cast<uint32_t>(a.F / 16)) + (col >> 4)] = static_cast<uint16_t>(bits);
            }
        } else {
            // Row cut by a chunk boundary: int32 atomics.  The sums are first laid out by column in this
            // wave's LDS strip so that consecutive lanes add to consecutive words (coalesced atomics).
            int *strip = stage[wv];
            if (gi == 0) {
#pragma unroll
                for (int j = 0; j < CPL; j += 4)
                    *reinterpret_cast<int4 *>(strip + col + j) = make_int4(acc[j], acc[j + 1], acc[j + 2], acc[j + 3]);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            int *orow = reinterpret_cast<int *>(a.out + static_cast<int64_t>(r) * a.F);
            for (int c = lane; c < a.F; c += 64) {
                const int v = strip[c];
                if (v != 0) atomicAdd(orow + c, v);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
#pragma unroll
        for (int j = 0; j < CPL; ++j) acc[j] = 0;
        pending = false;
    };

    // neighbour index (and edge id) of my edge of the next block, fetched one block ahead: a block then starts with its
    // dependent loads instead of waiting for the index first
    constexpr bool USE_EID = HAS_EID && WMODE != W_ATT_FWD;
    int nb_ahead = 0, eid_ahead = 0;
    if (c0i + lane < c1i) {
        nb_ahead = a.idx[c0i + lane];
        if (USE_EID) eid_ahead = a.eid[c0i + lane];
    }
    // DS: dS of the row being walked, per lane (lanes of equal lane % HP hold parts of one head's sum); reduced over the
    // lanes and added to dS_acc when the row changes or the chunk ends
    double ds_run = 0.0;
    int ds_row = -1;
    auto flush_dS = [&]() {
        if (DS && ds_row >= 0) {
            double v = ds_run;
            for (int o = 32; o >= HP; o >>= 1) v += __shfl_xor(v, o, 64);
            if (lane < a.heads && v != 0.0) atomicAdd(a.att.dS_acc + static_cast<int64_t>(ds_row) * a.heads + lane, v);
        }
        ds_run = 0.0;
    };
    for (int base = c0i; base < c1i; base += 64) {
        const int cnt = min(64, c1i - base);
        const int nb_now = nb_ahead, eid_now = eid_ahead;
        if (base + 64 + lane < c1i) {
            nb_ahead = a.idx[base + 64 + lane];
            if (USE_EID) eid_ahead = a.eid[base + 64 + lane];
        }
        // pass 1 over the rows of this block: every lane learns the row of its edge and where that row ends
        // (seg_r, seg_rt: the walker's state at the start of the block, replayed by pass 2)
        const int seg_r = cur_r, seg_rt = cur_rt;
        int my_row = cur_r, my_rt = cur_rt;
        for (int k = 0; k < cnt;) {
            const int k1 = min(cur_rt - base, cnt);
            if (lane >= k && lane < k1) {
                my_row = cur_r;
                my_rt = cur_rt;
            }
            k = k1;
            if (cur_rt <= base + cnt) next_row();
        }
        int my_nb = 0;
        uint32_t my_w0 = 0, my_w1 = 0;
        double P_r[4] = {0.0, 0.0, 0.0, 0.0};  // DS: P of my (edge, head) pairs of rounds 0-3, kept for the block's epilogue
        if (DS) {
            // The records (P, row_lse, D_q) of the destinations of the block's edges, one 16-byte load per (edge, head)
            // pair with the heads of an edge in adjacent lanes: pair p = lane + 64*round, edge = p / HP, head = p % HP.
            // A lane keeps P for the epilogue (which works on the same pairs) and passes row_lse and D_q through LDS to
            // the lane that owns the edge in the alpha phase below (dots_s and nbw_s are free until then).
            const tango_attn_rec *recs = static_cast<const tango_attn_rec *>(a.att.rec);
            // (the pair indices are a few shifts from the lane number: recomputed per block through an opaque copy of it,
            // because as loop invariants they would each occupy a register for the whole kernel)
            int lane_o = lane;
            asm volatile("" : "+v"(lane_o));
            for (int g0 = 0; g0 < HP; g0 += 4) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (g0 + j >= HP) break;
                    const int pr = lane_o + 64 * (g0 + j);
                    const int edge = pr >> log2HP, head = pr & (HP - 1);
                    const int nbe = __shfl(nb_now, edge, 64);
                    if (edge < cnt && head < a.heads) {
                        const tango_attn_rec rc = recs[static_cast<int64_t>(nbe) * HP + head];
                        if (g0 == 0) P_r[j] = rc.P;
                        dots_s[wv][edge * a.heads + head] = __float_as_int(rc.row_lse);
                        reinterpret_cast<int8_t *>(&nbw_s[wv][0])[edge * a.heads + head] = static_cast<int8_t>(rc.dq);
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        if (lane < cnt) {
            const int e = base + lane;
            my_nb = nb_now;
            if (ATT) {
                // steps 3-4 and the quantization of alpha for this edge, all heads.  Forward: the row is the
                // destination, the neighbour the source; reverse: the other way round, and the edge's
                // destination-major position (for the random bits) comes from eid.
                const int H = a.heads;
                const int64_t src_node = (WMODE == W_ATT_FWD) ? my_nb : my_row;
                const int64_t dst_node = (WMODE == W_ATT_FWD) ? my_row : my_nb;
                const int64_t i0 = (WMODE == W_ATT_FWD ? static_cast<int64_t>(e) : static_cast<int64_t>(eid_now)) * H;
                uint4 blk = make_uint4(0, 0, 0, 0);
                uint64_t have = ~uint64_t(0);
                // four heads at a time (one pass up to 4 heads, two up to 8)
                for (int h0 = 0; h0 < H; h0 += 4) {
                    int sq[4], dq[4];
                    float lse4[4] = {0.f, 0.f, 0.f, 0.f};
                    if (WMODE == W_ATT_FWD && a.att.src_codes)
                        tango_load_heads4(a.att.src_codes, e, H, h0, sq);
                    else
                        tango_load_heads4(a.att.Sq, src_node, H, h0, sq);
                    if (DS) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if (h0 + j >= H) break;
                            lse4[j] = __int_as_float(dots_s[wv][lane * H + h0 + j]);
                            dq[j] = static_cast<int>(reinterpret_cast<const int8_t *>(&nbw_s[wv][0])[lane * H + h0 + j]);
                        }
                    } else {
                        tango_load_heads4(a.att.Dq, dst_node, H, h0, dq);
                    }
                    uint32_t wpk = 0;
                    // head counts that are multiples of four: the group's four random fields are one 64-bit half of one
                    // Philox block (i0 and h0 are multiples of four), fetched once for the group
                    const bool one_block = (H & 3) == 0 && a.att.rounding == TANGO_SR;
                    uint64_t half = 0;
                    if (one_block) {
                        const uint4 b4 = tango_philox_block(a.att.rng, static_cast<uint64_t>(i0 + h0) >> 3);
                        half = ((i0 + h0) & 4) ? ((static_cast<uint64_t>(b4.w) << 32) | b4.z) : ((static_cast<uint64_t>(b4.y) << 32) | b4.x);
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int hh = h0 + j;
                        if (hh >= H) break;
                        bool pos;
                        const float ev = tango_attn_score(att_sS * static_cast<float>(sq[j]), att_sD * static_cast<float>(dq[j]),
                                                          a.att.slope, pos);
                        const float lse = DS ? lse4[j] : a.att.row_lse[dst_node * H + hh];
                        const float al = tango_attn_alpha(ev, lse);
                        if (DS) alf_s[wv][lane * H + hh] = pos ? al : -al;  // the sign bit says "pre-activation not positive"
                        if (WMODE == W_ATT_FWD && a.att.alpha_dump) a.att.alpha_dump[i0 + hh] = al;
                        int q;
                        if (one_block) {
                            q = tango_round_clamp<TANGO_SR>(al * inv_w, static_cast<uint32_t>(half >> (16 * j)) & 0xffffu);
                        } else if (a.att.rounding == TANGO_SR) {
                            const uint64_t bi = static_cast<uint64_t>(i0 + hh) >> 3;
                            if (bi != have) {
                                blk = tango_philox_block(a.att.rng, bi);
                                have = bi;
                            }
                            q = tango_round_clamp<TANGO_SR>(al * inv_w, tango_bits16(blk, static_cast<int>((i0 + hh) & 7)));
                        } else {
                            q = tango_round_clamp<TANGO_RN>(al * inv_w, 0u);
                        }
                        if (WMODE == W_ATT_FWD && a.att.alpha_q) a.att.alpha_q[i0 + hh] = static_cast<int8_t>(q);
                        wpk |= (static_cast<uint32_t>(q) & 0xffu) << (8 * j);
                    }
                    if (h0 == 0)
                        my_w0 = wpk;
                    else
                        my_w1 = wpk;
                }
            } else {
                const int64_t wp = (HAS_EID ? static_cast<int64_t>(eid_now) : static_cast<int64_t>(e)) * a.heads;
                if (a.w_words) {  // 4 or 8 heads, 4-byte aligned table: the edge's codes in one or two word loads
                    my_w0 = *reinterpret_cast<const uint32_t *>(a.w + wp);
                    if (a.heads == 8) my_w1 = *reinterpret_cast<const uint32_t *>(a.w + wp + 4);
                } else {
                    for (int hh = 0; hh < a.heads; ++hh) {
                        const uint32_t b = static_cast<uint8_t>(a.w[wp + hh]);
                        if (hh < 4)
                            my_w0 |= b << (8 * hh);
                        else
                            my_w1 |= b << (8 * (hh - 4));
                    }
                }
            }
        }
        {
            const uint64_t off = static_cast<uint64_t>(static_cast<uint32_t>(my_nb)) * static_cast<uint32_t>(row_bytes);
            nbw_s[wv][lane] = make_uint4(static_cast<uint32_t>(off), static_cast<uint32_t>(off >> 32), my_w0, my_w1);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        // pass 2: the row segments [k0, k1) of the block
        for (int k0 = 0; k0 < cnt;) {
            const int r = (k0 == 0) ? seg_r : __builtin_amdgcn_readlane(my_row, k0);
            const int rt = (k0 == 0) ? seg_rt : __builtin_amdgcn_readlane(my_rt, k0);
            const int k1 = min(rt - base, cnt);
            const int len = k1 - k0;
            uint32_t dw[VEC / 4];  // DS: my columns of the resident row X_q[r]
            if (DS) {
                const V dv = *reinterpret_cast<const V *>(a.att.Xrow + static_cast<int64_t>(r) * a.F + (active ? col : 0));
                unpack_words<VEC>(dv, dw);
            }
            if (rt - open_rb > a.short_max) {
                const int steps = (len + G - 1) / G;
                const int full = len >> log2G;  // steps in which every group has an edge
                // MASKED = false: every group's edge exists, so nothing in the batch depends on the edge count (no
                // selects, no branches: the eight gathers, dot products and lane sums interleave freely).
                auto batch = [&](int s0, auto uu, auto masked) {
                    constexpr int UU = decltype(uu)::value;
                    constexpr bool MASKED = decltype(masked)::value;
                    uint32_t ww[UU];
                    V xv[UU];
                    bool ok[UU];
#pragma unroll
                    for (int u = 0; u < UU; ++u) {
                        const int k = (s0 + u) * G + gi;
                        ok[u] = !MASKED || k < len;
                        const int kk = ok[u] ? k0 + k : 0;
                        const uint4 ent = nbw_s[wv][kk];
                        ww[u] = upper_heads ? ent.w : ent.z;
                        if (MASKED && !ok[u]) ww[u] = 0u;
                        xv[u] = *reinterpret_cast<const V *>(Xcol + ((static_cast<uint64_t>(ent.y) << 32) | ent.x));
                    }
                    // 4 edges at a time: transpose each 4x4 byte block so that one dot4 multiplies one column of
                    // four neighbour rows by the four edge weights
#pragma unroll
                    for (int u = 0; u < UU; u += 4) {
                        // byte (h & 3) of the four weight words, side by side
                        const uint32_t wpack = __builtin_amdgcn_perm(ww[u + 1], ww[u], sel01) | __builtin_amdgcn_perm(ww[u + 3], ww[u + 2], sel23);
                        uint32_t w0[VEC / 4], w1[VEC / 4], w2[VEC / 4], w3[VEC / 4];
                        unpack_words<VEC>(xv[u], w0);
                        unpack_words<VEC>(xv[u + 1], w1);
                        unpack_words<VEC>(xv[u + 2], w2);
                        unpack_words<VEC>(xv[u + 3], w3);
                        if (DS) {
                            // dalpha of the four edges: my columns' share of the dot product with the resident row,
                            // summed over the lanes of my head, left in LDS as [edge of the block][head]
                            int d4[4] = {0, 0, 0, 0};
#pragma unroll
                            for (int q = 0; q < VEC / 4; ++q) {
                                d4[0] = __builtin_amdgcn_sdot4(static_cast<int>(dw[q]), static_cast<int>(w0[q]), d4[0], false);
                                d4[1] = __builtin_amdgcn_sdot4(static_cast<int>(dw[q]), static_cast<int>(w1[q]), d4[1], false);
                                d4[2] = __builtin_amdgcn_sdot4(static_cast<int>(dw[q]), static_cast<int>(w2[q]), d4[2], false);
                                d4[3] = __builtin_amdgcn_sdot4(static_cast<int>(dw[q]), static_cast<int>(w3[q]), d4[3], false);
                            }
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                const int d = tango_group_sum_c<LPHC>(d4[v], LPH);
                                const int k = (s0 + u + v) * G + gi;
                                if (MASKED) {
                                    if (ok[u + v] && leader) dots_s[wv][(k0 + k) * a.heads + h] = d;
                                } else {
                                    // every lane of the head holds the sum and stores it (same value, same word)
                                    dots_s[wv][(k0 + k) * a.heads + h] = d;
                                }
                            }
                        }
#pragma unroll
                        for (int q = 0; q < VEC / 4; ++q) {
                            uint32_t t[4];
                            if (X4) {
                                // byte c of a word = columns 2c (low nibble) and 2c+1 (high nibble): split into two words
                                // of (code * 16) bytes and treat each like an int8 word
                                constexpr uint32_t HI = 0xf0f0f0f0u;
                                transpose4x4((w0[q] << 4) & HI, (w1[q] << 4) & HI, (w2[q] << 4) & HI, (w3[q] << 4) & HI, t);
#pragma unroll
                                for (int c = 0; c < 4; ++c)
                                    acc[8 * q + 2 * c] = __builtin_amdgcn_sdot4(static_cast<int>(t[c]), static_cast<int>(wpack),
                                                                                acc[8 * q + 2 * c], false);
                                transpose4x4(w0[q] & HI, w1[q] & HI, w2[q] & HI, w3[q] & HI, t);
#pragma unroll
                                for (int c = 0; c < 4; ++c)
                                    acc[8 * q + 2 * c + 1] = __builtin_amdgcn_sdot4(static_cast<int>(t[c]), static_cast<int>(wpack),
                                                                                    acc[8 * q + 2 * c + 1], false);
                            } else {
                                transpose4x4(w0[q], w1[q], w2[q], w3[q], t);
#pragma unroll
                                for (int c = 0; c < 4; ++c)
                                    acc[4 * q + c] = __builtin_amdgcn_sdot4(static_cast<int>(t[c]), static_cast<int>(wpack), acc[4 * q + c], false);
                            }
                        }
                    }
                };
                if (active) {  // lanes beyond the last whole group sit the gathers out
                    constexpr std::false_type all_there{};
                    constexpr std::true_type masked{};
                    int s0 = 0;
                    for (; s0 + U <= full; s0 += U) batch(s0, std::integral_constant<int, U>{}, all_there);
                    for (; s0 + 4 <= full; s0 += 4) batch(s0, std::integral_constant<int, 4>{}, all_there);
                    for (; s0 < steps; s0 += 4) batch(s0, std::integral_constant<int, 4>{}, masked);
                }
                pending = true;
            }
            if (base + k1 == rt) {  // the row ends here
                if (pending) finish_row(r, open_rb >= c0i);
                open_rb = rt;
            }
            k0 = k1;
        }
        if (DS) {
            // step 4', LeakyReLU' and step 3' for the edges of the block, on the (edge, head) pairs of the record loads
            // above: dE = alpha*(dalpha - P), times the slope where the score was not positive, summed per (row segment,
            // head) in fp64.  A lane's pairs all have the same head (64 is a multiple of HP), so the sums of all heads
            // build up in the lanes and one reduction over the lanes of equal head per row serves them all.
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const int H = a.heads;
            int lane_o = lane;
            asm volatile("" : "+v"(lane_o));
            const int head = lane_o & (HP - 1);
            for (int g0 = 0; g0 < HP; g0 += 4) {  // four rounds at a time (one pass up to 4 heads, two up to 8)
                double contrib[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    contrib[j] = 0.0;
                    if (g0 + j >= HP) break;
                    const int edge = (lane_o + 64 * (g0 + j)) >> log2HP;
                    if (edge < cnt && head < H) {
                        const float da = static_cast<float>(dots_s[wv][edge * H + head]) * sc_dot;
                        const float als = alf_s[wv][edge * H + head];
                        double Pv = P_r[j];
                        if (g0 > 0) {  // more than four heads: rounds 4-7 fetch P again
                            const uint4 ent = nbw_s[wv][edge];  // the neighbour's row offset, back to its index
                            const int nbe = static_cast<int>(((static_cast<uint64_t>(ent.y) << 32) | ent.x) /
                                                             static_cast<uint32_t>(row_bytes));
                            Pv = static_cast<const tango_attn_rec *>(a.att.rec)[static_cast<int64_t>(nbe) * HP + head].P;
                        }
                        const float dE = static_cast<float>(static_cast<double>(fabsf(als)) * (static_cast<double>(da) - Pv));
                        contrib[j] = static_cast<double>(dE * (__float_as_int(als) < 0 ? a.att.slope : 1.0f));
                    }
                }
                for (int k0 = 0; k0 < cnt;) {
                    const int r = __builtin_amdgcn_readlane(my_row, k0);
                    const int k1 = min(__builtin_amdgcn_readlane(my_rt, k0) - base, cnt);
                    double v = 0.0;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int edge = (lane_o + 64 * (g0 + j)) >> log2HP;
                        if (g0 + j < HP && edge >= k0 && edge < k1) v += contrib[j];
                    }
                    // a row that runs on over many blocks (a hub) is summed in the lanes and leaves the wave once
                    if (r != ds_row) {
                        flush_dS();
                        ds_row = r;
                    }
                    ds_run += v;
                    k0 = k1;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
    if (DS) flush_dS();
    if (pending) finish_row(cur_r, false);  // the last row continues in the next chunk
    if (a.absmax) {
        // max|out| over whole rows = (float)max|acc| * sc (conversion and the product are monotone)
        float m = static_cast<float>(maxabs) * sc;
        m = tango_wave_max(m);
        if (lane == 0 && m > 0.0f) tango_atomic_max_nonneg(a.absmax, m);
    }
}

// Short rows (at most a.short_max <= 64 edges), plain weights, small graphs: each group of LPR lanes owns one row and
// walks its edges alone, so a wave works on G rows at once and a row needs no cross-group reduction, no atomics and no
// chunk search.  Small low-degree graphs spend most of their edges here; the chunked kernel above then only sees the
// longer rows.
constexpr int SHORT_ROWS = 16;
template <int VEC, bool HAS_EID, int UE>
__global__ __launch_bounds__(256) void k_spmm_short(spmm_args a)
{
    using V = typename vec_bytes<VEC>::type;
    const int lane = threadIdx.x % TANGO_WAVE;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) / TANGO_WAVE;
    const int nwaves = gridDim.x * blockDim.x / TANGO_WAVE;
    const int LPR = a.F / VEC;
    const int G = 64 / LPR;
    const int gi = lane / LPR;
    const int li = lane - gi * LPR;
    const bool active = gi < G;
    const int col = li * VEC;
    const int h = col / a.dim;
    const float sc = (*a.s_w) * (*a.s_X);
    const int8_t *Xcol = a.X + col;
    int maxabs = 0;
    // a wave takes a.short_rows rows per pass and walks a row's edges UE at a time (small graphs: 16 rows, so that there
    // are many waves, and eight edges, one round of gathers for the typical short row)
    const int RP = max(a.short_rows, G);  // rows per pass: at least one per group
    for (int64_t base = static_cast<int64_t>(wave) * RP; base < a.n; base += static_cast<int64_t>(nwaves) * RP) {
        const int rl = static_cast<int>(base) + lane;
        int pb = 0, pt = 0;
        if (lane < RP && rl < a.n) {
            pb = a.ptr[rl];
            pt = a.ptr[rl + 1];
        }
        for (int k0 = 0; k0 < RP; k0 += G) {
            const int src_lane = min(k0 + gi, RP - 1);
            const int rb = __shfl(pb, src_lane, 64), rt = __shfl(pt, src_lane, 64);
            const int row = static_cast<int>(base) + k0 + gi;
            const int deg = rt - rb;
            if (!active || row >= a.n || row >= base + RP || deg <= 0 || deg > a.short_max) continue;
            int acc[VEC];
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc[j] = 0;
            for (int e = rb; e < rt; e += UE) {
                uint32_t wq[UE];
                V xv[UE];
#pragma unroll
                for (int u = 0; u < UE; ++u) {
                    // (edges beyond the row's end: no load at all, a zero weight)
                    wq[u] = 0u;
                    xv[u] = V();
                    if (e + u < rt) {
                        const int ee = e + u;
                        const int nb = a.idx[ee];
                        const int64_t wp = (HAS_EID ? static_cast<int64_t>(a.eid[ee]) : static_cast<int64_t>(ee)) * a.heads + h;
                        wq[u] = static_cast<uint32_t>(static_cast<uint8_t>(a.w[wp]));
                        xv[u] = *reinterpret_cast<const V *>(Xcol + static_cast<int64_t>(nb) * a.F);
                    }
                }
#pragma unroll
                for (int u = 0; u < UE; u += 4) {
                    const uint32_t wpack = wq[u] | (wq[u + 1] << 8) | (wq[u + 2] << 16) | (wq[u + 3] << 24);
                    uint32_t w0[VEC / 4], w1[VEC / 4], w2[VEC / 4], w3[VEC / 4];
                    unpack_words<VEC>(xv[u], w0);
                    unpack_words<VEC>(xv[u + 1], w1);
                    unpack_words<VEC>(xv[u + 2], w2);
                    unpack_words<VEC>(xv[u + 3], w3);
#pragma unroll
                    for (int q = 0; q < VEC / 4; ++q) {
                        uint32_t t[4];
                        transpose4x4(w0[q], w1[q], w2[q], w3[q], t);
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            acc[4 * q + c] = __builtin_amdgcn_sdot4(static_cast<int>(t[c]), static_cast<int>(wpack), acc[4 * q + c], false);
                    }
                }
            }
            float *orow = a.out + static_cast<int64_t>(row) * a.F + col;
#pragma unroll
            for (int j = 0; j < VEC; j += 4) {
                float4 o;
                o.x = static_cast<float>(acc[j + 0]) * sc;
                o.y = static_cast<float>(acc[j + 1]) * sc;
                o.z = static_cast<float>(acc[j + 2]) * sc;
                o.w = static_cast<float>(acc[j + 3]) * sc;
                *reinterpret_cast<float4 *>(orow + j) = o;
                maxabs = max(maxabs, max(max(abs(acc[j]), abs(acc[j + 1])), max(abs(acc[j + 2]), abs(acc[j + 3]))));
            }
        }
    }
    if (a.absmax) {
        float m = static_cast<float>(maxabs) * sc;
        m = tango_wave_max(m);
        if (lane == 0 && m > 0.0f) tango_atomic_max_nonneg(a.absmax, m);
    }
}

// Tiny rows (1 .. T edges, T = a.short_max = 4 or 8), plain weights at the edge's own position.  On a low-degree graph most rows are tiny (the
// self-loop and a neighbour or two) and hold few of the edges: what such a row costs is its 4F bytes of output and the
// chain row pointer -> neighbour index -> row gather, not arithmetic.  So the chain is taken apart: a wave takes 64 rows
// per pass; lane l first fetches, for row base+l, the bounds and the (up to) T neighbour indices and weight codes of the
// row - T wave-wide loads serve 64 rows - and leaves them in LDS; then each group of LPR lanes owns one row at a time,
// reads its row's entry back (one broadcast LDS read) and issues nothing but the row gathers, T per row and RU rows deep,
// back to back.  No loop depends on a row's length, so the lanes of a wave never wait for its longest row.
template <int VEC, int T>
__global__ __launch_bounds__(256) void k_spmm_tiny(spmm_args a)
{
    static_assert(T == 4 || T == 8, "one or two rounds of four edges");
    using V = typename vec_bytes<VEC>::type;
    // per wave and row: the T neighbour indices (0xffffffff: no such edge) and the packed weight codes of the T edges
    __shared__ __align__(16) uint32_t nb_s[WAVES_PER_BLOCK][64][T];
    __shared__ __align__(16) uint32_t w_s[WAVES_PER_BLOCK][64][T];   // heads 0-3 of edge j
    __shared__ __align__(16) uint32_t w2_s[WAVES_PER_BLOCK][64][T];  // heads 4-7 of edge j
    const int lane = threadIdx.x % TANGO_WAVE;
    const int wv = threadIdx.x / TANGO_WAVE;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) / TANGO_WAVE;
    const int nwaves = gridDim.x * blockDim.x / TANGO_WAVE;
    const int LPR = a.F / VEC;
    const int G = 64 / LPR;
    const int gi = lane / LPR;
    const int li = lane - gi * LPR;
    const bool active = gi < G;
    const int col = li * VEC;
    const int h = col / a.dim;
    const bool upper_heads = h >= 4;
    const uint32_t hshift = 8u * static_cast<uint32_t>(h & 3);
    const float sc = (*a.s_w) * (*a.s_X);
    const int8_t *Xcol = a.X + col;
    int maxabs = 0;
    constexpr int RU = 2;  // rows in flight per group
    for (int64_t base = static_cast<int64_t>(wave) * 64; base < a.n; base += static_cast<int64_t>(nwaves) * 64) {
        {
            const int64_t r = base + lane;
            int pb = 0, deg = 0;
            if (r < a.n) {
                pb = a.ptr[r];
                deg = a.ptr[r + 1] - pb;
            }
            if (deg > T) deg = 0;  // not mine: left to the chunked kernel
            uint32_t nb[T], w[T], w2[T];
#pragma unroll
            for (int j = 0; j < T; ++j) {
                nb[j] = 0xffffffffu;  // "no edge"
                w[j] = 0u;
                w2[j] = 0u;
                if (j < deg) {
                    const int e = pb + j;
                    nb[j] = static_cast<uint32_t>(a.idx[e]);
                    const int64_t wp = static_cast<int64_t>(e) * a.heads;
                    if (a.w_words) {
                        w[j] = *reinterpret_cast<const uint32_t *>(a.w + wp);
                        if (a.heads == 8) w2[j] = *reinterpret_cast<const uint32_t *>(a.w + wp + 4);
                    } else {
                        for (int hh = 0; hh < a.heads; ++hh) {
                            const uint32_t b = static_cast<uint8_t>(a.w[wp + hh]);
                            if (hh < 4)
                                w[j] |= b << (8 * hh);
                            else
                                w2[j] |= b << (8 * (hh - 4));
                        }
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < T; j += 4) {
                *reinterpret_cast<uint4 *>(&nb_s[wv][lane][j]) = make_uint4(nb[j], nb[j + 1], nb[j + 2], nb[j + 3]);
                *reinterpret_cast<uint4 *>(&w_s[wv][lane][j]) = make_uint4(w[j], w[j + 1], w[j + 2], w[j + 3]);
                if (a.heads > 4) *reinterpret_cast<uint4 *>(&w2_s[wv][lane][j]) = make_uint4(w2[j], w2[j + 1], w2[j + 2], w2[j + 3]);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        if (active) {
            for (int k0 = 0; k0 < 64; k0 += G * RU) {
                uint32_t nbr[RU][T], wr[RU][T];
                V xv[RU][T];
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    const int sl = min(k0 + u * G + gi, 63);
                    const bool there = k0 + u * G + gi < 64;
#pragma unroll
                    for (int j = 0; j < T; j += 4) {
                        const uint4 n4 = *reinterpret_cast<const uint4 *>(&nb_s[wv][sl][j]);
                        const uint4 w4 = upper_heads ? *reinterpret_cast<const uint4 *>(&w2_s[wv][sl][j])
                                                     : *reinterpret_cast<const uint4 *>(&w_s[wv][sl][j]);
                        nbr[u][j] = there ? n4.x : 0xffffffffu; nbr[u][j + 1] = there ? n4.y : 0xffffffffu;
                        nbr[u][j + 2] = there ? n4.z : 0xffffffffu; nbr[u][j + 3] = there ? n4.w : 0xffffffffu;
                        wr[u][j] = w4.x; wr[u][j + 1] = w4.y; wr[u][j + 2] = w4.z; wr[u][j + 3] = w4.w;
                    }
#pragma unroll
                    for (int j = 0; j < T; ++j) {
                        xv[u][j] = V();
                        if (nbr[u][j] != 0xffffffffu)
                            xv[u][j] = *reinterpret_cast<const V *>(Xcol + static_cast<int64_t>(nbr[u][j]) * a.F);
                    }
                }
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    if (nbr[u][0] == 0xffffffffu) continue;  // no such row, an empty row or a longer one
                    int acc[VEC];
#pragma unroll
                    for (int j = 0; j < VEC; ++j) acc[j] = 0;
#pragma unroll
                    for (int j = 0; j < T; j += 4) {
                        const uint32_t wpack = ((wr[u][j] >> hshift) & 0xffu) | (((wr[u][j + 1] >> hshift) & 0xffu) << 8) |
                                               (((wr[u][j + 2] >> hshift) & 0xffu) << 16) | (((wr[u][j + 3] >> hshift) & 0xffu) << 24);
                        uint32_t w0[VEC / 4], w1[VEC / 4], w2[VEC / 4], w3[VEC / 4];
                        unpack_words<VEC>(xv[u][j], w0);
                        unpack_words<VEC>(xv[u][j + 1], w1);
                        unpack_words<VEC>(xv[u][j + 2], w2);
                        unpack_words<VEC>(xv[u][j + 3], w3);
#pragma unroll
                        for (int q = 0; q < VEC / 4; ++q) {
                            uint32_t t[4];
                            transpose4x4(w0[q], w1[q], w2[q], w3[q], t);
#pragma unroll
                            for (int c = 0; c < 4; ++c)
                                acc[4 * q + c] = __builtin_amdgcn_sdot4(static_cast<int>(t[c]), static_cast<int>(wpack), acc[4 * q + c], false);
                        }
                    }
                    const int64_t row = base + k0 + u * G + gi;
                    float *orow = a.out + row * a.F + col;
#pragma unroll
                    for (int j = 0; j < VEC; j += 4) {
                        float4 o;
                        o.x = static_cast<float>(acc[j + 0]) * sc;
                        o.y = static_cast<float>(acc[j + 1]) * sc;
                        o.z = static_cast<float>(acc[j + 2]) * sc;
                        o.w = static_cast<float>(acc[j + 3]) * sc;
                        *reinterpret_cast<float4 *>(orow + j) = o;
                        maxabs = max(maxabs, max(max(abs(acc[j]), abs(acc[j + 1])), max(abs(acc[j + 2]), abs(acc[j + 3]))));
                    }
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();  // the entries are overwritten by the next pass
    }
    if (a.absmax) {
        float m = static_cast<float>(maxabs) * sc;
        m = tango_wave_max(m);
        if (lane == 0 && m > 0.0f) tango_atomic_max_nonneg(a.absmax, m);
    }
}

struct sddmm_dot_args {
    int n;
    int64_t nnz;
    const int32_t *ptr;   // in_ptr
    const int32_t *idx;   // in_src
    const int8_t *Xdst;   // n x F
    const int8_t *Xsrc;   // n x F
    const float *s_dst, *s_src;
    float *out;           // nnz x heads
    int heads, dim, F;
    // ATT_BWD instantiations only (rows = source nodes, ptr/idx = out_ptr/out_dst): instead of storing the
    // dot products, turn each into the gradient of the pre-activation score and sum it per (source, head)
    const int8_t *Sq, *Dq;
    const float *sS, *sD;
    float slope;
    const void *rec;       // per destination: row_lse and P of every head
    double *dS_acc;                  // n x heads, zero-initialised
    // DOT_DST instantiations only (rows = destination nodes): three running sums per (destination, head)
    const float *row_lse;            // n x heads
    int chunk_shift = CHUNK_SHIFT_DEFAULT;  // log2 of the edges per wavefront
    const int8_t *src_codes = nullptr;  // optional: S_q[src(e)] per in-edge, in edge order (read instead of gathered)
    double *stats;                   // n x heads x 3, zero-initialised: sum alpha*dalpha, sum alpha*dalpha*s, sum alpha*s
};

enum { DOT_STORE = 0, DOT_SRC = 1, DOT_DST = 2 };

// out[e][h] = (float)(Xdst[dst(e)][h][:] . Xsrc[src(e)][h][:]) * (s_dst*s_src); one wave per chunk of edges.
// ATT_BWD (step 3' fused with 5'', 4' and LeakyReLU', walking the out-edges of each source u): the dot product
// of edge (u -> v) is dalpha, alpha is recomputed from S_q[u], D_q[v], row_max[v], row_rden[v], and
// dS_acc[u][h] += alpha*(dalpha - P[v][h]) * lrelu'(t).
// DOT_DST (steps 5'', 4', 3'' in one walk over the in-edges of each destination v, nothing stored per edge): with
// s = 1 or the LeakyReLU slope by the sign of the pre-activation score, dE = alpha*(dalpha - P)*s summed over the
// row is B - P*C with P = A = sum alpha*dalpha, B = sum alpha*dalpha*s, C = sum alpha*s; the three sums go to
// stats[v][h][0..2] in fp64 and a finishing kernel forms P and dD.
// I4: both tables hold packed 4-bit codes; a.F and a.dim then count bytes (two columns each) and the products come
// from v_dot8_i32_i4.
// LPHC: lanes per head when known at compile time (0: computed from the arguments).
template <int VEC, int MODE, bool I4 = false, int LPHC = 0>
__global__ __launch_bounds__(64 * WAVES_PER_BLOCK) void k_sddmm_dot(sddmm_dot_args a)
{
    constexpr bool ATT_BWD = MODE == DOT_SRC;
    constexpr bool ATT_DST = MODE == DOT_DST;
    using V = typename vec_bytes<VEC>::type;
    // per wave: the dot products of a block of 64 edges (edge-major, heads <= 8) and the neighbours of those edges
    __shared__ int dots[WAVES_PER_BLOCK][64 * 8];
    __shared__ int nbl[WAVES_PER_BLOCK][64];
    __shared__ double red[ATT_BWD ? WAVES_PER_BLOCK : 1][64];
    // DOT_DST: the packed S_q codes (heads 0-3, 4-7) of the sources of a block's edges, fetched before the gathers
    __shared__ uint2 sqw_s[ATT_DST ? WAVES_PER_BLOCK : 1][ATT_DST ? 64 : 1];
    const int lane = threadIdx.x % TANGO_WAVE;
    const int wv = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x / TANGO_WAVE));  // wave-uniform, see k_spmm
    const int64_t chunk = static_cast<int64_t>(blockIdx.x) * WAVES_PER_BLOCK + wv;
    const int64_t c0 = chunk << a.chunk_shift;
    if (c0 >= a.nnz) return;
    const int64_t c1 = min(c0 + (int64_t(1) << a.chunk_shift), a.nnz);

    const int H = a.heads;
    const int LPR = a.F / VEC;
    const int G = 64 / LPR;
    const int gi = lane / LPR;
    const int li = lane - gi * LPR;
    const bool active = gi < G;
    const int col = li * VEC;
    const int h = col / a.dim;
    const int LPH = LPHC ? LPHC : a.dim / VEC;  // lanes per head (power of two)
    const float sc = (*a.s_dst) * (*a.s_src);
    constexpr int U = 8;
    // epilogue mapping: lane l < S handles the (edge, head) pairs l, l+S, l+2S, ... of a block, S a multiple of
    // the head count so that a lane always sees the same head.  DOT_DST: the head count is padded to a power of two
    // (lanes of a padding head idle), so that the lanes of one head are a fixed stride apart and the row sums can be
    // formed by lane rotations
    const int HP = ATT_DST ? tango_rec_heads(H) : H;
    const int S = (64 / HP) * HP;
    const int eh = lane % HP;      // my head in the epilogue
    const int ek0 = lane / HP;     // my first edge of a block
    const int ekstep = S / HP;
    const bool ep_on = lane < S && eh < H;
    float sS = 0.0f, sD = 0.0f;
    if (ATT_BWD || ATT_DST) {
        sS = *a.sS;
        sD = *a.sD;
    }

    // the blocks of a chunk follow each other in the edge array whatever rows they belong to, so the neighbour indices
    // of the next block can be requested while this one is gathered
    int nb_ahead = (c0 + lane < c1) ? a.idx[c0 + lane] : 0;
    int r = wave_find_row(a.ptr, a.n, static_cast<int>(c0));
    // row ends of 64 rows at a time in the lanes (one coalesced load instead of a dependent scalar load per row)
    int win_r0 = r;
    int win_end = (win_r0 + lane < a.n) ? a.ptr[win_r0 + lane + 1] : 0x7fffffff;
    int rb_next = a.ptr[r];
    for (; r < a.n; ++r) {
        if (r - win_r0 >= 64) {
            win_r0 = r;
            win_end = (win_r0 + lane < a.n) ? a.ptr[win_r0 + lane + 1] : 0x7fffffff;
        }
        const int rb = rb_next, rt = __builtin_amdgcn_readlane(win_end, r - win_r0);
        rb_next = rt;
        if (rb >= c1) break;
        const int sb = max(rb, static_cast<int>(c0)), se = min(rt, static_cast<int>(c1));
        if (sb >= se) continue;
        uint32_t dw[VEC / 4];
        {
            const V dv = *reinterpret_cast<const V *>(a.Xdst + static_cast<int64_t>(r) * a.F + (active ? col : 0));
            unpack_words<VEC>(dv, dw);
        }
        float td_row = 0.0f, lse_row = 0.0f;
        if (ATT_DST && ep_on) {
            td_row = sD * static_cast<float>(a.Dq[static_cast<int64_t>(r) * H + eh]);
            lse_row = a.row_lse[static_cast<int64_t>(r) * H + eh];
        }
        float ts_row = 0.0f;
        double acc_s = 0.0;
        if (ATT_BWD && lane < S) ts_row = sS * static_cast<float>(a.Sq[static_cast<int64_t>(r) * H + eh]);
        double acc_a = 0.0, acc_b = 0.0, acc_c = 0.0;
        for (int base = sb; base < se; base += 64) {
            const int cnt = min(64, se - base);
            const int my_nb = lane < cnt ? nb_ahead : 0;
            if (base + cnt + lane < c1) nb_ahead = a.idx[base + cnt + lane];
            if (ATT_BWD || ATT_DST) nbl[wv][lane] = my_nb;
            if (ATT_DST) {
                // S_q of my edge's source, all heads, needed only after the gathers: requested now
                uint2 w = make_uint2(0u, 0u);
                if (lane < cnt) {
                    const int8_t *sp = a.src_codes ? a.src_codes + (static_cast<int64_t>(base) + lane) * H
                                                   : a.Sq + static_cast<int64_t>(my_nb) * H;
                    if (H == 4) {
                        w.x = *reinterpret_cast<const uint32_t *>(sp);
                    } else if (H == 8) {
                        w = *reinterpret_cast<const uint2 *>(sp);
                    } else {
                        for (int hh = 0; hh < H; ++hh) {
                            const uint32_t b = static_cast<uint8_t>(sp[hh]);
                            if (hh < 4)
                                w.x |= b << (8 * hh);
                            else
                                w.y |= b << (8 * (hh - 4));
                        }
                    }
                }
                sqw_s[wv][lane] = w;
            }
            const int steps = (cnt + G - 1) / G;
            auto batch = [&](int s0, auto uu, auto masked) {
                constexpr int UU = decltype(uu)::value;
                constexpr bool MASKED = decltype(masked)::value;  // the last steps of a block may lie beyond its edges
                int dot[UU];
#pragma unroll
                for (int u = 0; u < UU; ++u) {
                    const int k = (s0 + u) * G + gi;
                    const bool ok = active && k < cnt;
                    const int nb = __shfl(my_nb, ok ? k : 0, 64);
                    V xv = V();
                    if (!MASKED || ok)
                        xv = *reinterpret_cast<const V *>(a.Xsrc + static_cast<int64_t>(nb) * a.F + (active ? col : 0));
                    uint32_t w[VEC / 4];
                    unpack_words<VEC>(xv, w);
                    int d = 0;
#pragma unroll
                    for (int j = 0; j < VEC / 4; ++j)
                        d = I4 ? __builtin_amdgcn_sdot8(static_cast<int>(dw[j]), static_cast<int>(w[j]), d, false)
                               : __builtin_amdgcn_sdot4(static_cast<int>(dw[j]), static_cast<int>(w[j]), d, false);
                    dot[u] = d;
                }
#pragma unroll
                for (int u = 0; u < UU; ++u) {
                    const int d = tango_group_sum_c<LPHC>(dot[u], LPH);
                    const int k = (s0 + u) * G + gi;
                    if (active && k < cnt && (li % LPH) == 0) dots[wv][k * H + h] = d;
                }
            };
            // whole batches of U steps, then what is left in one more batch (2, 4 or U steps, the excess masked): a
            // short row costs two rounds of gathers, not one per pair of steps
            const int full_steps = cnt / G;  // steps in which every group has an edge
            int s0 = 0;
            for (; s0 + U <= full_steps; s0 += U) batch(s0, std::integral_constant<int, U>{}, std::false_type{});
            const int left = steps - s0;
            if (left > 4) batch(s0, std::integral_constant<int, U>{}, std::true_type{});
            else if (left > 2) batch(s0, std::integral_constant<int, 4>{}, std::true_type{});
            else if (left > 0) batch(s0, std::integral_constant<int, 2>{}, std::true_type{});
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            // epilogue at full lane occupancy: one (edge, head) pair per lane and step
            if (ep_on) {
                for (int k = ek0; k < cnt; k += ekstep) {
                    const float da = static_cast<float>(dots[wv][k * H + eh]) * sc;
                    if (ATT_BWD) {
                        const int64_t vh = static_cast<int64_t>(nbl[wv][k]) * H + eh;
                        bool pos;
                        const float ev = tango_attn_score(ts_row, sD * static_cast<float>(a.Dq[vh]), a.slope, pos);
                        const tango_attn_rec rc =
                            static_cast<const tango_attn_rec *>(a.rec)[static_cast<int64_t>(nbl[wv][k]) * tango_rec_heads(H) + eh];
                        const float al = tango_attn_alpha(ev, rc.row_lse);
                        const float dE = static_cast<float>(static_cast<double>(al) * (static_cast<double>(da) - rc.P));
                        acc_s += static_cast<double>(dE * (pos ? 1.0f : a.slope));
                    } else if (ATT_DST) {
                        const uint2 sw = sqw_s[wv][k];
                        const int sq = static_cast<int>(static_cast<int8_t>((eh < 4 ? sw.x : sw.y) >> (8 * (eh & 3))));
                        bool pos;
                        const float ev = tango_attn_score(sS * static_cast<float>(sq), td_row, a.slope, pos);
                        const float al = tango_attn_alpha(ev, lse_row);
                        const double ad = static_cast<double>(al) * static_cast<double>(da);
                        const double sl = pos ? 1.0 : static_cast<double>(a.slope);
                        acc_a += ad;
                        acc_b += ad * sl;
                        acc_c += static_cast<double>(al) * sl;
                    } else {
                        a.out[(static_cast<int64_t>(base) + k) * H + eh] = da;
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        if (ATT_DST) {
            // the lanes of one head are HP apart: after the rotations every lane holds its head's three sums
            const double ta = tango_stride_sum_f64(acc_a, HP);
            const double tb = tango_stride_sum_f64(acc_b, HP);
            const double tc = tango_stride_sum_f64(acc_c, HP);
            const int w = lane / HP;  // lane = HP*(which sum) + head
            if (w < 3 && eh < H) {
                const double t = w == 0 ? ta : (w == 1 ? tb : tc);
                if (t != 0.0) atomicAdd(a.stats + (static_cast<int64_t>(r) * H + eh) * 3 + w, t);
            }
        }
        if (ATT_BWD) {
            // sum the lanes that share a head (lanes eh, eh+H, ...), in lane order
            red[wv][lane] = (lane < S) ? acc_s : 0.0;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (lane < H) {
                double t = 0.0;
                for (int l = lane; l < S; l += H) t += red[wv][l];
                if (t != 0.0) atomicAdd(a.dS_acc + static_cast<int64_t>(r) * H + lane, t);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
}

__global__ __launch_bounds__(256) void k_f64_to_f32(const double *__restrict__ x, int64_t n, float *__restrict__ y)
{
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x)
        y[i] = static_cast<float>(x[i]);
}

bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

// SDDMM-dot: 256 edges per wavefront, 64 on graphs too small to give every SIMD a few such chunks (a wave walks its
// rows one after the other, so on a small graph the longest chain of rows sets the time)
int dot_chunk_shift(int64_t nnz) { return (nnz >> CHUNK_SHIFT_DEFAULT) >= 4096 ? CHUNK_SHIFT_DEFAULT : 6; }

// Bytes of a feature row per lane: aim at ~16 lanes per row.  Every lane's bytes must stay inside one
// head, the lanes of one row must fit a wave, and the number of row groups per wave must be a power
// of two (shuffle reduction); SDDMM-dot also needs a power-of-two number of lanes per head.
// Returns 0 when no width qualifies.
int pick_vec(int F, int dim, bool pow2_lanes_per_head, bool wide_lanes = false)
{
    int pref[3] = {16, 8, 4};
    // wide_lanes (the plain in-direction SPMM and the plain SDDMM-dot, measured on 32- to 128-byte rows of a large
    // table): 16 bytes per lane also for narrow rows - more rows per load instruction, 8-20 % faster there
    if (wide_lanes && F >= 32) { /* 16, 8, 4 */ }
    else if (F <= 64) { pref[0] = 4; pref[1] = 8; pref[2] = 16; }
    else if (F <= 128) { pref[0] = 8; pref[1] = 4; pref[2] = 16; }
    for (int i = 0; i < 3; ++i) {
        const int vec = pref[i];
        if (dim % vec != 0 || F % vec != 0) continue;
        const int lpr = F / vec;
        if (lpr > 64 || !is_pow2(64 / lpr)) continue;
        if (pow2_lanes_per_head && !is_pow2(dim / vec)) continue;
        return vec;
    }
    return 0;
}

// Packed 4-bit rows (F/2 bytes): bytes per lane for the SPMM, 8 or 4 (16 or 8 columns per lane, all in one head,
// lanes per row dividing 64); 0 when neither fits.
int pick_vec_i4(int F, int dim)
{
    const int pref[2] = {F <= 128 ? 4 : 8, F <= 128 ? 8 : 4};
    for (int i = 0; i < 2; ++i) {
        const int cpl = 2 * pref[i];
        if (dim % cpl != 0 || F % cpl != 0) continue;
        const int lpr = F / cpl;
        if (lpr > 64 || !is_pow2(64 / lpr)) continue;
        return pref[i];
    }
    return 0;
}

// w_src[j][h] = w[eid[j]][h]: edge codes from destination-major to source-major order.
__global__ __launch_bounds__(256) void k_edge_to_src_order(int64_t nnz, int heads, const int32_t *__restrict__ eid,
                                                           const int8_t *__restrict__ w, int8_t *__restrict__ w_src)
{
    for (int64_t j = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; j < nnz;
         j += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const int64_t e = eid[j];
        for (int h = 0; h < heads; ++h) w_src[j * heads + h] = w[e * heads + h];
    }
}

int validate_graph_dir(const tango_graph *g, int direction)
{
    TANGO_REQUIRE(g != nullptr, TANGO_ERR_NULL);
    TANGO_REQUIRE(g->n_nodes > 0 && g->n_edges >= 0 && g->n_edges < (int64_t(1) << 31), TANGO_ERR_BAD_SHAPE);
    if (direction == TANGO_IN) {
        TANGO_REQUIRE(g->in_ptr && (g->n_edges == 0 || g->in_src), TANGO_ERR_NULL);
    } else if (direction == TANGO_OUT) {
        TANGO_REQUIRE(g->out_ptr && (g->n_edges == 0 || (g->out_dst && g->out_eid)), TANGO_ERR_NULL);
    } else {
        TANGO_REQUIRE(g->out_ptr && (g->n_edges == 0 || g->out_dst), TANGO_ERR_NULL);
    }
    return TANGO_OK;
}

int validate_feature_shape(int heads, int dim)
{
    TANGO_REQUIRE(heads >= 1 && heads <= 8 && dim >= 4 && dim % 4 == 0, TANGO_ERR_BAD_SHAPE);
    const int64_t F = static_cast<int64_t>(heads) * dim;
    TANGO_REQUIRE(F <= 1024, TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(pick_vec(static_cast<int>(F), dim, false) != 0, TANGO_ERR_UNSUPPORTED);
    return TANGO_OK;
}

}  // namespace

// The forward attention SPMM can also write its ReLU's sign bits when every lane holds 16 columns (one 16-bit store per
// lane) and a row is a whole number of 64-bit words.
bool tango_spmm_relu_bits_supported(int64_t n_nodes, int heads, int dim)
{
    const int F = heads * dim;
    return validate_feature_shape(heads, dim) == TANGO_OK && F % 64 == 0 && pick_vec(F, dim, false) == 16 &&
           n_nodes * (F / 16) < (int64_t(1) << 32);  // halfword index kept in 32 bits
}

static int spmm_launch(const tango_graph *g, int direction, int heads, int dim, const int8_t *w_q, const float *s_w,
                       const int8_t *X_q, const float *s_X, float *out, float *absmax_out, const attn_params *att,
                       hipStream_t st, bool x4 = false, float *dS_out = nullptr, bool out_prezeroed = false)
{
    spmm_args a;
    if (att) a.att = *att;
    // dS_out (reverse attention pass fused with step 3' only): the fp32 copy of the dS sums, written by the last launch
    a.cvt_src = (att && att->rec && dS_out) ? att->dS_acc : nullptr;
    a.cvt_dst = dS_out;
    a.cvt_n = static_cast<int64_t>(g->n_nodes) * heads;
    a.relu = (att && direction == TANGO_IN) ? att->relu_out : 0;
    a.relu_bits = (a.relu && att->relu_bits && tango_spmm_relu_bits_supported(g->n_nodes, heads, dim)) ? att->relu_bits : nullptr;
    a.w_words = (heads == 4 || heads == 8) && w_q != nullptr && tango_aligned(w_q, 4);
    a.n = g->n_nodes;
    a.nnz = g->n_edges;
    a.ptr = direction == TANGO_IN ? g->in_ptr : g->out_ptr;
    a.idx = direction == TANGO_IN ? g->in_src : g->out_dst;
    a.eid = direction == TANGO_OUT ? g->out_eid : nullptr;  // TANGO_OUT_SRC_ORDER: the weights are already in this order
    a.w = w_q;
    a.X = X_q;
    a.s_w = s_w;
    a.s_X = s_X;
    a.out = out;
    a.absmax = absmax_out;
    a.heads = heads;
    a.dim = dim;
    a.F = heads * dim;
    // edges per wavefront: large chunks mean fewer rows cut by a boundary (fewer atomics); small graphs
    // need small chunks to fill 256 CUs
    a.chunk_shift = 6;
    if ((a.nnz >> 10) >= 16384) a.chunk_shift = 10;  // at least 16 waves per SIMD worth of chunks
    else if ((a.nnz >> 8) >= 4096) a.chunk_shift = 8;
    // Low mean degree, plain weights.  Small graphs (too few rows to fill the chip with 64-row passes), either
    // direction, rows of at most two cache lines: rows of up to 64 edges go to the group-per-row kernel (measured: 3-20 %
    // faster there).  Large graphs, weights at the edge's own position: the tiny rows (the self-loop and a few
    // neighbours: most of the rows, few of the edges) go to k_spmm_tiny, everything longer to the chunked kernel
    // (measured on the scale-22 graph: 2.50 -> 2.09 ms at F = 128, 4.21 -> 3.56 ms at F = 256; with weights fetched
    // through the edge-id map the dependent byte reads make it slower, so the reversed direction keeps one kernel).
    const bool small_graph = a.n < 64 * 1024 * 8;
    const bool low_degree = !x4 && !att && a.n > 0 && a.nnz / a.n <= 20;
    int tiny = 0;
    a.short_max = 0;
    if (low_degree && small_graph && a.F <= 256) a.short_max = 64;
    else if (low_degree && !a.eid && a.F <= 512) a.short_max = tiny = (a.F <= 128 ? 8 : 4);
    // (a wave of the two helper kernels handles the flagged rows of its pass one after the other: where split rows are
    // dense - fewer than 16 rows per chunk boundary, i.e. small graphs and long rows - short passes spread that chain of
    // dependent row accesses over more waves: finalize 8.1 -> 4.0 us on a 1,024-node graph, 62 -> 39 us at 233 k rows of
    // ~490 edges; with 39 rows per boundary (2.4 M rows of ~26 edges) the long passes are faster)
    const int64_t rows_per_boundary = a.nnz > 0 ? (static_cast<int64_t>(a.n) << a.chunk_shift) / a.nnz : 64;
    a.fin_rows = rows_per_boundary < 16 ? 8 : 64;
    const unsigned row_blocks = tango_grid_for((static_cast<size_t>(a.n) + a.fin_rows - 1) / a.fin_rows, 4, 256 * 8);
    // (out_prezeroed: an earlier launch of the caller's chain cleared all of out, the sign bits and *absmax_out, which
    // covers what the prepare pass clears - the rows the main kernel adds to or never writes)
    if (!out_prezeroed) {
        k_spmm_prepare<<<row_blocks, 256, 0, st>>>(a);
        TANGO_LAUNCH_CHECK();
    }
    if (tiny && a.nnz > 0) {
        const int vec = pick_vec(a.F, dim, false, true);
        const unsigned sb = tango_grid_for((static_cast<size_t>(a.n) + 63) / 64, 4, 256 * 32);
#define TANGO_SPMM_TINY(V_)                                        \
    if (tiny == 4) k_spmm_tiny<V_, 4><<<sb, 256, 0, st>>>(a); \
    else k_spmm_tiny<V_, 8><<<sb, 256, 0, st>>>(a);
        if (vec == 4) { TANGO_SPMM_TINY(4) } else if (vec == 8) { TANGO_SPMM_TINY(8) } else { TANGO_SPMM_TINY(16) }
#undef TANGO_SPMM_TINY
        TANGO_LAUNCH_CHECK();
    } else if (a.short_max > 0 && a.nnz > 0) {
        const int vec = pick_vec(a.F, dim, false, !a.eid);
        a.short_rows = SHORT_ROWS;
        const int rp = std::max(a.short_rows, 64 / (a.F / vec));  // as in the kernel
        const unsigned sb = tango_grid_for((static_cast<size_t>(a.n) + rp - 1) / rp, 4, 256 * 32);
#define TANGO_SPMM_SHORT(V_)                                     \
    if (a.eid)                                                   \
        k_spmm_short<V_, true, 8><<<sb, 256, 0, st>>>(a);        \
    else                                                         \
        k_spmm_short<V_, false, 8><<<sb, 256, 0, st>>>(a);
        if (vec == 4) { TANGO_SPMM_SHORT(4) } else if (vec == 8) { TANGO_SPMM_SHORT(8) } else { TANGO_SPMM_SHORT(16) }
#undef TANGO_SPMM_SHORT
        TANGO_LAUNCH_CHECK();
    }
    if (a.nnz > 0) {
        const int64_t chunks = (a.nnz + (int64_t(1) << a.chunk_shift) - 1) >> a.chunk_shift;
        const unsigned blocks = static_cast<unsigned>((chunks + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
        if (x4) {  // packed 4-bit table, plain weights
            const int vec = pick_vec_i4(a.F, dim);
            if (vec == 4) {
                if (a.eid) k_spmm<4, true, W_LOAD, true><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
                else k_spmm<4, false, W_LOAD, true><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
            } else {
                if (a.eid) k_spmm<8, true, W_LOAD, true><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
                else k_spmm<8, false, W_LOAD, true><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
            }
            TANGO_LAUNCH_CHECK();
            k_spmm_finalize<<<row_blocks, 256, 0, st>>>(a);
            TANGO_LAUNCH_CHECK();
            return TANGO_OK;
        }
        if (att && att->rec) {  // reverse attention SPMM fused with step 3'
            switch (pick_vec(a.F, dim, true)) {
                case 4: k_spmm<4, true, W_ATT_REV, false, true><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a); break;
                case 8: k_spmm<8, true, W_ATT_REV, false, true><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a); break;
                default:
                    if (dim == 64) k_spmm<16, true, W_ATT_REV, false, true, 4><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
                    else if (dim == 128) k_spmm<16, true, W_ATT_REV, false, true, 8><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
                    else k_spmm<16, true, W_ATT_REV, false, true><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
                    break;
            }
            TANGO_LAUNCH_CHECK();
            k_spmm_finalize<<<row_blocks, 256, 0, st>>>(a);
            TANGO_LAUNCH_CHECK();
            return TANGO_OK;
        }
        const int vec = pick_vec(a.F, dim, false, !att && !a.eid);
#define TANGO_SPMM(V_)                                                                  \
    if (att && a.eid)                                                                   \
        k_spmm<V_, true, W_ATT_REV><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);        \
    else if (att)                                                                       \
        k_spmm<V_, false, W_ATT_FWD><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);       \
    else if (a.eid)                                                                     \
        k_spmm<V_, true, W_LOAD><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);           \
    else                                                                                \
        k_spmm<V_, false, W_LOAD><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
        if (vec == 4) { TANGO_SPMM(4) } else if (vec == 8) { TANGO_SPMM(8) } else { TANGO_SPMM(16) }
#undef TANGO_SPMM
        TANGO_LAUNCH_CHECK();
        k_spmm_finalize<<<row_blocks, 256, 0, st>>>(a);
        TANGO_LAUNCH_CHECK();
    }
    return TANGO_OK;
}

int tango_spmm_async(const tango_graph *g, int direction, int heads, int dim, const int8_t *w_q, const float *s_w,
                     const int8_t *X_q, const float *s_X, float *out, float *absmax_out, hipStream_t st)
{
    return spmm_launch(g, direction, heads, dim, w_q, s_w, X_q, s_X, out, absmax_out, nullptr, st);
}

// SPMM whose weights are the attention scores computed (and quantized) on the fly.  direction TANGO_IN: forward
// (step 5), also stores alpha_q / s_alpha / alpha_dump.  direction TANGO_OUT: step 5' on the reversed graph; the
// same int8 codes are recomputed, nothing is stored, s_alpha is read.
int tango_spmm_attention_async(const tango_graph *g, int direction, int heads, int dim, const int8_t *Sq,
                               const float *sS, const int8_t *Dq, const float *sD, float slope, const float *row_lse,
                               const float *absmax_alpha, int rounding, uint64_t seed, uint64_t stream_id,
                               int8_t *alpha_q, float *s_alpha, float *alpha_dump, const int8_t *X_q, const float *s_X,
                               float *out, float *absmax_out, int relu_out, uint16_t *relu_bits, const int8_t *src_codes,
                               hipStream_t st, bool out_prezeroed)
{
    attn_params att;
    att.relu_out = relu_out;
    att.relu_bits = relu_bits;
    att.src_codes = direction == TANGO_IN ? src_codes : nullptr;
    att.Sq = Sq; att.Dq = Dq; att.sS = sS; att.sD = sD; att.slope = slope;
    att.row_lse = row_lse; att.absmax_alpha = absmax_alpha;
    att.rng = tango_rng_make(seed, stream_id); att.rounding = rounding;
    att.alpha_q = alpha_q; att.s_alpha = s_alpha; att.alpha_dump = alpha_dump;
    att.Xrow = nullptr; att.s_Xrow = nullptr; att.rec = nullptr; att.dS_acc = nullptr;
    return spmm_launch(g, direction, heads, dim, alpha_q, s_alpha, X_q, s_X, out, absmax_out, &att, st, false, nullptr, out_prezeroed);
}

// Steps 5' and 3' in one walk over the out-edges (attention codes recomputed): out = the reverse SPMM of dOut_q,
// dS[u][h] = sum over out-edges of dE.  rec holds (P, row_lse) per (destination, head); dS_acc: n x heads doubles
// of scratch.  heads*dim must also satisfy the SDDMM-dot shape rule (power-of-two lanes per head).
int tango_spmm_attention_rev_ds_async(const tango_graph *g, int heads, int dim, const int8_t *Sq, const float *sS,
                                      const int8_t *Dq, const float *sD, float slope, const float *row_lse,
                                      const float *absmax_alpha, int rounding, uint64_t seed, uint64_t stream_id,
                                      const float *s_alpha, const int8_t *dOut_q, const float *s_dOut, const int8_t *X_q,
                                      const float *s_X, const void *rec, double *dS_acc, float *out,
                                      float *absmax_out, float *dS, bool dS_acc_zeroed, hipStream_t st, bool out_prezeroed)
{
    const int64_t nh = static_cast<int64_t>(g->n_nodes) * heads;
    int rc = TANGO_OK;
    if (!dS_acc_zeroed) rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(dS_acc), 0u, 2 * nh, st);
    if (rc != TANGO_OK) return rc;
    attn_params att;
    att.Sq = Sq; att.Dq = Dq; att.sS = sS; att.sD = sD; att.slope = slope;
    att.row_lse = row_lse; att.absmax_alpha = absmax_alpha;
    att.rng = tango_rng_make(seed, stream_id); att.rounding = rounding;
    att.alpha_q = nullptr; att.s_alpha = const_cast<float *>(s_alpha); att.alpha_dump = nullptr;
    att.Xrow = X_q; att.s_Xrow = s_X; att.rec = rec; att.dS_acc = dS_acc; att.relu_out = 0; att.relu_bits = nullptr; att.src_codes = nullptr;
    rc = spmm_launch(g, TANGO_OUT, heads, dim, nullptr, s_alpha, dOut_q, s_dOut, out, absmax_out, &att, st, false, dS, out_prezeroed);
    if (rc != TANGO_OK) return rc;
    if (g->n_edges == 0) {  // no edge, no main kernel and no finalize launch: dS = 0 from the cleared sums
        k_f64_to_f32<<<tango_grid_for(static_cast<size_t>(nh), 256), 256, 0, st>>>(dS_acc, nh, dS);
        TANGO_LAUNCH_CHECK();
    }
    return TANGO_OK;
}

int tango_validate_spmm_shape(int heads, int dim) { return validate_feature_shape(heads, dim); }

int tango_sddmm_dot_async(const tango_graph *g, int heads, int dim, const int8_t *X_dst, const float *s_dst,
                          const int8_t *X_src, const float *s_src, float *out, hipStream_t st)
{
    if (g->n_edges == 0) return TANGO_OK;
    sddmm_dot_args a;
    a.n = g->n_nodes;
    a.nnz = g->n_edges;
    a.ptr = g->in_ptr;
    a.idx = g->in_src;
    a.Xdst = X_dst;
    a.Xsrc = X_src;
    a.s_dst = s_dst;
    a.s_src = s_src;
    a.out = out;
    a.heads = heads;
    a.dim = dim;
    a.F = heads * dim;
    a.chunk_shift = dot_chunk_shift(a.nnz);
        const int64_t chunks = (a.nnz + (int64_t(1) << a.chunk_shift) - 1) >> a.chunk_shift;
    const unsigned blocks = static_cast<unsigned>((chunks + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
    switch (pick_vec(a.F, dim, true, true)) {
        case 4: k_sddmm_dot<4, DOT_STORE><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a); break;
        case 8: k_sddmm_dot<8, DOT_STORE><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a); break;
        default:
            if (a.dim == 64) k_sddmm_dot<16, DOT_STORE, false, 4><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
            else if (a.dim == 128) k_sddmm_dot<16, DOT_STORE, false, 8><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
            else k_sddmm_dot<16, DOT_STORE><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
            break;
    }
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

__global__ __launch_bounds__(256) void k_attn_dst_finish(int64_t nh, int heads, const double *__restrict__ stats, const float *__restrict__ row_lse,
                                                         const int8_t *__restrict__ Dq,
                                                         void *__restrict__ rec, float *__restrict__ dD)
{
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < nh;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const double A = stats[3 * i], B = stats[3 * i + 1], C = stats[3 * i + 2];
        const int64_t node = i / heads;
        const int h = static_cast<int>(i - node * heads);
        tango_attn_rec rc;
        rc.P = A;
        rc.row_lse = row_lse[i];
        rc.dq = static_cast<int>(Dq[i]);
        static_cast<tango_attn_rec *>(rec)[node * tango_rec_heads(heads) + h] = rc;
        dD[i] = static_cast<float>(B - A * C);
    }
}

// Steps 5'', 4' and 3'' without an edge tensor: P (into rec) and dD from one walk over the in-edges; stats: n x heads x 3
// doubles of scratch.
int tango_attn_bwd_dst_fused_async(const tango_graph *g, int heads, int dim, const int8_t *dOut_q, const float *s_dOut,
                                   const int8_t *X_q, const float *s_X, const int8_t *Sq, const float *sS, const int8_t *Dq,
                                   const float *sD, float slope, const float *row_lse, double *stats, void *rec,
                                   float *dD, const int8_t *src_codes, double *also_zero, bool prezeroed, hipStream_t st)
{
    // also_zero (may be NULL): n x heads more doubles zeroed by the same launch (the source-side pass's accumulator);
    // prezeroed: both were cleared by an earlier launch on this stream
    const int64_t nh = static_cast<int64_t>(g->n_nodes) * heads;
    if (!prezeroed) {
        int rc = tango_zero2_u32_async(reinterpret_cast<uint32_t *>(stats), 6 * nh,
                                       reinterpret_cast<uint32_t *>(also_zero), 2 * nh, st);
        if (rc != TANGO_OK) return rc;
    }
    if (g->n_edges > 0) {
        sddmm_dot_args a;
        a.n = g->n_nodes;
        a.nnz = g->n_edges;
        a.ptr = g->in_ptr;
        a.idx = g->in_src;
        a.Xdst = dOut_q;  // resident row: the destination's upstream gradient
        a.Xsrc = X_q;     // gathered: the source node's features
        a.s_dst = s_dOut;
        a.s_src = s_X;
        a.out = nullptr;
        a.heads = heads;
        a.dim = dim;
        a.F = heads * dim;
        a.Sq = Sq; a.Dq = Dq; a.sS = sS; a.sD = sD; a.slope = slope;
        a.rec = nullptr; a.dS_acc = nullptr;
        a.row_lse = row_lse; a.stats = stats; a.src_codes = src_codes;
        a.chunk_shift = dot_chunk_shift(a.nnz);
        const int64_t chunks = (a.nnz + (int64_t(1) << a.chunk_shift) - 1) >> a.chunk_shift;
        const unsigned blocks = static_cast<unsigned>((chunks + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
        switch (pick_vec(a.F, dim, true)) {
            case 4: k_sddmm_dot<4, DOT_DST><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a); break;
            case 8: k_sddmm_dot<8, DOT_DST><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a); break;
            default:
            if (a.dim == 64) k_sddmm_dot<16, DOT_DST, false, 4><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
            else if (a.dim == 128) k_sddmm_dot<16, DOT_DST, false, 8><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
            else k_sddmm_dot<16, DOT_DST><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
            break;
        }
        TANGO_LAUNCH_CHECK();
    }
    k_attn_dst_finish<<<tango_grid_for(static_cast<size_t>(nh), 256), 256, 0, st>>>(nh, heads, stats, row_lse, Dq, rec, dD);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

// dS[u][h] = sum over out-edges (u -> v) of alpha*(dalpha - P[v][h])*lrelu'(t) with dalpha recomputed as the
// quantized dot product of dOut_q[v] and X_q[u]; dS_acc: n x heads doubles of scratch.
int tango_attn_bwd_src_async(const tango_graph *g, int heads, int dim, const int8_t *dOut_q, const float *s_dOut,
                             const int8_t *X_q, const float *s_X, const int8_t *Sq, const float *sS, const int8_t *Dq,
                             const float *sD, float slope, const void *rec, double *dS_acc, float *dS,
                             hipStream_t st)
{
    const int64_t nh = static_cast<int64_t>(g->n_nodes) * heads;
    int rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(dS_acc), 0u, 2 * nh, st);
    if (rc != TANGO_OK) return rc;
    if (g->n_edges > 0) {
        sddmm_dot_args a;
        a.n = g->n_nodes;
        a.nnz = g->n_edges;
        a.ptr = g->out_ptr;
        a.idx = g->out_dst;
        a.Xdst = X_q;     // resident row: the source node's features
        a.Xsrc = dOut_q;  // gathered: the destination's upstream gradient
        a.s_dst = s_dOut;
        a.s_src = s_X;
        a.out = nullptr;
        a.heads = heads;
        a.dim = dim;
        a.F = heads * dim;
        a.Sq = Sq; a.Dq = Dq; a.sS = sS; a.sD = sD; a.slope = slope;
        a.rec = rec; a.dS_acc = dS_acc;
        a.chunk_shift = dot_chunk_shift(a.nnz);
        const int64_t chunks = (a.nnz + (int64_t(1) << a.chunk_shift) - 1) >> a.chunk_shift;
        const unsigned blocks = static_cast<unsigned>((chunks + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
        switch (pick_vec(a.F, dim, true)) {
            case 4: k_sddmm_dot<4, DOT_SRC><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a); break;
            case 8: k_sddmm_dot<8, DOT_SRC><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a); break;
            default:
            if (a.dim == 64) k_sddmm_dot<16, DOT_SRC, false, 4><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
            else if (a.dim == 128) k_sddmm_dot<16, DOT_SRC, false, 8><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
            else k_sddmm_dot<16, DOT_SRC><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a);
            break;
        }
        TANGO_LAUNCH_CHECK();
    }
    k_f64_to_f32<<<tango_grid_for(static_cast<size_t>(nh), 256), 256, 0, st>>>(dS_acc, nh, dS);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_validate_sddmm_dot_shape(int heads, int dim)
{
    int rc = validate_feature_shape(heads, dim);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(pick_vec(heads * dim, dim, true) != 0, TANGO_ERR_UNSUPPORTED);
    return TANGO_OK;
}

extern "C" {

int tango_qspmm(const tango_graph *g, int direction, int heads, int dim, const int8_t *w_q, const float *s_w,
                const int8_t *X_q, const float *s_X, float *out, float *absmax_out, void *stream)
{
    TANGO_REQUIRE(direction == TANGO_IN || direction == TANGO_OUT || direction == TANGO_OUT_SRC_ORDER, TANGO_ERR_BAD_ENUM);
    int rc = validate_graph_dir(g, direction);
    if (rc != TANGO_OK) return rc;
    rc = validate_feature_shape(heads, dim);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(X_q && s_w && s_X && out && (g->n_edges == 0 || w_q), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(out, 16) && tango_aligned(X_q, 16), TANGO_ERR_BAD_SHAPE);
    return tango_spmm_async(g, direction, heads, dim, w_q, s_w, X_q, s_X, out, absmax_out, tango_stream(stream));
}

int tango_edge_to_src_order(const tango_graph *g, int heads, const int8_t *w_q, int8_t *w_q_src, void *stream)
{
    TANGO_REQUIRE(g != nullptr, TANGO_ERR_NULL);
    TANGO_REQUIRE(g->n_edges >= 0 && g->n_edges < (int64_t(1) << 31) && heads >= 1 && heads <= 8, TANGO_ERR_BAD_SHAPE);
    if (g->n_edges == 0) return TANGO_OK;
    TANGO_REQUIRE(g->out_eid && w_q && w_q_src, TANGO_ERR_NULL);
    k_edge_to_src_order<<<tango_grid_for(static_cast<size_t>(g->n_edges), 256), 256, 0, tango_stream(stream)>>>(
        g->n_edges, heads, g->out_eid, w_q, w_q_src);
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_qspmm_i4(const tango_graph *g, int direction, int heads, int dim, const int8_t *w_q, const float *s_w,
                   const uint8_t *X_q4, const float *s_X, float *out, float *absmax_out, void *stream)
{
    TANGO_REQUIRE(direction == TANGO_IN || direction == TANGO_OUT, TANGO_ERR_BAD_ENUM);
    int rc = validate_graph_dir(g, direction);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(heads >= 1 && heads <= 8 && dim >= 8 && dim % 8 == 0 && static_cast<int64_t>(heads) * dim <= 1024,
                  TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(pick_vec_i4(heads * dim, dim) != 0, TANGO_ERR_UNSUPPORTED);
    TANGO_REQUIRE(X_q4 && s_w && s_X && out && (g->n_edges == 0 || w_q), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(out, 16) && tango_aligned(X_q4, 16), TANGO_ERR_BAD_SHAPE);
    return spmm_launch(g, direction, heads, dim, w_q, s_w, reinterpret_cast<const int8_t *>(X_q4), s_X, out, absmax_out,
                       nullptr, tango_stream(stream), true);
}

int tango_qsddmm_dot_i4(const tango_graph *g, int heads, int dim, const uint8_t *X_src4, const float *s_src,
                        const uint8_t *X_dst4, const float *s_dst, float *E, void *stream)
{
    int rc = validate_graph_dir(g, TANGO_IN);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(heads >= 1 && heads <= 8 && dim >= 8 && dim % 8 == 0 && static_cast<int64_t>(heads) * dim <= 2048,
                  TANGO_ERR_BAD_SHAPE);
    const int vec = pick_vec(heads * dim / 2, dim / 2, true);  // in bytes of the packed rows
    TANGO_REQUIRE(vec != 0, TANGO_ERR_UNSUPPORTED);
    TANGO_REQUIRE(X_src4 && X_dst4 && s_src && s_dst && (g->n_edges == 0 || E), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(X_src4, 16) && tango_aligned(X_dst4, 16), TANGO_ERR_BAD_SHAPE);
    if (g->n_edges == 0) return TANGO_OK;
    hipStream_t st = tango_stream(stream);
    sddmm_dot_args a;
    a.n = g->n_nodes;
    a.nnz = g->n_edges;
    a.ptr = g->in_ptr;
    a.idx = g->in_src;
    a.Xdst = reinterpret_cast<const int8_t *>(X_dst4);
    a.Xsrc = reinterpret_cast<const int8_t *>(X_src4);
    a.s_dst = s_dst;
    a.s_src = s_src;
    a.out = E;
    a.heads = heads;
    a.dim = dim / 2;
    a.F = heads * dim / 2;
    a.chunk_shift = dot_chunk_shift(a.nnz);
        const int64_t chunks = (a.nnz + (int64_t(1) << a.chunk_shift) - 1) >> a.chunk_shift;
    const unsigned blocks = static_cast<unsigned>((chunks + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
    switch (vec) {
        case 4: k_sddmm_dot<4, DOT_STORE, true><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a); break;
        case 8: k_sddmm_dot<8, DOT_STORE, true><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a); break;
        default: k_sddmm_dot<16, DOT_STORE, true><<<blocks, 64 * WAVES_PER_BLOCK, 0, st>>>(a); break;
    }
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_qspmm_bwd(const tango_graph *g, int heads, int dim, const int8_t *w_q, const float *s_w, const int8_t *X_q,
                    const float *s_X, const int8_t *dOut_q, const float *s_dOut, float *dX, float *absmax_dX, float *dW,
                    void *stream)
{
    int rc = validate_graph_dir(g, TANGO_IN);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(dOut_q && s_dOut, TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(dOut_q, 16), TANGO_ERR_BAD_SHAPE);
    hipStream_t st = tango_stream(stream);
    if (dX) {
        rc = validate_graph_dir(g, TANGO_OUT);
        if (rc != TANGO_OK) return rc;
        rc = validate_feature_shape(heads, dim);
        if (rc != TANGO_OK) return rc;
        TANGO_REQUIRE(s_w && (g->n_edges == 0 || w_q), TANGO_ERR_NULL);
        TANGO_REQUIRE(tango_aligned(dX, 16), TANGO_ERR_BAD_SHAPE);
    }
    if (dW) {
        rc = tango_validate_sddmm_dot_shape(heads, dim);
        if (rc != TANGO_OK) return rc;
        TANGO_REQUIRE(X_q && s_X, TANGO_ERR_NULL);
        TANGO_REQUIRE(tango_aligned(X_q, 16), TANGO_ERR_BAD_SHAPE);
    }
    if (dX) {
        rc = tango_spmm_async(g, TANGO_OUT, heads, dim, w_q, s_w, dOut_q, s_dOut, dX, absmax_dX, st);
        if (rc != TANGO_OK) return rc;
    }
    if (dW) {
        rc = tango_sddmm_dot_async(g, heads, dim, dOut_q, s_dOut, X_q, s_X, dW, st);
        if (rc != TANGO_OK) return rc;
    }
    return TANGO_OK;
}

}  // extern "C"
