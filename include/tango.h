/*
 * tango.h -- C ABI of the quantization-aware GNN-layer primitives for AMD
 * MI355X (gfx950).  Method: "Tango: rethinking quantization for graph neural
 * network training on GPUs" (SC'23).  Section / equation / figure numbers
 * below refer to that paper.
 *
 * Conventions (all entry points)
 *  - Every function returns TANGO_OK (0) or a negative tango_status.  Arguments
 *    are validated on the host before anything is launched; on error nothing
 *    is launched and no output is touched.
 *  - Unless marked "host", every pointer is a DEVICE pointer owned by the
 *    caller.  The library allocates nothing, keeps no state between calls and
 *    never synchronises: work is enqueued on `stream` (a hipStream_t passed as
 *    void*, NULL = the default stream) and outputs are valid once the stream
 *    reaches that point.
 *  - Scales and abs-max values live in device memory (one float each) so that
 *    chained calls need no host round trip.  A tensor X with scale s_X
 *    represents s_X * X_q (symmetric, per tensor, zero point 0; Sec. 2.3).
 *  - Dense tensors are row-major and contiguous.  Node-feature rows hold
 *    `heads` blocks of `dim` values, F = heads*dim (Sec. 2.1 step 1).  Edge
 *    tensors hold `heads` values per edge and are indexed by the edge's
 *    position in destination-major order (see tango_graph).
 *  - Indices are int32, n_edges < 2^31; element offsets are formed in 64 bit.
 *  - Floating-point inputs must be finite (the paper's quantizer is defined on
 *    finite tensors only).  A NaN never wins an abs-max and is cast to code 0,
 *    an infinity makes the scale infinite and every code 0: neither is
 *    reported, so a caller that wants divergence to surface checks its loss or
 *    its tensors before handing them over.
 *  - `ws`/`ws_bytes`: caller-provided scratch, at least the value returned by
 *    the matching *_workspace_bytes() query, 256-byte aligned.  Its contents
 *    on entry do not matter and are undefined on return.
 *  - `rounding`: TANGO_RN (nearest, ties to even) or TANGO_SR (stochastic
 *    rounding, Eq. 3).  (seed, stream_id) name the random stream of one
 *    tensor: element i of the tensor (row-major flat index) uses 16 bits of
 *    Philox4x32-10(key = seed, counter = (i/8, stream_id)): 32-bit word
 *    (i%8)/2, low half if i is even, high half if odd.  Results therefore do
 *    not depend on launch geometry.
 */
#ifndef TANGO_H
#define TANGO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum tango_status {
    TANGO_OK = 0,
    TANGO_ERR_NULL = -1,          /* a required pointer is NULL */
    TANGO_ERR_BAD_SHAPE = -2,     /* negative / zero / too large / unsupported size or alignment */
    TANGO_ERR_BAD_ENUM = -3,      /* unknown rounding, op or direction */
    TANGO_ERR_UNSUPPORTED = -4,   /* valid but not implemented shape */
    TANGO_ERR_WORKSPACE = -5,     /* ws is NULL, misaligned or too small */
    TANGO_ERR_LAUNCH = -6         /* the HIP runtime refused a launch */
} tango_status;

enum { TANGO_RN = 0, TANGO_SR = 1 };
enum { TANGO_SDDMM_ADD_LEAKYRELU = 0, TANGO_SDDMM_DOT = 1 };
enum { TANGO_IN = 0, TANGO_OUT = 1, TANGO_OUT_SRC_ORDER = 2 };

/*
 * Graph G (Sec. 1: node features H, edge features E, graph G), both
 * directions.  Destination-major (CSC): the in-edges of node v are positions
 * in_ptr[v] .. in_ptr[v+1]-1 and in_src[e] is the source of edge e; edge
 * tensors are indexed by this position e.  Storing edges of one destination
 * adjacently is what the paper's incidence-matrix formulation buys (Sec. 3.3,
 * Fig. 5).  Source-major (CSR): out-edges of u are out_ptr[u] .. out_ptr[u+1]-1
 * with destinations out_dst[j]; out_eid[j] is that edge's destination-major
 * position.  All arrays are device memory, int32.  The out_* arrays are only
 * needed by the backward entry points and may be NULL for forward-only use.
 */
typedef struct tango_graph {
    int32_t n_nodes;
    int64_t n_edges;
    const int32_t *in_ptr;   /* n_nodes + 1 */
    const int32_t *in_src;   /* n_edges */
    const int32_t *out_ptr;  /* n_nodes + 1 */
    const int32_t *out_dst;  /* n_edges */
    const int32_t *out_eid;  /* n_edges */
} tango_graph;

/* Library version (major*10000 + minor*100 + patch) and a static, host string for a status. */
int tango_version(void);
const char *tango_status_string(int status);

/* ------------------------------------------------------------------------ */
/* Quantization (Sec. 2.3 Eq. 1-2 with Z = 0; Sec. 3.2 Eq. 3; Sec. 3.3       */
/* "Quantization overhead": one abs-max reduction, then multiply + cast).    */
/* ------------------------------------------------------------------------ */

/*
 * absmax_out[0] = max_i |x[i]| (0 for n == 0).  x: n floats.
 */
int tango_absmax(const float *x, size_t n, float *absmax_out, void *stream);

/*
 * q[i] = clamp(round(x[i] * inv), -127, 127), inv = 127/absmax (0 if absmax
 * is 0); scale_out[0] = absmax/127 (1 if absmax is 0).
 * absmax_in: device float holding max|x| if the producer of x already
 * computed it (the fused scale computation of Sec. 3.2); NULL = reduce here
 * (needs ws).  x and q must not overlap.
 */
size_t tango_quantize_workspace_bytes(size_t n);
int tango_quantize(const float *x, size_t n, int rounding, uint64_t seed, uint64_t stream_id,
                   const float *absmax_in, int8_t *q, float *scale_out, void *ws, size_t ws_bytes,
                   void *stream);

/*
 * tango_quantize with stochastic rounding whose bits come from xoshiro256++
 * generators held in registers (Sec. 3.2 "GPU-accelerated stochastic
 * rounding") instead of the counter-based generator.  The result is defined
 * by a fixed mapping, not by the launch: 65,536 generators; generator g is
 * seeded with four splitmix64 outputs from
 * x0 = seed + stream_id*0xD1342543DE82EF95 + g*0x9E3779B97F4A7C15, and its
 * j-th 64-bit output serves elements 4v..4v+3 (16 bits each, lowest first)
 * of group v = j*65536 + g.  x 16-byte, q 4-byte aligned; other arguments
 * as in tango_quantize.  For the comparison of the two sources; the layer
 * entry points use the counter-based one.
 */
int tango_quantize_xoshiro(const float *x, size_t n, uint64_t seed, uint64_t stream_id,
                           const float *absmax_in, int8_t *q, float *scale_out, void *ws,
                           size_t ws_bytes, void *stream);

/* x[i] = scale[0] * q[i]  (Eq. 2). */
int tango_dequantize(const int8_t *q, size_t n, const float *scale, float *x, void *stream);

/*
 * Quantization of a gradient that arrives behind a ReLU (Sec. 3.3 caching rule applied to the activation: the
 * gradient is quantized once, and ReLU' is folded into that pass): q = quantize(x[i] if y[i] > 0 else 0), per-tensor
 * scale from the abs-max of the masked tensor, rounding and random stream as in tango_quantize.  x, y: n floats,
 * 16-byte aligned; q: n bytes, 8-byte aligned; ws: 256 bytes, 256-byte aligned (device).
 */
int tango_quantize_relu_bwd(const float *x, const float *y, size_t n, int rounding, uint64_t seed, uint64_t stream_id,
                            int8_t *q, float *scale_out, void *ws, size_t ws_bytes, void *stream);

/*
 * Quantization-error metric and bit-count rule (Sec. 3.2 Eq. 4): for each candidate bit count B (2..8, at most 4
 * candidates, host array) error_out[c] = mean_i |(x_i - xq_i) / (x_i + xq_i + 0.0005)| (device doubles), xq the grid
 * point of the B-bit symmetric per-tensor quantizer (codes in +-(2^(B-1)-1), scale absmax/(2^(B-1)-1), rounding and
 * random stream as in tango_quantize).  bits_out (device int, may be NULL) receives the first candidate whose
 * error is below `threshold` (the paper uses 0.3 on the first layer's output in the first epoch), else the last
 * candidate.  absmax_in as in tango_quantize.  ws: tango_error_x_workspace_bytes() bytes.
 */
size_t tango_error_x_workspace_bytes(void);
int tango_error_x(const float *x, size_t n, const int *candidate_bits /* host */, int n_candidates, float threshold,
                  int rounding, uint64_t seed, uint64_t stream_id, const float *absmax_in, double *error_out,
                  int *bits_out, void *ws, size_t ws_bytes, void *stream);

/*
 * Activation between stacked layers (the paper's models are 2-3 layers deep, Sec. 4.1; it does not name the
 * activation, ReLU is used): y = max(x, 0), absmax_y (may be NULL) = max y; dx = x > 0 ? dy : 0.
 * y may alias x; dx may alias dy.
 */
int tango_relu(const float *x, size_t n, float *y, float *absmax_y, void *stream);
int tango_relu_bwd(const float *x, const float *dy, size_t n, float *dx, void *stream);

/* ------------------------------------------------------------------------ */
/* Quantized GEMM (Sec. 3.2 Fig. 3; Sec. 3.3 "GEMM with on-the-fly           */
/* quantization", Fig. 4).                                                    */
/* ------------------------------------------------------------------------ */

/*
 * C (M x N, fp32) = dequantize(A_q . B_q), A (M x K) and B (K x N) fp32.
 * Both operands are quantized inside the call; their int8 copies A_q (M x K),
 * B_q (K x N) and scales s_A, s_B are written out for the backward pass
 * (the cache of Sec. 3.3 "Inter-primitive optimization").  Accumulation is
 * int32; C = (float)acc * (s_A*s_B); absmax_C[0] = max|C| (the scale
 * computation fused into the GEMM, Sec. 3.2).  absmax_C may be NULL.
 * A must be 16-byte aligned.  K <= 2048 runs the quantize-on-load kernel; a
 * longer reduction needs K % 16 == 0 (else TANGO_ERR_UNSUPPORTED) and runs
 * as a quantization pass followed by the tiled kernel of tango_qgemm_i8.
 */
size_t tango_qgemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
int tango_qgemm(int64_t M, int64_t N, int64_t K, const float *A, const float *B, int rounding,
                uint64_t seed, uint64_t stream_id_A, uint64_t stream_id_B, int8_t *A_q, float *s_A,
                int8_t *B_q, float *s_B, float *C, float *absmax_C, void *ws, size_t ws_bytes,
                void *stream);

/*
 * tango_qgemm for callers that cannot allocate device memory and have no
 * workspace to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and same
 * results as tango_qgemm, bit for bit, without `ws`: the scratch (two abs-max
 * words and the zero-padded transposed int8 copy of B) is a fixed device array
 * inside the library, TANGO_QGEMM_STATIC_SCRATCH_BYTES = 256 B + 2 MiB per GPU
 * the library is used on, held until the process ends.  Shapes whose
 * scratch does not fit -- round_up(N, 64) * round_up(K, 32) > 2 MiB, e.g.
 * N = 1024 with K > 2048 -- are refused with TANGO_ERR_WORKSPACE before anything
 * is launched.  Neither this call nor anything it calls allocates or frees.
 * The array's device address is looked up on the first call on each device
 * (that one call must not be made under stream capture).  All calls on one GPU
 * share the array: calls that may overlap in time on one GPU (different
 * streams, different host threads) race on it and must be serialised by the
 * caller; calls on one stream are ordered and safe.
 */
#define TANGO_QGEMM_STATIC_SCRATCH_BYTES ((size_t)256 + ((size_t)2 << 20))
int tango_qgemm_static(int64_t M, int64_t N, int64_t K, const float *A, const float *B, int rounding,
                       uint64_t seed, uint64_t stream_id_A, uint64_t stream_id_B, int8_t *A_q, float *s_A,
                       int8_t *B_q, float *s_B, float *C, float *absmax_C, void *stream);

/*
 * Backward of C = A.B from the cached quantized operands (Sec. 3.3): dC
 * (M x N, fp32) is quantized once (stream_id_dC; absmax_dC_in as in
 * tango_quantize) into dC_q / s_dC (outputs, kept by the caller), then
 *   dA (M x K) = (float)(dC_q . B_q^T) * (s_dC*s_B)
 *   dB (K x N) = (float)(A_q^T . dC_q) * (s_A*s_dC)      (Sec. 3.2: fp32
 * gradients for the full-precision weight update).  dA or dB may be NULL to
 * skip that product.  dA with N > 2048 needs N % 16 == 0.
 * dB is a reduction over all M rows: slabs of at most 2^17 rows are summed in
 * int32 (exact: 2^17 * 127^2 < 2^31) and the slabs are combined in 64-bit
 * integers, so dB is the exact integer product for any M (for sums that fit
 * int32 -- every case the paper's 32-bit accumulator covers, Sec. 3.2 -- the
 * result is the same bit for bit).
 */
size_t tango_qgemm_bwd_workspace_bytes(int64_t M, int64_t N, int64_t K);
int tango_qgemm_bwd(int64_t M, int64_t N, int64_t K, const int8_t *A_q, const float *s_A,
                    const int8_t *B_q, const float *s_B, const float *dC, int rounding, uint64_t seed,
                    uint64_t stream_id_dC, const float *absmax_dC_in, int8_t *dC_q, float *s_dC,
                    float *dA, float *dB, void *ws, size_t ws_bytes, void *stream);

/*
 * The quantized product alone (Sec. 3.2 Fig. 3: int8 operands, int32
 * accumulation, one fp32 factor), for operands that are already int8 and
 * for shapes wide enough that the matrix cores, not HBM, are the bound:
 *   C[m][n] (M x N, fp32) = (float)(sum_k A_q[m][k] * BT_q[n][k]) * (s_A*s_B)
 * A_q: M x K, BT_q: N x K (the right operand transposed), both row-major
 * with K contiguous, device, 16-byte aligned; K % 16 == 0 (else
 * TANGO_ERR_UNSUPPORTED); K <= 2^17 keeps the int32 accumulator exact.
 * absmax_C (may be NULL) = max|C|.  No workspace.
 */
int tango_qgemm_i8(int64_t M, int64_t N, int64_t K, const int8_t *A_q, const float *s_A,
                   const int8_t *BT_q, const float *s_B, float *C, float *absmax_C, void *stream);

/* ------------------------------------------------------------------------ */
/* Attention projections (Sec. 2.1 step 2 and 2'), fp32.                      */
/* ------------------------------------------------------------------------ */

/*
 * S[v][h] = sum_d X[v][h][d]*a_src[h][d], D likewise with a_dst.
 * X: n x (heads*dim); a_src, a_dst: heads x dim; S, D: n x heads.
 * absmax_S / absmax_D (may be NULL) receive max|S|, max|D|.
 */
int tango_head_proj(int64_t n, int heads, int dim, const float *X, const float *a_src,
                    const float *a_dst, float *S, float *D, float *absmax_S, float *absmax_D,
                    void *stream);

/*
 * Step 2' fused with the gradient sum that feeds step 1':
 *   dX[v][h][d]  = dX_agg[v][h][d] + (dS[v][h]*a_src[h][d] + dD[v][h]*a_dst[h][d])
 *   da_src[h][d] = sum_v dS[v][h] * (s_X * X_q[v][h][d]),   da_dst likewise with dD
 * X_q/s_X: the cached quantized H' (n x F int8).  dX may alias dX_agg.
 * absmax_dX (may be NULL) receives max|dX|.
 */
size_t tango_head_proj_bwd_workspace_bytes(int64_t n, int heads, int dim);
int tango_head_proj_bwd(int64_t n, int heads, int dim, const float *dS, const float *dD,
                        const float *a_src, const float *a_dst, const int8_t *X_q, const float *s_X,
                        const float *dX_agg, float *dX, float *absmax_dX, float *da_src,
                        float *da_dst, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------ */
/* Quantized SDDMM (Sec. 2.1 steps 3 and 5''; Sec. 3.3 "SDDMM with            */
/* on-the-fly dequantization").                                               */
/* ------------------------------------------------------------------------ */

/*
 * op = TANGO_SDDMM_ADD_LEAKYRELU: dim must be 1; X_src, X_dst are n x heads
 *   int8 (S_q, D_q);  E[e][h] = lrelu(s_src*X_src[src(e)][h] + s_dst*X_dst[dst(e)][h]).
 * op = TANGO_SDDMM_DOT: X_src, X_dst are n x (heads*dim) int8;
 *   E[e][h] = (float)(sum_d X_dst[dst(e)][h][d]*X_src[src(e)][h][d]) * (s_dst*s_src);
 *   `slope` ignored; dim must be a multiple of 4.
 * E: n_edges x heads fp32.  Uses g->in_ptr, g->in_src.
 */
int tango_qsddmm(const tango_graph *g, int op, int heads, int dim, const int8_t *X_src,
                 const float *s_src, const int8_t *X_dst, const float *s_dst, float slope, float *E,
                 void *stream);

/*
 * Backward of TANGO_SDDMM_ADD_LEAKYRELU (Sec. 2.1 steps 3', 3''; Sec. 3.3
 * "Incidence matrix-based SPMM": with destination-major edge storage dD is a
 * sum over a contiguous edge segment).  dE: gradient w.r.t. the activated
 * scores (n_edges x heads).  The LeakyReLU derivative (1 if t > 0 else slope)
 * uses t recomputed from the quantized S_q (=X_src), D_q (=X_dst).
 *   dE_pre (may be NULL) = dE * lrelu'(t)
 *   dD[v][h] = sum over in-edges of v,  dS[u][h] = sum over out-edges of u.
 * Needs g->out_ptr, g->out_eid for dS.
 * (The DOT op needs no entry point of its own: its gradients are an SPMM and
 * an SPMM on the reversed graph.)
 */
int tango_qsddmm_bwd(const tango_graph *g, int heads, const int8_t *X_src, const float *s_src,
                     const int8_t *X_dst, const float *s_dst, float slope, const float *dE,
                     float *dE_pre, float *dS, float *dD, void *stream);

/* ------------------------------------------------------------------------ */
/* Edge softmax in full precision (Sec. 2.1 steps 4 and 4'; Sec. 3.2          */
/* "Full precision for the layer before Softmax").                            */
/* ------------------------------------------------------------------------ */

/*
 * alpha[e][h] = exp(E[e][h] - m) / sum_{e' -> dst(e)} exp(E[e'][h] - m), m the
 * maximum over the same in-edges.  absmax_alpha (may be NULL) = max alpha.
 * alpha may alias E.
 */
int tango_edge_softmax(const tango_graph *g, int heads, const float *E, float *alpha,
                       float *absmax_alpha, void *stream);

/*
 * dE[e][h] = alpha[e][h] * (dalpha[e][h] - P[dst(e)][h]),
 * P[v][h] = sum_{e -> v} dalpha[e][h]*alpha[e][h].  dE may alias dalpha.
 */
int tango_edge_softmax_bwd(const tango_graph *g, int heads, const float *alpha, const float *dalpha,
                           float *dE, void *stream);

/* ------------------------------------------------------------------------ */
/* Quantized SPMM (Sec. 2.1 steps 5 and 5'; Sec. 3.3 "Incidence matrix-based  */
/* adaptive SPMM": node and edge features are both int8, only the result is  */
/* dequantized).                                                              */
/* ------------------------------------------------------------------------ */

/*
 * direction TANGO_IN : out[v][h][:] = (s_w*s_X) * sum_{e=(u->v)} w_q[e][h]*X_q[u][h][:]
 * direction TANGO_OUT: out[u][h][:] = (s_w*s_X) * sum_{e=(u->v)} w_q[e][h]*X_q[v][h][:]
 *                      (the same product on the reversed graph; needs out_*).
 * direction TANGO_OUT_SRC_ORDER: as TANGO_OUT, but w_q is indexed by the edge's
 *                      source-major position (the order of out_dst), so no weight is fetched through
 *                      out_eid (one dependent random byte read per edge less; out_eid may be NULL).
 *                      For weights that do not change between iterations (GCN normalisation, typed
 *                      layers): permute them once with tango_edge_to_src_order.
 * w_q: n_edges x heads int8 (destination-major positions for TANGO_IN and TANGO_OUT);
 * X_q: n x F int8, F = heads*dim, dim a multiple of 4 and F <= 1024;
 * out: n x F fp32, 16-byte aligned; absmax_out (may be NULL) = max|out|.
 * Accumulation is exact int32 (wrap-around beyond 2^31).
 */
int tango_qspmm(const tango_graph *g, int direction, int heads, int dim, const int8_t *w_q,
                const float *s_w, const int8_t *X_q, const float *s_X, float *out, float *absmax_out,
                void *stream);

/*
 * w_q_src[j][h] = w_q[out_eid[j]][h]: the edge codes (n_edges x heads int8) re-ordered from destination-major to
 * source-major positions, the operand of tango_qspmm(TANGO_OUT_SRC_ORDER).  A cached quantized tensor in the sense of
 * Sec. 3.3 "Inter-primitive optimization": made once per graph for fixed edge weights.  w_q and w_q_src must not overlap.
 */
int tango_edge_to_src_order(const tango_graph *g, int heads, const int8_t *w_q, int8_t *w_q_src, void *stream);

/*
 * Backward of tango_qspmm(direction = TANGO_IN) given the quantized upstream
 * gradient dOut_q (n x F int8, scale s_dOut), quantized once and shared by
 * both products (Sec. 3.3):
 *   dX (n x F fp32, may be NULL)      = SPMM on the reversed graph with w_q (step 5')
 *   dW (n_edges x heads, may be NULL) = SDDMM-dot of dOut_q[dst] with X_q[src] (step 5'')
 * absmax_dX may be NULL.
 */
int tango_qspmm_bwd(const tango_graph *g, int heads, int dim, const int8_t *w_q, const float *s_w,
                    const int8_t *X_q, const float *s_X, const int8_t *dOut_q, const float *s_dOut,
                    float *dX, float *absmax_dX, float *dW, void *stream);

/* ------------------------------------------------------------------------ */
/* Fused attention forward (allowed in addition to the primitives, never    */
/* instead of them): Sec. 2.1 steps 3, 4 and 5 with the fusions of Sec. 3.3   */
/* -- E and alpha are never written in fp32.                                  */
/* ------------------------------------------------------------------------ */

/*
 * Equivalent to  E = tango_qsddmm(ADD_LEAKYRELU); alpha = tango_edge_softmax(E);
 * alpha_q = tango_quantize(alpha); out = tango_qspmm(TANGO_IN, alpha_q, X_q)
 * up to the summation order of the softmax denominator and the last bits of exp
 * (the hardware exponential is used).  S_q and D_q must be aligned to `heads` bytes
 * when heads is 2, 4 or 8.  Outputs:
 *   row_lse (n x heads fp32): per (node, head) the logarithm of the sum of exp(E) over
 *       its in-edges, so that alpha = exp(E - row_lse); the backward pass recomputes the
 *       fp32 alpha from it;
 *   alpha_q (nnz x heads int8) or NULL: the quantized attention; s_alpha, absmax_alpha:
 *       its scale and abs-max (the backward pass can recompute the identical codes from
 *       S_q, D_q, row_lse, absmax_alpha and the random stream, so caching alpha_q is optional);
 *   alpha_dump (nnz x heads fp32) or NULL: the exact fp32 alpha values that were
 *       quantized (for verification: alpha_q must equal the quantization of this
 *       tensor bit for bit);
 *   out (n x F fp32), absmax_out (may be NULL).
 * ws: at least tango_gat_attention_workspace_bytes() bytes.
 */
size_t tango_gat_attention_workspace_bytes(int64_t n_nodes, int64_t n_edges, int heads);
int tango_gat_attention_fwd(const tango_graph *g, int heads, int dim, const int8_t *S_q,
                            const float *s_S, const int8_t *D_q, const float *s_D, float slope,
                            const int8_t *X_q, const float *s_X, int rounding, uint64_t seed,
                            uint64_t stream_id_alpha, float *row_lse, int8_t *alpha_q, float *s_alpha,
                            float *absmax_alpha, float *alpha_dump, float *out, float *absmax_out,
                            void *ws, size_t ws_bytes, void *stream);

/*
 * Backward of tango_gat_attention_fwd (Fig. 1b steps 5', 5'', 4', 3', 3'') from its caches:
 *   dX_agg (n x F fp32)     = SPMM on the reversed graph of alpha_q and dOut_q (step 5'); absmax_dX may be NULL.
 *                             alpha_q = NULL: its codes are recomputed on the fly (same rounding, seed, stream id
 *                             as the forward call), which replaces one random 4-byte read per edge by reads of
 *                             the small cache-resident S_q, D_q, row_lse tables;
 *   dalpha (nnz x heads)    = SDDMM-dot of dOut_q[dst] and X_q[src] (step 5''), fp32 scratch that is also an output.
 *                             With alpha_q = NULL it may be NULL while dS and dD are given: then no edge tensor is
 *                             written at all - one walk over the in-edges forms P and dD from three running sums
 *                             per (node, head) (dD = B - P*C with P = sum alpha*dalpha, B = sum alpha*dalpha*s,
 *                             C = sum alpha*s, s = 1 or the slope by the sign of the score; fp64), and one walk
 *                             over the out-edges forms dX_agg and dS together;
 *   dD, dS (n x heads fp32) = sums over in-/out-edges of alpha*(dalpha - P)*lrelu'(t) with the fp32 alpha
 *                             recomputed from S_q, D_q, row_lse exactly as the forward pass computed it
 *                             (the gradient of the pre-activation scores is never written to memory).
 *                             dalpha, dS and dD may all three be NULL: then only step 5' runs.
 * ws: at least tango_gat_attention_bwd_workspace_bytes() bytes.
 */
size_t tango_gat_attention_bwd_workspace_bytes(int64_t n_nodes, int64_t n_edges, int heads);
int tango_gat_attention_bwd(const tango_graph *g, int heads, int dim, const int8_t *S_q,
                            const float *s_S, const int8_t *D_q, const float *s_D, float slope,
                            const float *row_lse, const int8_t *alpha_q, const float *s_alpha,
                            const float *absmax_alpha, int rounding, uint64_t seed,
                            uint64_t stream_id_alpha, const int8_t *X_q, const float *s_X,
                            const int8_t *dOut_q, const float *s_dOut, float *dX_agg, float *absmax_dX,
                            float *dalpha, float *dS, float *dD, void *ws, size_t ws_bytes, void *stream);

/*
 * The two halves of tango_gat_attention_bwd's no-edge-tensor path as calls of their own (the whole call is their
 * composition):
 *   _dst: one walk over the in-edges of every destination v (steps 5'', 4', 3''): dD (n x heads fp32) and, in `rec`
 *         (device, tango_gat_attention_bwd_rec_bytes() bytes, 16-byte aligned; an opaque table with one record
 *         per node: row_lse and, as fp64, P of every head), what the other half needs;
 *   _src: one walk over the out-edges of every source u (steps 5' and 3'): dX_agg (n x F fp32, absmax_dX may be
 *         NULL) and dS (n x heads fp32), with the int8 attention codes recomputed as in tango_gat_attention_bwd.
 * ws: device scratch of the matching _workspace_bytes(), 256-byte aligned.  Other arguments as in
 * tango_gat_attention_bwd.
 */
size_t tango_gat_attention_bwd_rec_bytes(int64_t n_nodes, int heads);
size_t tango_gat_attention_bwd_dst_workspace_bytes(int64_t n_nodes, int heads);
size_t tango_gat_attention_bwd_src_workspace_bytes(int64_t n_nodes, int heads);
int tango_gat_attention_bwd_dst(const tango_graph *g, int heads, int dim, const int8_t *S_q, const float *s_S,
                                const int8_t *D_q, const float *s_D, float slope, const float *row_lse,
                                const int8_t *X_q, const float *s_X, const int8_t *dOut_q, const float *s_dOut,
                                void *rec, float *dD, void *ws, size_t ws_bytes, void *stream);
int tango_gat_attention_bwd_src(const tango_graph *g, int heads, int dim, const int8_t *S_q, const float *s_S,
                                const int8_t *D_q, const float *s_D, float slope, const float *row_lse,
                                const float *s_alpha, const float *absmax_alpha, int rounding, uint64_t seed,
                                uint64_t stream_id_alpha, const int8_t *X_q, const float *s_X,
                                const int8_t *dOut_q, const float *s_dOut, const void *rec, float *dX_agg,
                                float *absmax_dX, float *dS, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------ */
/* 4-bit operands (Sec. 4 "Speed impact for # of quantization bits").         */
/* ------------------------------------------------------------------------ */

/*
 * The quantizer of tango_quantize with codes in [-7, 7] (s = absmax/7,
 * inv = 7/absmax; same rounding rules, same random bits per element),
 * stored packed: byte j of q4 holds element 2j in its low nibble and 2j+1 in
 * its high nibble, each a 4-bit two's-complement number.  n even; x 16-byte,
 * q4 4-byte aligned; q4 has n/2 bytes.  absmax_in / ws as in tango_quantize.
 */
int tango_quantize_i4(const float *x, size_t n, int rounding, uint64_t seed, uint64_t stream_id,
                      const float *absmax_in, uint8_t *q4, float *scale_out, void *ws, size_t ws_bytes,
                      void *stream);

/*
 * tango_qspmm with a packed 4-bit feature table X_q4 (n x heads*dim/2 bytes,
 * layout of tango_quantize_i4 along each row); the edge weights w_q stay
 * int8.  Halves the gathered bytes per edge.  The paper measures no INT4
 * SPMM (its baselines have none); this is the same operation as steps 5 / 5'
 * on the narrower table.  dim % 8 == 0; heads*dim <= 1024; exact while every
 * |integer sum| < 2^27.  Other arguments as in tango_qspmm.
 */
int tango_qspmm_i4(const tango_graph *g, int direction, int heads, int dim, const int8_t *w_q,
                   const float *s_w, const uint8_t *X_q4, const float *s_X, float *out, float *absmax_out,
                   void *stream);

/*
 * SDDMM, dot-product case (step 5''), with both node tables packed 4-bit:
 * E[e][h] = (float)(sum_d X_dst4[dst(e)][h][d] * X_src4[src(e)][h][d]) * (s_dst*s_src),
 * E: nnz x heads fp32 in destination-major edge order.  dim % 8 == 0;
 * heads*dim <= 2048; tables 16-byte aligned.
 */
int tango_qsddmm_dot_i4(const tango_graph *g, int heads, int dim, const uint8_t *X_src4, const float *s_src,
                        const uint8_t *X_dst4, const float *s_dst, float *E, void *stream);

/* ------------------------------------------------------------------------ */
/* Full-precision twins of the two gather-bound primitives, for measuring     */
/* what quantization buys on the same graph (Sec. 3.3: the random accesses    */
/* hit a 4x smaller table).  Not part of the quantized path.                  */
/* ------------------------------------------------------------------------ */

/*
 * out (n x F fp32) = SPMM of fp32 edge weights w (nnz x heads, destination-major positions) and fp32 features
 * X (n x F); direction as in tango_qspmm.  Sums are formed in fp32 (order not fixed for rows longer than 1,024
 * edges).  F = heads*dim must be a power of two <= 256 with dim a power of two >= 4, or a multiple of 256 with
 * heads == 1.  X, out 16-byte aligned.
 */
int tango_spmm_f32(const tango_graph *g, int direction, int heads, int dim, const float *w, const float *X,
                   float *out, void *stream);

/* E[e][h] = X_dst[dst(e)][h][:] . X_src[src(e)][h][:] in fp32; shapes as above. */
int tango_sddmm_dot_f32(const tango_graph *g, int heads, int dim, const float *X_src, const float *X_dst,
                        float *E, void *stream);

/* ------------------------------------------------------------------------ */
/* Whole-layer entry points: the primitives above chained on one stream,     */
/* with every quantized tensor produced once and reused (Sec. 3.3             */
/* "Inter-primitive optimization": forward tensors cached for backward, one  */
/* quantized copy shared by several operators).  They add no arithmetic of   */
/* their own: each is checkable against the composition of the primitives.   */
/* ------------------------------------------------------------------------ */

/*
 * Buffers of one GAT layer (Fig. 1).  n = g->n_nodes, nnz = g->n_edges,
 * F = heads*dim.  All device memory, caller-owned, contiguous.  "out" fields
 * are written by the call named in brackets and read by later calls.
 * Random streams: tensor t of layer `layer_id` uses stream_id 16*layer_id + t
 * with t = 1 H, 2 W, 3 H', 4 S, 5 D, 6 alpha, 7 upstream gradient, 8 dH'.
 */
typedef struct tango_gat_layer {
    const tango_graph *g;
    int k_in, heads, dim;
    float slope;            /* LeakyReLU slope */
    int rounding;
    uint64_t seed, layer_id;
    /* parameters and input */
    const float *H;         /* n x k_in */
    const float *W;         /* k_in x F */
    const float *a_src;     /* heads x dim */
    const float *a_dst;     /* heads x dim */
    /* forward results and caches [fwd] */
    int8_t *H_q;  float *s_H;     /* n x k_in */
    int8_t *W_q;  float *s_W;     /* k_in x F */
    float *Hp;    float *absmax_Hp; /* n x F: H' = H.W dequantized */
    int8_t *Hp_q; float *s_Hp;    /* n x F */
    float *S, *D;                 /* n x heads fp32 (step 2) */
    int8_t *S_q;  float *s_S;     /* n x heads */
    int8_t *D_q;  float *s_D;     /* n x heads */
    float *E;                     /* nnz x heads: activated scores (step 3); may alias alpha */
    float *alpha;                 /* nnz x heads: softmax output, fp32 (kept for step 4') */
    int8_t *alpha_q; float *s_alpha; /* nnz x heads */
    float *out;   float *absmax_out; /* n x F: layer output H^(l) */
    /* backward input, results and scratch [bwd] */
    const float *grad_out;        /* n x F */
    int8_t *g_q;  float *s_g;     /* n x F: quantized upstream gradient */
    float *dHp;   float *absmax_dHp; /* n x F: dH' = dH'_agg + dH'_att */
    float *dalpha;                /* nnz x heads: step 5''; overwritten by step 4' (dE); with fused = 1 and
                                     alpha_q = NULL it may be NULL (nothing is stored per edge) */
    float *dS, *dD;               /* n x heads */
    int8_t *dHp_q; float *s_dHp;  /* n x F */
    float *dW;                    /* k_in x F  (fp32 gradient for the full-precision weight update) */
    float *dH;                    /* n x k_in, or NULL to skip (first layer) */
    float *da_src, *da_dst;       /* heads x dim */
    /* fused = 1: steps 3-5 and 5'-3'' run through tango_gat_attention_fwd / _bwd.  Then E is unused (may be
     * NULL), alpha is optional (if not NULL it receives the fp32 attention that was quantized, for
     * verification), alpha_q is optional (NULL: the backward pass recomputes its codes), dalpha keeps step
     * 5'' (it is not overwritten), and row_lse (n x heads) and absmax_alpha are required.
     * fused = 0: the primitives are chained one by one and row_lse / absmax_alpha are unused. */
    int fused;
    float *row_lse;
    float *absmax_alpha;
    /* scratch */
    void *ws;
    size_t ws_bytes;              /* >= tango_gat_layer_workspace_bytes(...) */
    /* Stacked layers (the paper does not say what sits between layers; a ReLU is taken).  relu_out != 0: the forward
     * pass writes out = max(0, aggregate) from the SPMM's own epilogue (absmax_out is of that), and the backward pass
     * takes grad_out as the gradient behind that ReLU: ReLU' (out > 0) is applied while grad_out is quantized, so no
     * activation kernel and no extra fp32 tensor exist between two layers; grad_out and out must then be 16-byte
     * aligned.  absmax_H: max|H| on the device if the caller already has it (the absmax_out of the layer below),
     * else NULL - it saves the pass over H that finds it.  relu_bits (optional, device, 8-byte aligned,
     * n*heads*dim/8 bytes, written by the forward pass and read by the backward pass): one bit per output element,
     * bit i%8 of byte i/8 set where out[i] > 0.  Where it is given, the layer is fused and a row is wider than 128
     * columns (heads*dim in {256, 512, 1024}, dim a multiple of 16), the backward pass reads these bits instead of the
     * fp32 `out` (1/32 of the bytes); otherwise it is ignored, in both passes alike. */
    int relu_out;
    const float *absmax_H;
    void *relu_bits;
    /* Optional cache of the fused layer (device, 8-byte aligned, n_edges*heads bytes, else NULL): the forward pass's first
     * walk over the in-edges leaves S_q[src(e)] of every edge here, in edge order, and its second walk and the backward
     * pass's walk over the in-edges read that stream instead of gathering from S_q once more per edge (Sec. 3.3's
     * caching of quantized tensors between operators, applied to a gathered tensor).  Results do not change. */
    int8_t *src_codes;
    /* Stacked layers, the ReLU' of the layer below applied where the gradient is produced (all optional, else NULL):
     * dH_keep_bits - the relu_bits of the layer below (whose ReLU output is this layer's H; k_in a multiple of 32 and at
     * most 2048): the backward pass writes dH with zeros where the bit is clear; absmax_dH (device, out) receives max|dH|
     * as written.  absmax_grad_out (device, in) - max|grad_out| if the caller has it (the absmax_dH of the layer above):
     * the pass over grad_out that finds it is skipped, and with relu_out set grad_out is then taken to carry the ReLU'
     * mask already (the layer above applied it through its dH_keep_bits). */
    const void *dH_keep_bits;
    float *absmax_dH;
    const float *absmax_grad_out;
} tango_gat_layer;

size_t tango_gat_layer_workspace_bytes(int64_t n_nodes, int64_t n_edges, int k_in, int heads, int dim);

/* Steps 1-5 of Fig. 1a: qGEMM, projections, quantize, SDDMM-add, edge softmax, quantize, qSPMM. */
int tango_gat_layer_fwd(const tango_gat_layer *L, void *stream);

/* Steps 5', 5'', 4', 3', 3'', 2', 1' of Fig. 1b, reading the caches tango_gat_layer_fwd left in *L. */
int tango_gat_layer_bwd(const tango_gat_layer *L, void *stream);

/*
 * One GCN layer (Sec. 2.2): H' = H.W (qGEMM), out = (G (.) w) . H' (qSPMM) with
 * fixed edge weights w already quantized by the caller (w_q: nnz x 1, s_w).
 * Random streams as in tango_gat_layer.
 */
typedef struct tango_gcn_layer {
    const tango_graph *g;
    int k_in, f_out;
    int rounding;
    uint64_t seed, layer_id;
    const float *H;          /* n x k_in */
    const float *W;          /* k_in x f_out */
    const int8_t *w_q; const float *s_w;  /* nnz edge weights */
    int8_t *H_q;  float *s_H;
    int8_t *W_q;  float *s_W;
    float *Hp;    float *absmax_Hp;   /* n x f_out */
    int8_t *Hp_q; float *s_Hp;
    float *out;   float *absmax_out;  /* n x f_out */
    const float *grad_out;            /* n x f_out */
    int8_t *g_q;  float *s_g;
    float *dHp;   float *absmax_dHp;  /* n x f_out */
    int8_t *dHp_q; float *s_dHp;
    float *dW;                        /* k_in x f_out */
    float *dH;                        /* n x k_in or NULL */
    void *ws;
    size_t ws_bytes;
    /* Optional (else NULL): w_q in source-major order (tango_edge_to_src_order), made once per graph; the backward
     * pass then runs its reverse SPMM as TANGO_OUT_SRC_ORDER.  Same results. */
    const int8_t *w_q_src_order;
} tango_gcn_layer;

size_t tango_gcn_layer_workspace_bytes(int64_t n_nodes, int64_t n_edges, int k_in, int f_out);
int tango_gcn_layer_fwd(const tango_gcn_layer *L, void *stream);
int tango_gcn_layer_bwd(const tango_gcn_layer *L, void *stream);

/*
 * One GEMM + SPMM layer over typed edges.  Sec. 2.2 names GraphSAGE and the
 * relational GCN as models built from these two primitives; with a type t(e)
 * in 0 .. n_types-1 and a fixed weight w(e) on every edge both are
 *     Z = H . [W_0 | W_1 | ... | W_{n_types-1}]        (one qGEMM, Z: n x n_types*f_out)
 *     out[v,:] = sum over e = (u -> v) of w(e) * Z[u, t(e)*f_out : (t(e)+1)*f_out]   (qSPMM)
 * (relational GCN: t = 0 the self-connection, t = r the r-th relation, w = 1/c_{v,r};
 * GraphSAGE with the mean aggregator: t = 0 self with w = 1, t = 1 neighbours with w = 1/degree).
 * Row-major Z is also an (n*n_types) x f_out table whose row u*n_types + t is
 * block t of node u, so the typed graph is passed as two one-directional views
 * of a bipartite graph between these table rows and the n destinations:
 *   g_dst: n_nodes = n, in_ptr[n+1], in_src[e] = u*n_types + t(e); out_* unused (may be NULL);
 *   g_src: n_nodes = n*n_types, out_ptr[n*n_types+1], out_dst[j] = destination, out_eid[j] =
 *          position of that edge in g_dst's order; in_* unused (may be NULL).
 * Both views hold the same n_edges edges.  With n_types = 1 and g_dst = g_src
 * this is tango_gcn_layer.  Buffers as in tango_gcn_layer with Hp, Hp_q, dHp,
 * dHp_q of n x n_types*f_out, W, W_q, dW of k_in x n_types*f_out and out,
 * grad_out, g_q of n x f_out.  Random streams as in tango_gat_layer.
 * Limits: f_out % 4 == 0, f_out <= 1024, n*n_types < 2^31.
 */
typedef struct tango_typed_layer {
    const tango_graph *g_dst;
    const tango_graph *g_src;         /* backward only; may be NULL for forward-only use */
    int n_types;
    int k_in, f_out;
    int rounding;
    uint64_t seed, layer_id;
    const float *H;          /* n x k_in */
    const float *W;          /* k_in x n_types*f_out */
    const int8_t *w_q; const float *s_w;  /* nnz edge weights, g_dst order */
    int8_t *H_q;  float *s_H;
    int8_t *W_q;  float *s_W;
    float *Hp;    float *absmax_Hp;   /* Z */
    int8_t *Hp_q; float *s_Hp;
    float *out;   float *absmax_out;
    const float *grad_out;
    int8_t *g_q;  float *s_g;
    float *dHp;   float *absmax_dHp;  /* dZ */
    int8_t *dHp_q; float *s_dHp;
    float *dW;
    float *dH;                        /* n x k_in or NULL */
    void *ws;
    size_t ws_bytes;                  /* >= tango_typed_layer_workspace_bytes(...) */
    const int8_t *w_q_src_order;      /* optional (else NULL): w_q in g_src's order, as in tango_gcn_layer */
} tango_typed_layer;

size_t tango_typed_layer_workspace_bytes(int64_t n_nodes, int64_t n_edges, int n_types, int k_in, int f_out);
int tango_typed_layer_fwd(const tango_typed_layer *L, void *stream);
int tango_typed_layer_bwd(const tango_typed_layer *L, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TANGO_H */
