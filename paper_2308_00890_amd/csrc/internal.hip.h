// Cross-file internal entry points (not exported through the C ABI).
#pragma once

#include "common.hip.h"

// p[0..n) = v on the stream (a kernel, so it is safe inside captured graphs).
int tango_fill_u32_async(uint32_t *p, uint32_t v, int64_t n, hipStream_t st);

// p1[0..n1) = 0 and p2[0..n2) = 0 in one launch (either pointer may be NULL, its count is then ignored).
int tango_zero2_u32_async(uint32_t *p1, int64_t n1, uint32_t *p2, int64_t n2, hipStream_t st);

// Every run of z cleared in one launch.
int tango_zero_regions_async(const tango_zero_regions &z, hipStream_t st);

// Two tensors quantized (abs-max values known, device) in one launch; same results as two tango_quantize calls.
int tango_quantize_pair_with_absmax_async(const float *x1, size_t n1, uint64_t stream_id1, const float *absmax1, int8_t *q1,
                                          float *scale1, const float *x2, size_t n2, uint64_t stream_id2, const float *absmax2,
                                          int8_t *q2, float *scale2, int rounding, uint64_t seed, hipStream_t st);

// *out = max(*out, max|x|) with *out holding the bits of a non-negative float.
int tango_absmax_accumulate_async(const float *x, size_t n, float *out, hipStream_t st);

// q = quantize(x where mask > 0, else 0) with the abs-max of that masked tensor (found into absmax_ws[0], device);
// x and mask 16-byte aligned, q 8-byte aligned.
int tango_quantize_masked_async(const float *x, const float *mask, size_t n, int rounding, uint64_t seed, uint64_t stream_id,
                                int8_t *q, float *scale_out, float *absmax_ws, hipStream_t st);

// The same with the ReLU's sign bits (bit i of mask_bits set where output i is positive); n a multiple of 8.
int tango_quantize_bitmasked_async(const float *x, const uint8_t *mask_bits, size_t n, int rounding, uint64_t seed,
                                   uint64_t stream_id, int8_t *q, float *scale_out, float *absmax_ws, hipStream_t st);

// tango_head_proj and the quantization of X (abs-max known: absmax_X, device) in one pass over X; X 16-byte and X_q
// 8-byte aligned; only where tango_head_proj_quantize_supported.  The results are those of the two separate calls.
bool tango_head_proj_quantize_supported(int heads, int dim);
int tango_head_proj_quantize_async(int64_t n, int heads, int dim, const float *X, const float *a_src, const float *a_dst,
                                   float *S, float *D, float *absmax_S, float *absmax_D, const float *absmax_X, int rounding,
                                   uint64_t seed, uint64_t stream_id, int8_t *X_q, float *s_X, hipStream_t st,
                                   bool absmax_zeroed = false);  // true: *absmax_S and *absmax_D were cleared by an earlier launch

// Step 2' (tango_head_proj_bwd without its argument checks).  zeroed: the runs that tango_head_proj_bwd_zero_regions names
// were cleared by an earlier launch of the same chain.
int tango_head_proj_bwd_async(int64_t n, int heads, int dim, const float *dS, const float *dD, const float *a_src,
                              const float *a_dst, const int8_t *X_q, const float *s_X, const float *dX_agg, float *dX,
                              float *absmax_dX, float *da_src, float *da_dst, void *ws, hipStream_t st, bool zeroed = false,
                              tango_colsum_job *deferred = nullptr);  // non-NULL: the final column sums are left to the caller's next launch
void tango_head_proj_bwd_zero_regions(int heads, int dim, void *ws, float *absmax_dX, tango_zero_regions &z);

// tango_qgemm_bwd with a ReLU' on dA's way out: dA_keep_bits (optional; bit i of the flat M x K tensor, 4-byte aligned,
// K a multiple of 32 and at most 2048) clear -> dA[i] = 0; absmax_dA (optional, device) receives max|dA| as written.
int tango_qgemm_bwd_masked(int64_t M, int64_t N, int64_t K, const int8_t *A_q, const float *s_A, const int8_t *B_q,
                           const float *s_B, const float *dC, int rounding, uint64_t seed, uint64_t stream_id_dC,
                           const float *absmax_dC_in, int8_t *dC_q, float *s_dC, float *dA, const uint32_t *dA_keep_bits,
                           float *absmax_dA, float *dB, void *ws, size_t ws_bytes, void *stream,
                           const tango_colsum_job *tail = nullptr);  // done by the call's first launch (only with dA and N <= 2048)

// tango_qgemm with max|A| already on the device (absmax_A_in, may be NULL).
int tango_qgemm_known_absmax(int64_t M, int64_t N, int64_t K, const float *A, const float *absmax_A_in, const float *B,
                             int rounding, uint64_t seed, uint64_t stream_id_A, uint64_t stream_id_B, int8_t *A_q, float *s_A,
                             int8_t *B_q, float *s_B, float *C, float *absmax_C, void *ws, size_t ws_bytes, void *stream,
                             const tango_zero_regions *also_zero = nullptr);  // cleared by the call's first launch

// Whether the forward attention SPMM can write its ReLU's sign bits for this shape (rows wider than 128 columns).
bool tango_spmm_relu_bits_supported(int64_t n_nodes, int heads, int dim);

// tango_gat_attention_fwd with an optional ReLU on the aggregate (relu_out != 0: out = max(0, .), absmax_out of that);
// relu_bits (optional, 8-byte aligned, n*heads*dim/8 bytes, only where tango_spmm_relu_bits_supported): bit i of the flat
// output set where out[i] > 0.  src_codes (optional, 8-byte aligned, n_edges*heads bytes): receives S_q[src(e)] of every
// in-edge in edge order; the aggregation pass and tango_gat_attention_bwd_cached read it instead of gathering from S_q.
int tango_gat_attention_fwd_act(const tango_graph *g, int heads, int dim, const int8_t *S_q, const float *s_S,
                                const int8_t *D_q, const float *s_D, float slope, const int8_t *X_q, const float *s_X,
                                int rounding, uint64_t seed, uint64_t stream_id_alpha, float *row_lse, int8_t *alpha_q,
                                float *s_alpha, float *absmax_alpha, float *alpha_dump, float *out, float *absmax_out,
                                int relu_out, void *relu_bits, int8_t *src_codes, void *ws, size_t ws_bytes, void *stream,
                                bool absmax_alpha_zeroed = false,  // true: *absmax_alpha was cleared by an earlier launch
                                bool out_prezeroed = false);  // true: so were all of out, relu_bits and *absmax_out

// tango_gat_attention_bwd with the edge-ordered source codes the forward pass left (src_codes, may be NULL).
int tango_gat_attention_bwd_cached(const tango_graph *g, int heads, int dim, const int8_t *S_q, const float *s_S,
                                   const int8_t *D_q, const float *s_D, float slope, const float *row_lse,
                                   const int8_t *alpha_q, const float *s_alpha, const float *absmax_alpha, int rounding,
                                   uint64_t seed, uint64_t stream_id_alpha, const int8_t *X_q, const float *s_X,
                                   const int8_t *dOut_q, const float *s_dOut, float *dX_agg, float *absmax_dX, float *dalpha,
                                   float *dS, float *dD, const int8_t *src_codes, void *ws, size_t ws_bytes, void *stream,
                                   bool prezeroed = false, bool out_prezeroed = false);  // out_prezeroed: all of dX_agg is zero already
// The runs of the workspace that the call above clears first when it keeps no edge tensor (alpha_q and dalpha NULL);
// a caller that clears them in an earlier launch of the same chain passes prezeroed = true.
void tango_gat_attention_bwd_zero_regions(const tango_graph *g, int heads, void *ws, tango_zero_regions &z);

// Quantize with a known abs-max (device float).
// (absmax_count > 1: `absmax` holds that many partial maxima, see tango_absmax_partials_async; x, q vector-aligned then)
int tango_quantize_with_absmax_async(const float *x, size_t n, int rounding, uint64_t seed, uint64_t stream_id,
                                     const float *absmax, int8_t *q, float *scale_out, hipStream_t st, int absmax_count = 1);

// For a small tensor: per-workgroup maxima of |x| into partials[0 .. *count) (x 16-byte aligned, *count <= 64) and the
// runs of z cleared, in one launch: an abs-max without atomics, hence without a launch that clears their target first.
int tango_absmax_partials_async(const float *x, size_t n, float *partials, int *count, const tango_zero_regions &z, hipStream_t st);
