// Cross-file internal entry points (not exported through the C ABI).
#pragma once

#include "common.hip.h"

// p[0..n) = v on the stream (a kernel, so it is safe inside captured graphs).
int tango_fill_u32_async(uint32_t *p, uint32_t v, int n, hipStream_t st);

// *out = max(*out, max|x|) with *out holding the bits of a non-negative float.
int tango_absmax_accumulate_async(const float *x, size_t n, float *out, hipStream_t st);

// Quantize with a known abs-max (device float).
int tango_quantize_with_absmax_async(const float *x, size_t n, int rounding, uint64_t seed, uint64_t stream_id,
                                     const float *absmax, int8_t *q, float *scale_out, hipStream_t st);
