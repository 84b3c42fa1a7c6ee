/*
 * tango_benchaid.h -- measurement aids of the benchmark harness.  NOT part of
 * the method and not part of libtango.so: they live in libtango_benchaid.so
 * and exist so that the roofline figures the harness prints can be calibrated
 * on the machine they are measured on.  Conventions as in tango.h: device
 * pointers owned by the caller, nothing allocated, nothing synchronised, work
 * enqueued on `stream`; the return value is 0 or a negative tango_status.
 */
#ifndef TANGO_BENCHAID_H
#define TANGO_BENCHAID_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Register-only matrix-core loop: launches 256 workgroups x 4 waves that each
 * issue 8*iters independent v_mfma_i32_32x32x32_i8 from registers (no LDS, no
 * memory).  random_operands != 0 fills the operand registers with
 * pseudo-random bytes (realistic switching activity; the chip then runs
 * power-limited), 0 with constant bytes.  *ops (host) receives the int8
 * operation count (2 per multiply-add) of the launch; the caller times it.
 * ws: device scratch of tango_benchaid_mfma_i8_workspace_bytes().
 */
size_t tango_benchaid_mfma_i8_workspace_bytes(void);
int tango_benchaid_mfma_i8_launch(int iters, int random_operands, void *ws, size_t ws_bytes, double *ops,
                                  void *stream);

/*
 * The same loop with the scaled 8-bit / 4-bit floating-point matrix
 * instruction of gfx950 (v_mfma_scale_f32_32x32x64_f8f6f4, unit scales):
 * format 0 = fp8 (e4m3) operands, 1 = fp4 (e2m1) operands.  *ops receives
 * 2 operations per multiply-add.
 */
int tango_benchaid_mfma_f8f6f4_launch(int iters, int format, int random_operands, void *ws, size_t ws_bytes,
                                      double *ops, void *stream);

/*
 * dst[i] = src[i] for n 16-byte words (both device, 16-byte aligned): a plain
 * streaming copy of known size, the yardstick for rocprofv3's FETCH_SIZE /
 * WRITE_SIZE counters and for the HBM rate a kernel can reach in practice.
 */
int tango_benchaid_copy(const void *src, void *dst, size_t n_words16, void *stream);

/*
 * A streaming kernel with a chosen mix of reads and writes: for every unit
 * i < n_units it loads 16 bytes from each of `reads` arrays (src holds them
 * end to end: reads * n_units * 16 bytes) and stores 16 bytes to each of
 * `writes` arrays (dst: writes * n_units * 16 bytes, at least 16).  Allowed
 * (reads, writes): (1,0) (0,1) (1,1) (2,1) (4,1) (1,2) (1,4); anything else
 * returns TANGO_ERR_BAD_ENUM.  The HBM rate this reaches at a kernel's own
 * read : write ratio is the yardstick its streaming rate is compared with.
 */
int tango_benchaid_stream_mix(const void *src, void *dst, size_t n_units, int reads, int writes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TANGO_BENCHAID_H */
