// Measurement aid, not a step of the method: the int8 matrix-core rate the chip sustains when every SIMD issues
// v_mfma_i32_32x32x32_i8 back to back from registers (no LDS, no memory).  With operand bits that toggle (random
// bytes) the chip runs power-limited well below its nominal clock, so this is the practical ceiling a GEMM main loop
// is measured against, next to the published peak.
#include "internal.hip.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void k_mfma_rate(int iters, int random_operands, int *sink)
{
    v16i acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = v16i{0};
    v4i av[4], bv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            unsigned h = (threadIdx.x * 16u + i * 4u + c + blockIdx.x * 4096u) * 2654435761u;
            h ^= h >> 15;
            h *= 2246822519u;
            h ^= h >> 13;
            unsigned g = h * 3266489917u;
            g ^= g >> 16;
            av[i][c] = random_operands ? static_cast<int>(h) : 0x01010101;
            bv[i][c] = random_operands ? static_cast<int>(g) : 0x02020202;
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av[i % 4], bv[i / 2], acc[i], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    sink[blockIdx.x * 256 + threadIdx.x] = s;  // keeps the loop alive
}

}  // namespace

extern "C" {

size_t tango_mfma_i8_rate_workspace_bytes(void) { return static_cast<size_t>(256) * 256 * sizeof(int); }

int tango_mfma_i8_rate_launch(int iters, int random_operands, void *ws, size_t ws_bytes, double *ops, void *stream)
{
    TANGO_REQUIRE(iters >= 1 && iters <= (1 << 24), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(ws && ops, TANGO_ERR_NULL);
    TANGO_REQUIRE(ws_bytes >= tango_mfma_i8_rate_workspace_bytes(), TANGO_ERR_WORKSPACE);
    const int blocks = 256;  // one workgroup of 4 waves per compute unit: one wave per SIMD
    k_mfma_rate<<<blocks, 256, 0, tango_stream(stream)>>>(iters, random_operands, static_cast<int *>(ws));
    TANGO_LAUNCH_CHECK();
    *ops = 2.0 * 32 * 32 * 32 * 8.0 * iters * blocks * 4;
    return TANGO_OK;
}

}  // extern "C"
