// Measured ceilings of the box, for the roofline figures of the benchmark: what the matrix cores sustain
// on int8 operands with no memory traffic at all, and what a plain read-only stream gets out of HBM.
// Measurement support; nothing on the path of Eq. 7 / Eq. 8 calls these.
#include "../../include/llmint8.h"
#include "common.h"

namespace llmint8 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Register-only issue loop of v_mfma_i32_32x32x32_i8 in the shape of the prefill GEMM's main loop: a wave
// holds 4 x 4 accumulator tiles (256 registers) and two double-buffered operand sets of two k-steps
// (4 + 4 operand tiles each), loaded ONCE from the given tiled int8 matrices, and cycles through them:
// 64 MFMAs per iteration, every one on another pair of operand tiles, nothing else in the loop.  With the
// tiled codes of a real workload the operands have that workload's bit statistics (the rate depends on
// them: the chip is power-limited); with a buffer of zeros this is the pure issue rate.
__global__ void __launch_bounds__(256, 1) probe_mfma_kernel(const int8_t* __restrict__ A, size_t a_tiles,
                                                           const int8_t* __restrict__ B, size_t b_tiles, int iters,
                                                           int32_t* __restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    v4i RP[2][2][4], RQ[2][2][4];
#pragma unroll
    for (int q = 0; q < 16; q++) {
        const size_t ta = (wave * 16 + q) * 2654435761ull % a_tiles, tb = (wave * 16 + q) * 40503ull % b_tiles;
        RP[q >> 3][(q >> 2) & 1][q & 3] = *((const v4i*)(A + ta * TILE_BYTES) + lane);
        RQ[q >> 3][(q >> 2) & 1][q & 3] = *((const v4i*)(B + tb * TILE_BYTES) + lane);
    }
    v16i acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
        for (int b = 0; b < 4; b++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[a][b][r] = 0;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int S = 0; S < 2; S++)
#pragma unroll
            for (int c = 0; c < 2; c++)
#pragma unroll
                for (int a = 0; a < 4; a++)
#pragma unroll
                    for (int b = 0; b < 4; b++)
                        acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(RP[S][c][a], RQ[S][c][b], acc[a][b], 0, 0, 0);
    }
    int t = 0;
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
        for (int b = 0; b < 4; b++)
#pragma unroll
            for (int r = 0; r < 16; r++) t ^= acc[a][b][r];
    if (t == 0x5a5a5a5a) sink[0] = t;  // keeps the loop alive; the value is of no interest
}

// Read-only stream: the buffer is cut into one contiguous run of 1 KiB pieces per wave (a wave-wide 16-byte
// load moves one piece, as in the weight stream of the decode kernel), four non-temporal loads in flight
// per lane.  Many more waves than the chip holds at once, so finished ones are replaced all the time and
// neither a ramp nor a tail shows.  (Of the forms tried on one box - grid stride against contiguous runs,
// 4 / 8 / 16 loads in flight, plain against non-temporal loads, 1 024 to 16 384 workgroups - this one was
// the fastest: 7.0 TB/s over 604 MB; a grid-stride loop with plain loads got 5.6 TB/s.)
__global__ void __launch_bounds__(256) probe_read_kernel(const v4i* __restrict__ p, size_t pieces, int32_t* __restrict__ sink)
{
    const size_t waves = (size_t)gridDim.x * 4, wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const size_t per = (pieces + waves - 1) / waves;
    size_t k = wave * per, k1 = k + per;
    if (k1 > pieces) k1 = pieces;
    v4i s = {0, 0, 0, 0};
    for (; k + 4 <= k1; k += 4) {
        const v4i a = __builtin_nontemporal_load(p + k * 64 + lane), b = __builtin_nontemporal_load(p + (k + 1) * 64 + lane);
        const v4i c = __builtin_nontemporal_load(p + (k + 2) * 64 + lane), d = __builtin_nontemporal_load(p + (k + 3) * 64 + lane);
        s += a + b + c + d;
    }
    for (; k < k1; k++) s += __builtin_nontemporal_load(p + k * 64 + lane);
    if ((s.x ^ s.y ^ s.z ^ s.w) == 0x12345679) sink[0] = 1;  // keeps the loads alive; the value is of no interest
}

}  // namespace llmint8

using namespace llmint8;

extern "C" {

int llmint8_probe_mfma(const int8_t* A_tiles, size_t a_bytes, const int8_t* B_tiles, size_t b_bytes, int iters,
                       int32_t* sink, double* ops, llmint8_stream_t stream)
{
    if (!A_tiles || !B_tiles || !sink || iters < 1 || a_bytes < TILE_BYTES || b_bytes < TILE_BYTES) return LLMINT8_INVALID_ARG;
    if (((uintptr_t)A_tiles & 15) || ((uintptr_t)B_tiles & 15)) return LLMINT8_INVALID_ARG;
    int cus = 0;
    if (prefill_device_setup(&cus) != hipSuccess) return LLMINT8_HIP;
    probe_mfma_kernel<<<cus, 256, 0, (hipStream_t)stream>>>(A_tiles, a_bytes / TILE_BYTES, B_tiles, b_bytes / TILE_BYTES, iters,
                                                           sink);
    if (ops) *ops = (double)cus * 4.0 * iters * 64.0 * 65536.0;  // 2 * 32 * 32 * 32 int8 operations per MFMA
    return hipGetLastError() == hipSuccess ? LLMINT8_OK : LLMINT8_HIP;
}

int llmint8_probe_read(const void* buf, size_t bytes, int32_t* sink, llmint8_stream_t stream)
{
    if (!buf || !sink || bytes < 1024 || ((uintptr_t)buf & 15)) return LLMINT8_INVALID_ARG;
    int cus = 0;
    if (prefill_device_setup(&cus) != hipSuccess) return LLMINT8_HIP;
    probe_read_kernel<<<cus * 64, 256, 0, (hipStream_t)stream>>>((const v4i*)buf, bytes / 1024, sink);
    return hipGetLastError() == hipSuccess ? LLMINT8_OK : LLMINT8_HIP;
}

}  // extern "C"
