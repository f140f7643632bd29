// Decode path of Eq. 7 + Eq. 8 for s <= 32 tokens: the int8 weights are
// streamed from HBM exactly once; the few tokens ride along as the second MFMA
// operand.  Bandwidth bound (h * o bytes of W_i8 dominate).
#include "common.h"

namespace llmint8 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// One workgroup = 4 waves owns NJ tiles of 32 output columns.  The waves split
// K four ways; each streams its quarter of the W tiles (1 KiB contiguous per
// wave load, U tiles in flight per column tile) and multiplies it with the
// matching X tile (row tile 0 of Xq: tokens 0..31, zero padded).  The four
// partial accumulators meet in LDS; int32 sums are exact in any order.
template <int NJ, int U>
__global__ void __launch_bounds__(256)
gemm_decode_kernel(const int8_t* __restrict__ Wq, const int8_t* __restrict__ Xq, int KT, int JT,
                   const unsigned short* __restrict__ cw, const unsigned short* __restrict__ cx,
                   const unsigned short* __restrict__ Wf, const int32_t* __restrict__ idx,
                   const unsigned short* __restrict__ Xo, const int32_t* __restrict__ count, int cap, int opad, _Float16* __restrict__ Out,
                   int32_t* __restrict__ Cdbg, int s, int h, int o)
{
    __shared__ int red[4][NJ][16][64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kq = KT / 4;  // KT is a multiple of 4
    const int jt0 = blockIdx.x * NJ;
    const v4i* wp[NJ];
#pragma unroll
    for (int n = 0; n < NJ; n++) {
        int jt = jt0 + n;
        jt = jt < JT ? jt : JT - 1;
        wp[n] = (const v4i*)(Wq + ((size_t)jt * KT + (size_t)w * kq) * TILE_BYTES) + lane;
    }
    const v4i* xp = (const v4i*)(Xq + (size_t)w * kq * TILE_BYTES) + lane;

    v16i acc[NJ];
#pragma unroll
    for (int n = 0; n < NJ; n++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[n][r] = 0;

    int kt = 0;
    for (; kt + U <= kq; kt += U) {
        v4i wv[NJ][U], xv[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
#pragma unroll
            for (int n = 0; n < NJ; n++) wv[n][u] = __builtin_nontemporal_load(wp[n] + (size_t)(kt + u) * 64);
            xv[u] = xp[(size_t)(kt + u) * 64];
        }
#pragma unroll
        for (int u = 0; u < U; u++)
#pragma unroll
            for (int n = 0; n < NJ; n++)
                acc[n] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wv[n][u], xv[u], acc[n], 0, 0, 0);
    }
    for (; kt < kq; kt++) {
        v4i xv = xp[(size_t)kt * 64];
#pragma unroll
        for (int n = 0; n < NJ; n++) {
            v4i wv = __builtin_nontemporal_load(wp[n] + (size_t)kt * 64);
            acc[n] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wv, xv, acc[n], 0, 0, 0);
        }
    }
#pragma unroll
    for (int n = 0; n < NJ; n++)
#pragma unroll
        for (int r = 0; r < 16; r++) red[w][n][r][lane] = acc[n][r];
    __syncthreads();

    // Epilogue: thread -> (token i, column jj of a tile) so that consecutive threads write
    // consecutive columns.  Accumulator element (i, jj) of a tile lives in register
    // r = 4*(jj/8) + jj%4 of lane l = i + 32*((jj/4)%2).
    int cnt = *count;
    cnt = cnt < 0 ? 0 : (cnt > cap ? cap : cnt);
    const int jj = tid & 31;
    const int r = 4 * (jj >> 3) + (jj & 3);
    const int lsel = 32 * ((jj >> 2) & 1);
#pragma unroll
    for (int n = 0; n < NJ; n++) {
        const int j = (jt0 + n) * 32 + jj;
        if (j >= o) continue;
        const float cwj = f16_bits_to_float(cw[j]);
        for (int i = tid >> 5; i < s; i += 8) {
            const int l = i + lsel;
            const int c = red[0][n][r][l] + red[1][n][r][l] + red[2][n][r][l] + red[3][n][r][l];
            if (Cdbg) Cdbg[(size_t)i * o + j] = c;
            // Eq. 7 dequantization, then the outlier product of Eq. 8 accumulated in fp32
            float d = (float)c * (f16_bits_to_float(cx[i]) * (1.0f / 16129.0f)) * cwj;
            for (int t = 0; t < cnt; t++) {
                const unsigned k = (unsigned)idx[t];  // row of the original fp16 weights
                if (k < (unsigned)h)
                    d = __builtin_fmaf(f16_bits_to_float(Xo[(size_t)i * opad + t]),
                                       f16_bits_to_float(Wf[(size_t)k * o + j]), d);
            }
            Out[(size_t)i * o + j] = (_Float16)d;
        }
    }
}

hipError_t launch_gemm_decode(const int8_t* Xq, const unsigned short* cx, const unsigned short* Xo,
                              const int32_t* count, int cap, const int8_t* Wq, const unsigned short* cw,
                              const unsigned short* Wf, const int32_t* idx, int s, int h, int o,
                              unsigned short* Out, int32_t* Cdbg, hipStream_t st)
{
    const int KT = k_tiles(h), JT = row_tiles(o);
    constexpr int NJ = 1, U = 8;
    gemm_decode_kernel<NJ, U><<<(JT + NJ - 1) / NJ, 256, 0, st>>>(Wq, Xq, KT, JT, cw, cx, Wf, idx, Xo, count, cap,
                                                                 opad_of(cap), (_Float16*)Out, Cdbg, s, h, o);
    return hipGetLastError();
}

}  // namespace llmint8
