// Decode path of Eq. 7 + Eq. 8 for few tokens (s <= 32, and up to 64 against a
// wide W): the int8 weights are streamed from HBM exactly once; the tokens ride
// along as the second MFMA operand.  Bandwidth bound (h * o bytes of W_i8
// dominate).
#include <type_traits>

#include "common.h"

namespace llmint8 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define FENCE() __builtin_amdgcn_sched_barrier(0)

constexpr int DSLOTS = 16;  // outlier slots whose operands are fetched before the weight stream starts

// One workgroup = 4 waves owns NJ tiles of 32 output columns and NI tiles of 32
// tokens.  The waves split K four ways; each streams its quarter of the W tiles
// (1 KiB contiguous per wave load) in batches of U k-tiles, two batches in
// flight, and multiplies them with the matching X tiles (row tiles 0 .. NI-1 of
// Xq, zero padded, from L2).  The four partial accumulators meet in LDS, one
// token tile after the other; int32 sums are exact in any order.  With one
// token tile, what the epilogue needs (c_w, c_x, the outlier columns of X and
// the matching rows of the fp16 weights) is requested before the stream starts,
// so that no workgroup ends with a chain of dependent loads; with more, only
// the per-column part is (the per-token part would take too many registers) and
// the rest is loaded in the epilogue, under the stream of the compute unit's
// other workgroup.
//
// ZP: zeropoint constants (Eq. 1-5) in place of c_x / c_w: the epilogue adds the three correction
// terms of the unrolled product of Eq. 5 to the accumulator (in double: with zeropoints far from 0
// they are large and cancel) and divides by nd_x nd_w.
template <int NJ, int NI, int U, bool ZP>
__global__ void __launch_bounds__(256)
gemm_decode_kernel(const int8_t* __restrict__ Wq, const int8_t* __restrict__ Xq, int KT, int JT,
                   const unsigned short* __restrict__ cw, const unsigned short* __restrict__ cx,
                   const unsigned short* __restrict__ Wf, int rows_are_slots, int wrows,
                   const int32_t* __restrict__ idx, const unsigned short* __restrict__ Xo,
                   const int32_t* __restrict__ count, int cap, int opad,
                   _Float16* __restrict__ Out, int32_t* __restrict__ Cdbg, int s, int h, int o, const ZpArgs zp)
{
    __shared__ int red[4][NJ][16][64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kq = KT / 4;  // KT is a multiple of 4
    const int jt0 = blockIdx.x * NJ;

    // ---- epilogue operands, requested first.  Thread -> column jj of a tile, tokens ig, ig+8, ig+16, ig+24.
    // Every load here is unconditional (an index that does not exist is replaced by one that does; the value is
    // never used, because the epilogue skips tokens >= s, columns >= o and slots >= count), and nothing is done
    // with a loaded value before the first batch of the weight stream has been requested: a load under a bounds
    // check of its own is compiled as branch, load, wait, and the operands would arrive one round trip after the
    // other (sixteen of them for the rows of Wf alone) before the stream could start.
    int cnt = *count;
    cnt = cnt < 0 ? 0 : (cnt > cap ? cap : cnt);
    const int jj = tid & 31, ig = tid >> 5;
    constexpr bool EARLY = NI == 1;  // per-token epilogue operands fetched before the stream
    float cwj[NJ], sxi[4];
    unsigned wo[NJ][DSLOTS / 2];  // fp16 pairs: slots 2q (low half) and 2q+1 of this thread's columns
    uint4 xo[4][DSLOTS / 8];      // slots 0..15 of this thread's tokens (Xo holds zeros past |O|)
    double zp_[ZP ? NJ : 1], zq_[ZP ? NJ : 1], zr_[ZP ? NJ : 1];  // column factors p, q, r of zp_kcol_kernel
    double zsa[ZP ? 4 : 1], zza[ZP ? 4 : 1], zrs[ZP ? 4 : 1];     // D_x / 254, zp_x, row sums of the codes
    // the rows of Wf that the outlier slots need: lanes 0 .. DSLOTS-1 fetch idx[lane] in one load (entries
    // past the count hold whatever the caller left there and are not used)
    unsigned kraw = (unsigned)lane;
    if (!rows_are_slots) kraw = (unsigned)idx[(lane < DSLOTS && lane < cap) ? lane : 0];
    unsigned short cw_raw[NJ], cx_raw[4];
    int4 zx_raw[ZP ? 4 : 1];
#pragma unroll
    for (int n = 0; n < NJ; n++) {
        const int j = (jt0 + n) * 32 + jj;
        if constexpr (ZP) {
            zp_[n] = zp.colc[j];  // planes are padded to a multiple of 256 columns
            zq_[n] = zp.colc[(size_t)zp.pitch + j];
            zr_[n] = zp.colc[2 * (size_t)zp.pitch + j];
        } else {
            cw_raw[n] = cw[j < o ? j : 0];
        }
    }
    // the per-token operands of token tile ti: this thread's tokens 32 ti + ig + 8 m
    auto token_loads = [&](int ti) {
#pragma unroll
        for (int m = 0; m < 4; m++) {
            const int i = 32 * ti + ig + 8 * m;
            const int ii = i < s ? i : s - 1;
            if constexpr (ZP) zx_raw[m] = zp.zcx[ii]; else cx_raw[m] = cx[ii];
#pragma unroll
            for (int q = 0; q < DSLOTS / 8; q++) xo[m][q] = *(const uint4*)(Xo + (size_t)ii * opad + 8 * q);
        }
    };
    auto token_values = [&]() {
#pragma unroll
        for (int m = 0; m < 4; m++) {
            if constexpr (ZP) {
                zsa[m] = zp_range((unsigned)zx_raw[m].x) * (1.0 / 254.0);
                zza[m] = (double)zx_raw[m].y;
                zrs[m] = (double)zx_raw[m].z;
            } else {
                sxi[m] = f16_bits_to_float(cx_raw[m]) * (1.0f / 16129.0f);
            }
        }
    };
    if constexpr (EARLY) token_loads(0);
    FENCE();

    // ---- weight stream
    const v4i* wp[NJ];
#pragma unroll
    for (int n = 0; n < NJ; n++) {
        int jt = jt0 + n;
        jt = jt < JT ? jt : JT - 1;  // tiles past the matrix re-read the last one, results unused
        wp[n] = (const v4i*)(Wq + ((size_t)jt * KT + (size_t)w * kq) * TILE_BYTES) + lane;
    }
    // a lane holds token (lane % 32) of an X tile; tokens >= s are zero padding and need not be fetched
    const v4i* xp[NI];
    bool xrow[NI];
#pragma unroll
    for (int ti = 0; ti < NI; ti++) {
        xp[ti] = (const v4i*)(Xq + ((size_t)ti * KT + (size_t)w * kq) * TILE_BYTES) + lane;
        xrow[ti] = 32 * ti + (lane & 31) < s;
    }

    v16i acc[NJ][NI];
#pragma unroll
    for (int n = 0; n < NJ; n++)
#pragma unroll
        for (int ti = 0; ti < NI; ti++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[n][ti][r] = 0;

    v4i wv[2][NJ][U], xv[2][NI][U];
    auto load = [&](auto B, int kt) {
        constexpr int BB = decltype(B)::value;
#pragma unroll
        for (int u = 0; u < U; u++) {
#pragma unroll
            for (int n = 0; n < NJ; n++) wv[BB][n][u] = __builtin_nontemporal_load(wp[n] + (size_t)(kt + u) * 64);
#pragma unroll
            for (int ti = 0; ti < NI; ti++) xv[BB][ti][u] = xrow[ti] ? xp[ti][(size_t)(kt + u) * 64] : v4i{0, 0, 0, 0};
        }
    };
    auto mm = [&](auto B) {
        constexpr int BB = decltype(B)::value;
#pragma unroll
        for (int u = 0; u < U; u++)
#pragma unroll
            for (int n = 0; n < NJ; n++)
#pragma unroll
                for (int ti = 0; ti < NI; ti++)
                    acc[n][ti] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wv[BB][n][u], xv[BB][ti][u], acc[n][ti], 0, 0, 0);
    };
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;
    const int nb = kq / U;  // full batches
    if (nb > 0) load(B0{}, 0);
    FENCE();
    // the rows of Wf, behind the first weight batch: they wait for the column indices, the batch does not
    unsigned okmask = 0;  // slots whose row of Wf exists (uniform)
    unsigned short wo_raw[NJ][DSLOTS];
#pragma unroll
    for (int t = 0; t < DSLOTS; t++) {
        const unsigned k = (unsigned)__builtin_amdgcn_readlane((int)kraw, t);
        const bool ok = k < (unsigned)wrows;
        okmask |= ok ? 1u << t : 0u;
#pragma unroll
        for (int n = 0; n < NJ; n++) {
            const int j = (jt0 + n) * 32 + jj;
            wo_raw[n][t] = Wf[(size_t)(ok ? k : 0u) * o + (j < o ? j : 0)];
        }
    }
    FENCE();
    int b = 0;
    for (; b + 2 <= nb; b += 2) {
        load(B1{}, (b + 1) * U);
        FENCE();
        mm(B0{});
        FENCE();
        if (b + 2 < nb) load(B0{}, (b + 2) * U);
        FENCE();
        mm(B1{});
        FENCE();
    }
    if (b < nb) mm(B0{});  // odd number of batches: the last one is already in flight in buffer 0
    for (int kt = nb * U; kt < kq; kt++) {
        v4i x1[NI];
#pragma unroll
        for (int ti = 0; ti < NI; ti++) x1[ti] = xrow[ti] ? xp[ti][(size_t)kt * 64] : v4i{0, 0, 0, 0};
#pragma unroll
        for (int n = 0; n < NJ; n++) {
            const v4i w1 = __builtin_nontemporal_load(wp[n] + (size_t)kt * 64);
#pragma unroll
            for (int ti = 0; ti < NI; ti++)
                acc[n][ti] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w1, x1[ti], acc[n][ti], 0, 0, 0);
        }
    }

    // ---- the epilogue operands into the form the epilogue wants (not earlier: their loads complete in the order
    // of issue, and a use in front of the stream would wait for everything requested before them)
#pragma unroll
    for (int n = 0; n < NJ; n++) {
        if constexpr (!ZP) cwj[n] = f16_bits_to_float(cw_raw[n]);
#pragma unroll
        for (int t = 0; t < DSLOTS; t += 2) wo[n][t >> 1] = (unsigned)wo_raw[n][t] | ((unsigned)wo_raw[n][t + 1] << 16);
    }
    if constexpr (EARLY) token_values();
    FENCE();
    // ---- reduction over the four waves and epilogue, token tile by token tile.  Accumulator element (token
    // i of the tile, column jj) lives in register r = 4*(jj/8) + jj%4 of lane l = i + 32*((jj/4)%2).
    const int r = 4 * (jj >> 3) + (jj & 3);
    const int lsel = 32 * ((jj >> 2) & 1);
#pragma unroll
    for (int ti = 0; ti < NI; ti++) {
    if (ti > 0) __syncthreads();  // every thread is done reading the tile before
#pragma unroll
    for (int n = 0; n < NJ; n++)
#pragma unroll
        for (int q = 0; q < 16; q++) red[w][n][q][lane] = acc[n][ti][q];
    if constexpr (!EARLY) {
        token_loads(ti);
        token_values();
    }
    __syncthreads();
#pragma unroll
    for (int n = 0; n < NJ; n++) {
        const int j = (jt0 + n) * 32 + jj;
        if (j >= o) continue;
#pragma unroll
        for (int m = 0; m < 4; m++) {
            const int il = ig + 8 * m, i = 32 * ti + il;
            if (i >= s) continue;
            const int l = il + lsel;
            const int c = red[0][n][r][l] + red[1][n][r][l] + red[2][n][r][l] + red[3][n][r][l];
            if (Cdbg) Cdbg[(size_t)i * o + j] = c;
            // Eq. 7 dequantization, then the outlier product of Eq. 8 accumulated in fp32
            float d;
            if constexpr (ZP) {
                // Eq. 5 over nd_w: C p + rowsum q + zp_x r, then the division by nd_x
                d = (float)(zsa[m] * __builtin_fma((double)c, zp_[n], __builtin_fma(zrs[m], zq_[n], zza[m] * zr_[n])));
            } else {
                d = (float)c * sxi[m] * cwj[n];
            }
#pragma unroll
            for (int t = 0; t < DSLOTS; t++)
                if (t < cnt && ((okmask >> t) & 1u)) {
                    const unsigned xw = ((const unsigned*)&xo[m][t >> 3])[(t & 7) >> 1];
                    const unsigned short xh = (unsigned short)((t & 1) ? (xw >> 16) : (xw & 0xffff));
                    const unsigned short wh = (unsigned short)((t & 1) ? (wo[n][t >> 1] >> 16) : (wo[n][t >> 1] & 0xffff));
                    d = __builtin_fmaf(f16_bits_to_float(xh), f16_bits_to_float(wh), d);
                }
            for (int t = DSLOTS; t < cnt; t++) {  // more outlier columns than were prefetched: rare
                const unsigned k = rows_are_slots ? (unsigned)t : (unsigned)idx[t];
                if (k < (unsigned)wrows)
                    d = __builtin_fmaf(f16_bits_to_float(Xo[(size_t)i * opad + t]),
                                       f16_bits_to_float(Wf[(size_t)k * o + j]), d);
            }
            Out[(size_t)i * o + j] = (_Float16)d;
        }
    }
    }  // token tiles
}

std::atomic<int> g_decode_cfg{-1};  // test hook, as g_force_cfg

// Which token counts take this kernel: up to 32 always; 33 to 48 (two token tiles per workgroup) when W is
// wide enough for its halved grid to fill the chip with two workgroups per compute unit, where the call is
// bound by the weight stream and the tiled GEMM gets less out of it: 119.4 against 133.3 us at 33 tokens,
// 127.6 against 134.5 at 48, but 142.7 against 123.5 at 64, where the X tiles that every workgroup re-reads
// from L2 are as many bytes as W (175B-shaped decode size).  Absmax only: with the zeropoint epilogue that
// instantiation needs more registers than two workgroups per compute unit leave.
bool decode_kernel_takes(int s, int h, int o, bool zeropoint)
{
    const int forced = g_decode_cfg.load(std::memory_order_relaxed);
    if (forced == 0) return false;  // test hook: every token count through the tiled kernel
    if (s > 48 || (s > 32 && zeropoint)) return false;
    int cus = 0;
    if (prefill_device_setup(&cus) != hipSuccess) cus = 256;
    const int JT = row_tiles(o);
    if (s <= 32) {
        // Two workgroups of this kernel fit a compute unit, so a W of 2 to 4 column tiles per compute unit is
        // taken in two rounds, the second one part empty, while the tiled kernel has one 128 x 128 tile for
        // each of more than half of the compute units.  Per call at 8 / 16 / 32 tokens: 33.6 / 34.0 / 36.3 us
        // tiled against 36.2 / 38.2 / 43.3 on 6 656 x 17 920, 47.4 / 48.1 / 49.2 against 49.6 / 51.2 / 57.3 on
        // 8 192 x 28 672, 49.3 / 50.5 / 52.8 against 52.0 / 53.9 / 61.5 on 12 288 x 20 480.  One tile per compute
        // unit streams its 128 columns at what one compute unit can pull, which costs more the longer K is:
        // with the second round at least half full and K above 8 192 this kernel stays ahead (55.7 / 57.0 /
        // 64.6 against 68.8 / 73.0 / 75.0 us on 12 288 x 24 576), as it does with a full second round (32.0 /
        // 33.3 / 38.2 against 34.4 / 35.7 / 39.3 on 4 096 x 32 768) and outside the range (23.6 against 29.6 us
        // at 15 360 columns, 62.5 against 70.2 at 36 864).
        const int second = JT - 2 * cus;  // workgroups of the second round
        // (the zeropoint forms of the two kernels compare the same way: 39.1 against 44.3 us at 32 tokens on
        // 5 120 x 20 480, 55.9 against 68.0 on 8 192 x 28 672, 79.7 against 73.3 on 12 288 x 24 576)
        if (forced < 0 && second > 0 && second < 2 * cus && (o + 127) / 128 <= cus && (second < cus || h <= 8192))
            return false;
        return true;
    }
    return (JT + 1) / 2 >= 2 * cus;
}

hipError_t launch_gemm_decode(const int8_t* Xq, const unsigned short* cx, const unsigned short* Xo,
                              const int32_t* count, int cap, const int8_t* Wq, const unsigned short* cw,
                              const unsigned short* Wf, int rows_are_slots, const int32_t* idx, int s, int h, int o,
                              unsigned short* Out, int32_t* Cdbg, hipStream_t st, const ZpArgs* zp)
{
    const int KT = k_tiles(h), JT = row_tiles(o);
    const int wrows = rows_are_slots ? opad_of(cap) : h;
    const ZpArgs none = {nullptr, nullptr, 0};
    // Work split: one column tile per workgroup up to 16 tokens; above that every workgroup re-reads twice as
    // much of X_i8 from L2 per weight tile, and two column tiles per workgroup (half the re-reads) are faster:
    // 113.5 against 120.9 us at 32 tokens, 109.8 against 110.5 at 24, 107.4 against 104.6 at 16 (175B-shaped
    // decode size) - as long as the halved grid still fills the chip with two workgroups per compute unit
    // (at 5 120 x 20 480, 320 instead of 640 workgroups: 42.2 against 39.5 us at 32 tokens).
    int cus = 0;
    if (prefill_device_setup(&cus) != hipSuccess) cus = 256;
    const bool wide = s > 16 && (JT + 1) / 2 >= 2 * cus;
    if (s > 32) {  // two token tiles (decode_kernel_takes said so)
        if (zp || s > 64) return hipErrorInvalidValue;
        gemm_decode_kernel<2, 2, 4, false><<<(JT + 1) / 2, 256, 0, st>>>(Wq, Xq, KT, JT, cw, cx, Wf, rows_are_slots, wrows, idx,
                                                                        Xo, count, cap, opad_of(cap), (_Float16*)Out, Cdbg, s, h, o, none);
        return hipGetLastError();
    }
    if (zp) {
        if (wide)
            gemm_decode_kernel<2, 1, 4, true><<<(JT + 1) / 2, 256, 0, st>>>(Wq, Xq, KT, JT, cw, cx, Wf, rows_are_slots, wrows, idx, Xo,
                                                                        count, cap, opad_of(cap), (_Float16*)Out, Cdbg, s, h, o, *zp);
        else
            gemm_decode_kernel<1, 1, 8, true><<<JT, 256, 0, st>>>(Wq, Xq, KT, JT, cw, cx, Wf, rows_are_slots, wrows, idx, Xo,
                                                               count, cap, opad_of(cap), (_Float16*)Out, Cdbg, s, h, o, *zp);
        return hipGetLastError();
    }
#define LAUNCH_DECODE(NJ, U)                                                                                     \
    gemm_decode_kernel<NJ, 1, U, false><<<(JT + NJ - 1) / NJ, 256, 0, st>>>(Wq, Xq, KT, JT, cw, cx, Wf, rows_are_slots, wrows, idx, Xo, count, cap, \
                                                                 opad_of(cap), (_Float16*)Out, Cdbg, s, h, o, none)
    switch (g_decode_cfg.load(std::memory_order_relaxed)) {
        case 3: LAUNCH_DECODE(2, 8); break;
        case 4: LAUNCH_DECODE(3, 4); break;
        case 5: LAUNCH_DECODE(1, 4); break;
        case 2: LAUNCH_DECODE(2, 4); break;
        case 1: LAUNCH_DECODE(1, 8); break;
        default:  // not forced.  1 x 8: twice as many workgroups as 2 x 4, three full rounds of two per CU at the
                  // 175B-shaped decode size (16 tokens: 96.2 against 98.0 us; 1 x 4: 97.4, 1 x 6: 98.0, 1 x 12 and
                  // 1 x 16: 109.6, 2 x 4 with eight waves per workgroup, one workgroup per CU: 111)
            if (wide)
                LAUNCH_DECODE(2, 4);
            else
                LAUNCH_DECODE(1, 8);
            break;
    }
#undef LAUNCH_DECODE
    return hipGetLastError();
}

}  // namespace llmint8
