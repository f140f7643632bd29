// Prefill path of Eq. 7 + Eq. 8: int8 MFMA GEMM over the tiled operands with
// the dequantization and the fp16 outlier product fused into the epilogue.
#include "common.h"

namespace llmint8 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));

#define GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define LPTR(p) ((__attribute__((address_space(3))) void*)(p))
#define SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)

// s_waitcnt immediate for gfx9: vmcnt = n, lgkmcnt and expcnt left open.
// WAIT_VMCNT_LGKM0 additionally waits for every LDS / scalar-memory operation of the wave.
#define WAIT_VMCNT_LGKM0(n) __builtin_amdgcn_s_waitcnt(0x0070 | ((n) & 0xf) | ((((n) >> 4) & 3) << 14))

// ---------------------------------------------------------------------------
// int8 GEMM, 256 output columns x 256 tokens per workgroup, 4 waves, each
// wave a 128 x 128 sub-tile = 4 x 4 MFMA tiles of 32 x 32 (256 accumulator
// registers per lane).  The MFMA "A" operand is a W tile (its 32 rows are
// output columns j), the "B" operand an X tile (32 tokens i), so a lane ends
// up with 4 consecutive output columns of one token per register quad.
//
// K pipeline: a stage is 64 features (2 MFMA k-steps) of all 16 row tiles =
// 32 KiB; NB stages form a ring in LDS (128 KiB).  Tiles go global -> LDS
// with 16-byte direct loads, one 1 KiB tile per wave instruction, and are
// read back with one ds_read_b128 per operand (linear, conflict free).
// One barrier per stage, placed before the stage's last k-step: it publishes
// stage st+1 (every wave waited for its own loads of it) and retires the ring
// slot of stage st (all its operands are in registers by then), which is
// refilled right away with stage st+NB: NB-1 stages of lookahead.
// ---------------------------------------------------------------------------
constexpr int NB = 4;
constexpr int STAGE_BYTES = 16 * 2 * TILE_BYTES;  // 32 KiB
constexpr int LOADS_PER_STAGE = 8;                // per wave: 32 tiles / 4 waves

__global__ void __launch_bounds__(256, 1)
gemm_prefill_kernel(const int8_t* __restrict__ Wq, const int8_t* __restrict__ Xq, int KT, int JT, int RT,
                    int nP, int nQ, const unsigned short* __restrict__ cw, const unsigned short* __restrict__ cx,
                    const unsigned short* __restrict__ Wf, const int32_t* __restrict__ idx,
                    const _Float16* __restrict__ Xo, const int32_t* __restrict__ count, int cap, int opad, _Float16* __restrict__ Out,
                    int32_t* __restrict__ Cdbg, int s, int h, int o)
{
    extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- workgroup -> output tile.  Hardware deals consecutive workgroup ids
    // round-robin to the 8 XCDs; give each XCD a contiguous run of the tile
    // order so that tiles sharing operand panels meet in one L2.  Within the
    // order, bands of 4 token blocks are walked column block by column block.
    int pj, qi;
    {
        const int total = nP * nQ;
        const int wg = blockIdx.x;
        const int xcd = wg & 7, within = wg >> 3;
        const int base = total >> 3, rem = total & 7;
        const int logical = xcd * base + (xcd < rem ? xcd : rem) + within;
        constexpr int BAND = 4;
        const int band = logical / (BAND * nP);
        const int inband = logical - band * BAND * nP;
        const int q0 = band * BAND;
        const int bh = (nQ - q0) < BAND ? (nQ - q0) : BAND;  // rows in this band
        pj = inband / bh;
        qi = q0 + inband - pj * bh;
    }

    // ---- loader role: waves 0,1 bring W row tiles 0-3 / 4-7 of the block, waves 2,3 X row tiles
    const bool isQ = w >= 2;
    const int8_t* gsrc = isQ ? Xq : Wq;
    const int ntile = isQ ? RT : JT;
    const int tbase = (isQ ? qi : pj) * 8 + (w & 1) * 4;
    const int8_t* gp[4];
    const unsigned voff = lane * 16;
#pragma unroll
    for (int a = 0; a < 4; a++) {
        int t = tbase + a;
        t = t < ntile ? t : ntile - 1;  // clamp: rows past the matrix re-read the last tile, results unused
        gp[a] = gsrc + (size_t)t * KT * TILE_BYTES;
    }
    const int lslot = ((isQ ? 8 : 0) + (w & 1) * 4) * 2;  // first 1 KiB slot this wave fills in a stage
    const int wp = w >> 1, wq = w & 1;                    // compute role: column half, token half

    v16i acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
        for (int b = 0; b < 4; b++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[a][b][r] = 0;

    const int nst = KT / 2;
    // stage `st` of the operands -> ring slot `slot`
    auto issue = [&](int st, int slot) {
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
            for (int c = 0; c < 2; c++)
                __builtin_amdgcn_global_load_lds(GPTR(gp[a] + (size_t)st * 2048 + c * 1024 + voff),
                                                 LPTR(lds + slot * STAGE_BYTES + (lslot + a * 2 + c) * 1024), 16, 0, 0);
    };
    const int8_t* Pl = lds + (wp * 4) * 2048 + lane * 16;
    const int8_t* Ql = lds + (8 + wq * 4) * 2048 + lane * 16;
    auto rdP = [&](v4i(&P)[4], int buf, int c) {
#pragma unroll
        for (int a = 0; a < 4; a++) P[a] = *(const v4i*)(Pl + buf * STAGE_BYTES + a * 2048 + c * 1024);
    };
    auto rdQ = [&](v4i(&Q)[4], int buf, int c) {
#pragma unroll
        for (int b = 0; b < 4; b++) Q[b] = *(const v4i*)(Ql + buf * STAGE_BYTES + b * 2048 + c * 1024);
    };
    auto mm = [&](v4i(&P)[4], v4i(&Q)[4]) {
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
            for (int b = 0; b < 4; b++)
                acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(P[a], Q[b], acc[a][b], 0, 0, 0);
    };

    // prologue: fill the whole ring (stage indices past the end re-read the last stage; never consumed)
#pragma unroll
    for (int st = 0; st < NB; st++) issue(st < nst ? st : nst - 1, st);
    WAIT_VMCNT_LGKM0((NB - 1) * LOADS_PER_STAGE);
    __syncthreads();
    v4i P0[4], Q0[4], P1[4], Q1[4];
    rdP(P0, 0, 0);
    rdQ(Q0, 0, 0);
    for (int st = 0; st < nst; st++) {
        const int buf = st % NB;
        // k-step 0, while the operands of k-step 1 come in from the same stage
        rdP(P1, buf, 1);
        rdQ(Q1, buf, 1);
        mm(P0, Q0);
#pragma unroll
        for (int g = 0; g < 8; g++) {
            SGB(0x008, 2);
            SGB(0x100, 1);
        }
        __builtin_amdgcn_sched_barrier(0);
        // My loads of stage st+1 have landed (the NB-2 younger stages may still fly) and my reads of
        // stage st are complete; after the barrier the same holds for every wave, so slot `buf` is
        // free and is refilled with stage st+NB.
        WAIT_VMCNT_LGKM0((NB - 2) * LOADS_PER_STAGE);
        __syncthreads();
        {
            const int nx = st + NB;
            issue(nx < nst ? nx : nst - 1, buf);
        }
        rdP(P0, (st + 1) % NB, 0);
        rdQ(Q0, (st + 1) % NB, 0);
        mm(P1, Q1);
#pragma unroll
        for (int g = 0; g < 8; g++) {
            SGB(0x008, 2);
            SGB(0x020, 1);
            SGB(0x100, 1);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    WAIT_VMCNT_LGKM0(0);  // drain the redundant tail loads before the LDS allocation goes away

    // ---- epilogue ----------------------------------------------------------
    // acc[a][b][r] of lane l: token i = I0 + b*32 + (l & 31),
    //                         column j = J0 + a*32 + 8*(r >> 2) + 4*(l >> 5) + (r & 3)
    int cnt = *count;
    cnt = cnt < 0 ? 0 : (cnt > cap ? cap : cnt);
    const int J0 = pj * 256 + wp * 128;
    const int I0 = qi * 256 + wq * 128;
    const int g = lane >> 5;
    const bool vec_store = (o & 3) == 0;

    if (Cdbg) {
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
            for (int b = 0; b < 4; b++) {
                const int i = I0 + b * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int j = J0 + a * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (i < s && j < o) Cdbg[(size_t)i * o + j] = acc[a][b][r];
                }
            }
    }

    float sx[4];
#pragma unroll
    for (int b = 0; b < 4; b++) {
        const int i = I0 + b * 32 + (lane & 31);
        // c_x / 127^2 for this lane's token (Eq. 7: S = c_x (x) c_w / 127^2)
        sx[b] = (i < s) ? f16_bits_to_float(cx[i]) * (1.0f / 16129.0f) : 0.0f;
    }
    // Eq. 8, outlier term: the rows O of the original fp16 weights are read straight from W_f16
    // (|O| * o * 2 bytes in all).  Lane l supplies outlier slots 8*(l>>5) .. +7 of a 16-slot k-step
    // for column J0 + a*32 + (l & 31) (MFMA "A" operand) and for its token (MFMA "B" operand).
    auto load_w = [&](int jcol, int t0) {
        v8h wa;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const int t = t0 + 8 * g + e;
            unsigned short v = 0;
            if (t < cnt && jcol < o) {
                const unsigned k = (unsigned)idx[t];
                if (k < (unsigned)h) v = Wf[(size_t)k * o + jcol];
            }
            wa[e] = __builtin_bit_cast(_Float16, v);
        }
        return wa;
    };
    v8h xb0[4];
#pragma unroll
    for (int b = 0; b < 4; b++) {
        const int i = I0 + b * 32 + (lane & 31);
        xb0[b] = (v8h)(0);
        if (i < s && cnt > 0) xb0[b] = *(const v8h*)(Xo + (size_t)i * opad + 8 * g);
    }
#pragma unroll
    for (int a = 0; a < 4; a++) {
        const int jb = J0 + a * 32 + 4 * g;
        float cwv[16];
#pragma unroll
        for (int rr = 0; rr < 4; rr++) {
            const int j = jb + 8 * rr;
            if (j + 3 < o) {
                const uint2 pk = *(const uint2*)(cw + j);  // 4 halves, j % 4 == 0
                cwv[4 * rr + 0] = f16_bits_to_float((unsigned short)(pk.x & 0xffff));
                cwv[4 * rr + 1] = f16_bits_to_float((unsigned short)(pk.x >> 16));
                cwv[4 * rr + 2] = f16_bits_to_float((unsigned short)(pk.y & 0xffff));
                cwv[4 * rr + 3] = f16_bits_to_float((unsigned short)(pk.y >> 16));
            } else {
#pragma unroll
                for (int e = 0; e < 4; e++) cwv[4 * rr + e] = (j + e < o) ? f16_bits_to_float(cw[j + e]) : 0.0f;
            }
        }
        const int ja = J0 + a * 32 + (lane & 31);
        v8h wa0 = (v8h)(0);
        if (cnt > 0) wa0 = load_w(ja, 0);
#pragma unroll
        for (int b = 0; b < 4; b++) {
            const int i = I0 + b * 32 + (lane & 31);
            const bool iok = i < s;
            v16f d;
#pragma unroll
            for (int r = 0; r < 16; r++) d[r] = (float)acc[a][b][r] * sx[b] * cwv[r];
            if (cnt > 0) d = __builtin_amdgcn_mfma_f32_32x32x16_f16(wa0, xb0[b], d, 0, 0, 0);
            for (int t0 = 16; t0 < cnt; t0 += 16) {  // more than 16 outlier columns: rare
                v8h wa = load_w(ja, t0);
                v8h xb = (v8h)(0);
                if (iok) xb = *(const v8h*)(Xo + (size_t)i * opad + t0 + 8 * g);
                d = __builtin_amdgcn_mfma_f32_32x32x16_f16(wa, xb, d, 0, 0, 0);
            }
            if (iok) {
#pragma unroll
                for (int rr = 0; rr < 4; rr++) {
                    const int j = jb + 8 * rr;
                    if (vec_store && j + 3 < o) {
                        v4h hv = {(_Float16)d[4 * rr], (_Float16)d[4 * rr + 1], (_Float16)d[4 * rr + 2],
                                  (_Float16)d[4 * rr + 3]};
                        *(v4h*)(Out + (size_t)i * o + j) = hv;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; e++)
                            if (j + e < o) Out[(size_t)i * o + j + e] = (_Float16)d[4 * rr + e];
                    }
                }
            }
        }
    }
}

hipError_t launch_gemm_prefill(const int8_t* Xq, const unsigned short* cx, const unsigned short* Xo,
                               const int32_t* count, int cap, const int8_t* Wq, const unsigned short* cw,
                               const unsigned short* Wf, const int32_t* idx, int s, int h, int o,
                               unsigned short* Out, int32_t* Cdbg, hipStream_t st)
{
    const int KT = k_tiles(h), JT = row_tiles(o), RT = row_tiles(s);
    const int nP = (JT + 7) / 8, nQ = (RT + 7) / 8;
    static bool attr_set = false;
    const int shm = NB * STAGE_BYTES;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)gemm_prefill_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, shm);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    gemm_prefill_kernel<<<nP * nQ, 256, shm, st>>>(Wq, Xq, KT, JT, RT, nP, nQ, cw, cx, Wf, idx,
                                                   (const _Float16*)Xo, count, cap, opad_of(cap),
                                                   (_Float16*)Out, Cdbg, s, h, o);
    return hipGetLastError();
}

}  // namespace llmint8
