// Prefill path of Eq. 7 + Eq. 8: int8 MFMA GEMM over the tiled operands with
// the dequantization and the fp16 outlier product fused into the epilogue.
#include <atomic>
#include <mutex>
#include <type_traits>

#include "common.h"

namespace llmint8 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));

#define GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define LPTR(p) ((__attribute__((address_space(3))) void*)(p))
#define FENCE() __builtin_amdgcn_sched_barrier(0)

// s_waitcnt immediate for gfx9: vmcnt = n (6 bits, split 4 + 2), lgkmcnt = 0, expcnt left open.
#define WAIT_VMCNT_LGKM0(n) __builtin_amdgcn_s_waitcnt(0x0070 | ((n) & 0xf) | ((((n) >> 4) & 3) << 14))
// Workgroup barrier of the K pipeline: wait until at most n of this wave's direct loads are in flight and
// all its LDS reads are done, then s_barrier.  __syncthreads() is not used here: its release fence waits
// for every direct-to-LDS load in flight (vmcnt(0)), which would drain the pipeline at every stage.
#define STAGE_SYNC(n)                        \
    do {                                     \
        asm volatile("" ::: "memory");       \
        WAIT_VMCNT_LGKM0(n);                 \
        __builtin_amdgcn_s_barrier();        \
        asm volatile("" ::: "memory");       \
    } while (0)

struct GemmArgs {
    const int8_t* Wq;            // tiled W_i8 (tile rows = output columns)
    const int8_t* Xq;            // tiled X_i8 (tile rows = tokens)
    int KT, JT, RT;              // k tiles, column tiles of W, token tiles of X
    int nP, nQ;                  // workgroup grid: column blocks, token blocks
    const unsigned short* cw;    // [o] fp16 bits
    const unsigned short* cx;    // [s]
    const unsigned short* Wf;    // [h x o] original fp16 weights, or [opad x o] rebuilt outlier rows
    int rows_are_slots;          // 0: outlier slot t uses row idx[t] of Wf; 1: row t
    int wrows;                   // rows of Wf (h or opad)
    const int32_t* idx;          // [cap] outlier columns
    const _Float16* Xo;          // [s x opad] gathered outlier columns of X
    const int32_t* count;
    int cap, opad;
    _Float16* Out;               // [s x o]
    int32_t* Cdbg;               // NULL or [s x o]
    int s, h, o;
    int fast_ok;                 // o % 8 == 0, o < 2^21 and every epilogue operand 16-byte aligned
    int many_only;               // guarded kernel launched behind the unguarded one: it runs only if *count > OSLOTS
    ZpArgs zp;                   // zeropoint constants (ZP kernels only)
};

// ---------------------------------------------------------------------------
// One workgroup = 2 x WQ waves (column halves x token parts; WQ = 2 or 4) computes
// 64*WA output columns x 32*WQ*WB tokens; a wave owns WA x WB MFMA tiles of
// 32 x 32 (16*WA*WB accumulator registers per lane).  The MFMA "A" operand is a
// W tile (its 32 rows are output columns j), the "B" operand an X tile (32
// tokens i): a lane ends up with 4 consecutive output columns of one token per
// register quad.
//
// Shapes built: 256 x 256 and 128 x 256 (columns x tokens) with eight waves
// (two per SIMD, 128 / 64 accumulator registers each), 192 x 256, 128 x 128,
// 192 x 128 and 192 x 64 with four.  Eight waves read each X tile from LDS twice as often, but two
// waves per SIMD cover each other's waits in the epilogue, which takes 7.5 k
// to 9 k clocks instead of 13 k at 256 x 256 (the K loop is fed by the same
// loads: 1 100-1 170 clocks per stage either way); measured A/B on one box:
// 338.5 against 344.7 us on a 4096 x 5120 x 20480 product, 38.1 against
// 39.3 us on 2048 x 4096 x 4096.  192 x 256 does not split evenly over eight
// waves (14 row tiles).
//
// K pipeline.  A stage is 64 features (2 MFMA k-steps) of all 2*WA + WQ*WB row
// tiles; NB = 4 stages form a ring in LDS.  Tiles go global -> LDS with
// 16-byte direct loads (one 1 KiB tile piece per wave instruction, the pieces
// of a stage dealt evenly to the waves) and come back with one ds_read_b128
// per operand (linear, conflict free).  The operands of a whole stage sit in registers, double
// buffered: while the MFMAs of stage st run from one register set, stage st+1
// is read from LDS into the other and stage st+4 is requested from memory.
// One barrier per stage, at its top: it publishes stage st+1 (every wave
// waited for its own pieces) and retires the ring slot of stage st (every wave
// has it in registers), which is refilled right away.
//
// The stage sequence of a tile continues past K with two "epilogue stages"
// that bring c_w, c_x, the gathered outlier columns Xo and rows O of the
// original fp16 weights into the ring slots that fall free first, so that the
// epilogue finds them in LDS without having waited for them.
//
// Workgroups are persistent: the grid is one workgroup per compute unit and
// each walks its share of the tiles.  The first two stages of the next tile
// are requested before the epilogue of the current one starts (into the two
// slots its last two stages leave), the next two right after it (into the
// slots of the epilogue stages), so a tile does not start with an empty
// pipeline.  Ring slots are addressed relative to a per-tile base for that.
// ---------------------------------------------------------------------------
// Measurement build (-DLLMINT8_GEMM_STAMPS, a library of its own: see build.py): every wave of one workgroup
// records the shader clock at the phase boundaries of its second tile (its only tile, if it has one).
// Stamp k of wave w is g_stamps[w][k]:
//   0 tile start, 1 first stage in LDS, 2 K loop done, 3 epilogue operands in LDS, 4 next tile's first two
//   stages requested, 5 row constants / outlier columns of X in registers, then per pass over two column
//   tiles (p = 0, 1): 6+6p column constants / outlier rows of W in registers, and per staged block of 64
//   columns (q = 0, 1; 64 tokens with four waves, 32 with eight) 7+6p+2q dequantized and staged, 8+6p+2q
//   written out; 20 tile done; 21 kernel entry; 22 / 23 the constant 100 MHz counter at stamps 0 / 20 (the
//   shader clock inside the tile follows from the two pairs).
// In the product build the macro is empty.
#ifdef LLMINT8_GEMM_STAMPS
__device__ long long g_stamps[8][32];
#define STAMP(k)                                                                                   \
    do {                                                                                           \
        if (blockIdx.x == 9 && lane == 0 && pos == stamp_pos) {                                    \
            g_stamps[w][k] = clock64();                                                            \
            if ((k) == 0 || (k) == 20) g_stamps[w][(k) == 0 ? 22 : 23] = wall_clock64();           \
        }                                                                                          \
    } while (0)
#else
#define STAMP(k) do { } while (0)
#endif

constexpr int NB = 4;
constexpr int OSLOTS = 32;  // outlier slots staged through LDS; more are read from memory directly

//
// ZP: zeropoint constants (Eq. 1-5) in place of c_x / c_w.  The epilogue adds the correction terms of
// the unrolled product of Eq. 5 to the accumulators (in double: with zeropoints far from 0 they are
// large and cancel) and divides by nd_x nd_w.  The records of the tile's tokens and the three planes
// of column factors travel through the epilogue stages like the absmax constants do.
//
// GUARDED: the epilogue reads its operands from memory with every access guarded and can export the raw
// accumulators (o not a multiple of 8, unaligned operands, more than 32 outlier columns, or the export asked
// for).  Otherwise the epilogue is fed from LDS by the two epilogue stages and nothing in it is guarded.
template <int WA, int WB, int WQ, bool ZP, bool GUARDED>
__global__ void __launch_bounds__(128 * WQ, 1) gemm_prefill_kernel(const GemmArgs g)
{
    constexpr int NWAVES = 2 * WQ;               // waves: 2 along the columns x WQ along the tokens
    constexpr int TW = 2 * WA, TX = WQ * WB;     // row tiles of W and of X in the workgroup tile
    constexpr int PIECES = (TW + TX) / WQ;       // direct loads per wave per stage
    static_assert(PIECES * WQ == TW + TX && (WQ == 2 || WQ == 4), "the pieces of a stage must divide evenly among the waves");
    constexpr int STAGE = (TW + TX) * 2 * TILE_BYTES;
    constexpr int NMFMA = 2 * WA * WB;
    constexpr int NRD = 2 * (WA + WB);
    constexpr int NOPS = PIECES + NRD;
    constexpr int OPSPAN = NMFMA;                // MFMA slots of a stage that carry its requests and LDS reads
    constexpr int NEW = 16;                      // epilogue-stage pieces holding W rows: [32 slots][256 columns] fp16
    constexpr int NEX = 2 * TX;                  // pieces holding Xo: [32*TX tokens][opad <= 32 slots] fp16
    constexpr int NZX = ZP ? TX / 2 : 0;         // zeropoint: pieces holding the tokens' records, 64 of 16 bytes each
    constexpr int NZP = ZP ? (WA + 1) / 2 : 0;   // zeropoint: pieces per plane of column factors, 128 doubles each
    constexpr int NST = (WA + 1) / 2 * 4 * WB;   // store instructions of a wave in the unguarded epilogue
    static_assert((NB - 2) * PIECES + NST < 64, "vmcnt is a 6-bit counter");
    static_assert(TX % 2 == 0 && NEW + NEX + 1 + NZX + 3 * NZP <= 2 * NWAVES * PIECES, "epilogue operands must fit two stages");

    extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int s = g.s, o = g.o, KT = g.KT, opad = g.opad;
    const int lpad = opad < OSLOTS ? opad : OSLOTS;  // slots per token in the LDS image of Xo (16 or 32)
    const int wp = w / WQ, wq = w % WQ;  // wave position: column half, token part

    // ---- this workgroup's tiles.  Hardware deals consecutive workgroup ids round-robin to the 8
    // XCDs; each XCD gets a contiguous run of the tile order, so that tiles sharing operand panels
    // meet in one L2, and its workgroups walk that run side by side.  Within the order, bands of 4
    // token blocks are walked column block by column block.
    const int total = g.nP * g.nQ;
    const int xcd = blockIdx.x & 7;
    const int x0 = xcd * (total >> 3) + (xcd < (total & 7) ? xcd : (total & 7));  // first tile of the XCD's run
    const int n_x = (total >> 3) + (xcd < (total & 7) ? 1 : 0);                  // its length
    const int gx = ((int)gridDim.x - xcd + 7) >> 3;                              // workgroups on this XCD
    int pos = blockIdx.x >> 3;
    if (pos >= n_x) return;
#ifdef LLMINT8_GEMM_STAMPS
    const int stamp_pos = pos + (pos + gx < n_x ? gx : 0);
#endif

#ifdef LLMINT8_GEMM_STAMPS
    if (blockIdx.x == 9 && lane == 0) g_stamps[w][21] = clock64();  // kernel entry
#endif
    // The number of outlier columns, and in lane t < 32 the weight row of outlier slot t (row 0 for unused
    // slots: finite values that meet the zeros of Xo).  Both are loaded below, behind the requests of the
    // first tile's first two stages: two dependent round trips that would otherwise sit in front of them.
    int cnt = 0;
    int myk = 0;

    // ---- loader state: the tile whose stages are being requested.
    // Piece p = w*PIECES + k of a stage is k-half (p & 1) of row tile p >> 1 (W tiles first, then
    // X tiles); it lands at byte p * 1024 of the stage's ring slot.
    const unsigned voff = lane * 16;
    const int8_t* gpp[PIECES];
    int J0w, I0w;   // first column / token of the tile
    auto set_loader = [&](int logical) {
        constexpr int BAND = 4;
        const int nP = g.nP, nQ = g.nQ;
        const int band = logical / (BAND * nP);
        const int inband = logical - band * BAND * nP;
        const int q0 = band * BAND;
        const int bh = (nQ - q0) < BAND ? (nQ - q0) : BAND;  // token blocks in this band
        const int pj = inband / bh;
        const int qi = q0 + inband - pj * bh;
        J0w = pj * 64 * WA;
        I0w = qi * 32 * TX;
#pragma unroll
        for (int k = 0; k < PIECES; k++) {
            const int p = w * PIECES + k;
            const int r = p >> 1;
            const int8_t* base;
            if (r < TW) {
                int t = pj * TW + r;
                t = t < g.JT ? t : g.JT - 1;  // rows past the matrix re-read the last tile, results unused
                base = g.Wq + (size_t)t * KT * TILE_BYTES;
            } else {
                int t = qi * TX + (r - TW);
                t = t < g.RT ? t : g.RT - 1;
                base = g.Xq + (size_t)t * KT * TILE_BYTES;
            }
            const unsigned long long b = (unsigned long long)(base + (p & 1) * TILE_BYTES);
            const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)b);
            const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(b >> 32));
            gpp[k] = (const int8_t*)(((unsigned long long)hi << 32) | lo);  // uniform: lives in scalar registers
        }
    };
    set_loader(x0 + pos);
    const int nst = KT / 2;   // KT is a multiple of 4, so nst is even and >= 2
    int sbase = 0;            // ring slot of the current tile's stage 0 (0 or 2); stage v sits in slot (sbase + v) % NB

    // Source of piece n (0 .. 8*PIECES-1) of the epilogue stages, per lane.  Layout of the two stages:
    // pieces 0..15: rows O of W_f16, [32 slots][256 columns] (a slot row is 512 bytes whatever WA is; lanes past
    // the tile's 64*WA columns repeat chunk 0); then 2*TX pieces of Xo, [32*TX tokens][opad slots] as it lies in
    // memory; then one piece with c_w (lanes 0-31) and c_x (lanes 32-63).  Zeropoint: that piece is idle, and
    // TX/2 pieces with the records of the tile's tokens and 3 x NZP pieces with the planes of column factors
    // follow.  Whatever is left of the two stages re-reads a harmless piece.  Where a ragged tile reaches past the
    // last token, the lanes re-read a token that exists (the last one; for c_x, whose 16-byte chunks hold eight
    // tokens, the tile's first chunk); where it reaches past the last column, the tile's first columns (o is a
    // multiple of 8 here).  Nothing computed from those values is stored.  The chunk of c_x that holds the last
    // token is read whole: when s is not a multiple of 8 that is up to 14 bytes past the array, inside the same
    // aligned 16 bytes (c_x is 16-byte aligned here), hence inside the same page as c_x[s-1].
    auto esrc = [&](int n) -> const void* {
        // The addresses depend on the tile only; the opaque copy of the lane number keeps the compiler from
        // computing all of them at the start of the tile and carrying them through the K loop in registers.
        int ln = lane;
        asm volatile("" : "+v"(ln));
        if constexpr (GUARDED) return g.Xq + ln * 16;  // the guarded epilogue reads its operands from memory itself
        int wchunk = ((ln & 31) < 8 * WA ? (ln & 31) : 0) * 8;  // column offset of this lane in a W row
        wchunk = J0w + wchunk < o ? wchunk : 0;
        if (n < NEW) {
            const int k0 = __builtin_amdgcn_readlane(myk, 2 * n), k1 = __builtin_amdgcn_readlane(myk, 2 * n + 1);
            const int k = (ln >> 5) ? k1 : k0;  // the piece holds slots 2n (lanes 0-31) and 2n+1 (lanes 32-63)
            return g.Wf + ((size_t)k * o + J0w + wchunk);
        }
        if (n < NEW + NEX) {
            const int pn = (n - NEW) * 32 < NEX * lpad ? (n - NEW) : 0;  // 16 slots: half as many pieces
            const int e = pn * 512 + ln * 8;                              // element of the image [32*TX tokens][lpad]
            int i = I0w + (lpad == 32 ? e >> 5 : e >> 4);
            i = i < s ? i : s - 1;
            return g.Xo + ((size_t)i * opad + (e & (lpad - 1)));
        }
        if constexpr (ZP) {
            const int m = n - (NEW + NEX + 1);
            if (m >= 0 && m < NZX) {
                const int i = I0w + m * 64 + ln;
                return g.zp.zcx + (i < s ? i : s - 1);
            }
            if (m >= NZX && m < NZX + 3 * NZP) {
                const int q = (m - NZX) / NZP, pp = (m - NZX) % NZP;
                const int c = pp * 128 + 2 * ln;  // columns past the tile (odd WA) or past o re-read the tile's first two
                return g.zp.colc + ((size_t)q * g.zp.pitch + J0w + (c < 64 * WA && J0w + c < o ? c : 0));
            }
            return g.Xq + ln * 16;
        } else {
            if (n > NEW + NEX) return g.Xq + ln * 16;
            if (ln < 32) return g.cw + (J0w + wchunk);
            const int c = (ln - 32) < 4 * TX && I0w + (ln - 32) * 8 < s ? (ln - 32) : 0;
            return g.cx + (I0w + c * 8);
        }
    };
    // Request piece k of an operand stage into ring slot `slot`.  vo = byte offset of this lane within the
    // piece's row tile (stage * 2 KiB + lane * 16), the same for all pieces of a stage.  Uniform 64-bit base
    // + 32-bit lane offset is the scalar-base form of the load: two instructions per request (LDS address
    // into M0, the load), no address arithmetic in the K pipeline.
    auto dma_k = [&](unsigned vo, int slot, int k) {
        int8_t* dst = lds + slot * STAGE + (w * PIECES + k) * TILE_BYTES;
        const __attribute__((address_space(1))) int8_t* sb = (const __attribute__((address_space(1))) int8_t*)gpp[k];
        __builtin_amdgcn_global_load_lds(sb + vo, LPTR(dst), 16, 0, 0);
    };
    // The lane offset of operand stage v.  Opaque to the compiler, so that its zero extension stays next to
    // the loads that use it (hoisted out of the loop, it turns every request into a 64-bit vector add).
    auto stage_off = [&](int v) {
        unsigned vo = voff;
        asm volatile("" : "+v"(vo));  // (nor is voff + constant worth a register of its own across the K loop)
        vo += (unsigned)v * (2 * TILE_BYTES);
        asm volatile("" : "+v"(vo));
        return vo;
    };
    auto dma_e = [&](int e, int slot, int k) {
        int8_t* dst = lds + slot * STAGE + (w * PIECES + k) * TILE_BYTES;
        __builtin_amdgcn_global_load_lds(GPTR(esrc(e * NWAVES * PIECES + w * PIECES + k)), LPTR(dst), 16, 0, 0);
    };

    v16i acc[WA][WB];
    // operand registers of two stages: [set][k-step][tile]
    v4i RP[2][2][WA], RQ[2][2][WB];
    const int8_t* Pl = lds + (wp * WA) * 2 * TILE_BYTES + lane * 16;
    const int8_t* Ql = lds + (TW + wq * WB) * 2 * TILE_BYTES + lane * 16;
    // read number i (0 .. NRD-1) of a stage into register set S
    auto rd = [&](auto S, int slot, int i) {
        constexpr int SS = decltype(S)::value;
        const int c = i / (WA + WB), t = i % (WA + WB);
        if (t < WA)
            RP[SS][c][t] = *(const v4i*)(Pl + slot * STAGE + (t * 2 + c) * TILE_BYTES);
        else
            RQ[SS][c][t - WA] = *(const v4i*)(Ql + slot * STAGE + ((t - WA) * 2 + c) * TILE_BYTES);
    };
    // request all pieces of stage v (operand stage, or epilogue stage v - nst) of the loader tile
    auto issue_stage = [&](int v, int slot) {
        if (v < nst) {
            const unsigned vo = stage_off(v);
#pragma unroll
            for (int k = 0; k < PIECES; k++) dma_k(vo, slot, k);
        } else {
#pragma unroll
            for (int k = 0; k < PIECES; k++) dma_e(v - nst, slot, k);
        }
    };

    // One stage: MFMAs from register set S, interleaved with the requests of stage st+NB into the
    // slot of stage st and the reads of stage st+1 into the other register set.
    // MODE 0: operand stage st+NB; 1 / 2: first / second epilogue stage; 3: nothing left to request;
    // 4: last stage (nothing to request, nothing to read).
    // MODE 5: MODE 0 for stage 0 of a tile, where the stores of the previous tile's epilogue may still fly too.
    auto stage = [&](auto S, auto M, int st) {
        constexpr int SS = decltype(S)::value;
        constexpr int MODE = decltype(M)::value == 5 ? 0 : decltype(M)::value;
        // My pieces of stage st+1 have landed (two younger stages may still fly) and my reads of stage st
        // are complete; after the barrier the same holds for every wave.
        STAGE_SYNC((NB - 2) * PIECES + (decltype(M)::value == 5 ? NST : 0));
        FENCE();
        const int slot = (unsigned)(sbase + st) % NB, nslot = (unsigned)(sbase + st + 1) % NB;
        const unsigned vo = MODE == 0 ? stage_off(st + NB) : 0u;
#pragma unroll
        for (int i = 0; i < NMFMA; i++) {
            // boustrophedon over the WA x WB tiles: consecutive MFMAs share one operand register set
            const int c = i / (WA * WB), a = (i / WB) % WA, b = (a & 1) ? WB - 1 - i % WB : i % WB;
            acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(RP[SS][c][a], RQ[SS][c][b], acc[a][b], 0, 0, 0);
            FENCE();
#pragma unroll
            for (int q = (i < OPSPAN ? i : OPSPAN) * NOPS / OPSPAN; q < (i + 1 < OPSPAN ? i + 1 : OPSPAN) * NOPS / OPSPAN; q++) {
                // Four waves: the requests first, then the reads (with the reads first 192 x 256 loses a quarter
                // of its speed).  Eight waves: the reads first (0.5 % faster: the next stage's wait is for them).
                const bool is_req = WQ == 4 ? q >= NRD : q < PIECES;
                const int qr = WQ == 4 ? q - NRD : q, qd = WQ == 4 ? q : q - PIECES;
                if (is_req) {
                    if (MODE == 0) dma_k(vo, slot, qr);
                    if (MODE == 1 || MODE == 2) dma_e(MODE - 1, slot, qr);
                } else if (MODE != 4) {
                    rd(std::integral_constant<int, 1 - SS>{}, nslot, qd);
                }
            }
            FENCE();
        }
    };
    using I0_ = std::integral_constant<int, 0>;
    using I1_ = std::integral_constant<int, 1>;

    // stages 0 and 1 of the first tile (later tiles get theirs before the epilogue of the tile before)
    issue_stage(0, 0);
    issue_stage(1, 1);
    FENCE();
    {
        // idx is read up to the buffer's size, not up to the count, so that the two loads do not wait for
        // one another (entries past the count hold whatever the caller left there and are not used)
        unsigned kraw = 0;
        if (!g.rows_are_slots && (lane & 31) < g.cap) kraw = (unsigned)g.idx[lane & 31];
        cnt = *g.count;
        cnt = cnt < 0 ? 0 : (cnt > g.cap ? g.cap : cnt);
        if ((lane & 31) < cnt) {
            const unsigned k = g.rows_are_slots ? (unsigned)(lane & 31) : kraw;
            myk = k < (unsigned)g.wrows ? (int)k : 0;
        }
    }
    // once per kernel: with this load known to be complete, the compiler has no reason to drain the
    // direct-to-LDS loads in flight when myk is used later in the K pipeline
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
    FENCE();
    // An outlier buffer of more than OSLOTS columns: the launcher cannot know how many columns were found, so
    // it launches this kernel and its guarded instantiation behind it; the one whose case it is not leaves
    // here (every wave alike, nothing of its in flight any more).
    if constexpr (!GUARDED) {
        if (cnt > OSLOTS) return;
    } else {
        if (g.many_only && cnt <= OSLOTS) return;
    }

    // Memory operations of a wave complete in the order they were issued, and the requests of a tile's first two
    // stages are issued before the epilogue of the tile before it.  After an unguarded epilogue exactly NST
    // stores follow them (anything else the compiler may add only makes the waits below stricter), so the first
    // two waits of the next tile can leave those stores in flight and the K loop starts while they drain.
    // After a guarded epilogue, or with no tile before, everything is waited for instead.
    bool after_fast = false;
    for (;;) {  // tiles of this workgroup
        const int cJ0w = J0w, cI0w = I0w;  // the tile being computed (the loader moves on before its epilogue)
#pragma unroll
        for (int a = 0; a < WA; a++)
#pragma unroll
            for (int b = 0; b < WB; b++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[a][b][r] = 0;
        // Stage 0 has landed once at most the pieces of stage 1 (and the stores of an unguarded epilogue
        // before this tile) are in flight.  The barrier also tells that every wave is done with
        // the previous tile's epilogue stages, whose slots take stages 2 and 3 (with nst == 2: this
        // tile's own epilogue stages) once stage 0 is on its way into registers.
        STAMP(0);
        if (nst < 6)
            STAGE_SYNC(PIECES);
        else if (after_fast)
            STAGE_SYNC(PIECES + NST);
        else
            STAGE_SYNC(0);
        STAMP(1);
#pragma unroll
        for (int i = 0; i < NRD; i++) rd(I0_{}, sbase, i);
        FENCE();
        issue_stage(2, (sbase + 2) % NB);
        issue_stage(3, (sbase + 3) % NB);
        FENCE();
        int st = 0;
        if (nst >= 6) {
            stage(I0_{}, std::integral_constant<int, 5>{}, 0);
            stage(I1_{}, I0_{}, 1);
            st = 2;
        }
        for (; st + 6 <= nst; st += 2) {
            stage(I0_{}, I0_{}, st);
            stage(I1_{}, I0_{}, st + 1);
        }
        if (nst >= 4) {  // st == nst - 4
            stage(I0_{}, std::integral_constant<int, 1>{}, st);
            stage(I1_{}, std::integral_constant<int, 2>{}, st + 1);
            st += 2;
        }
        stage(I0_{}, std::integral_constant<int, 3>{}, st);
        stage(I1_{}, std::integral_constant<int, 4>{}, st + 1);
        STAMP(2);
        STAGE_SYNC(0);  // the epilogue stages have landed, every wave is done with the operand slots
        STAMP(3);

        const int eslot = (sbase + nst) % NB;  // 0 or 2; the second epilogue stage follows it
        const bool has_next = pos + gx < n_x;
        if (has_next) {
            // next tile: its stages 0 and 1 go to the slots of this tile's last two stages
            set_loader(x0 + pos + gx);
            issue_stage(0, (eslot + 2) % NB);
            issue_stage(1, (eslot + 3) % NB);
        }

        STAMP(4);
        // ---- epilogue ----------------------------------------------------------
        // acc[a][b][r] of lane l: token i = I0 + b*32 + (l & 31),
        //                         column j = J0 + a*32 + 8*(r >> 2) + 4*(l >> 5) + (r & 3)
        const int J0 = cJ0w + wp * 32 * WA;
        const int I0 = cI0w + wq * 32 * WB;
        // lane-derived offsets are taken from an opaque copy of the lane number, so that they are recomputed
        // here for every tile instead of being carried through the K loop in registers
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
        const int gl = lane_e >> 5, ll = lane_e & 31;

        const int8_t* E = lds + eslot * STAGE;
        const unsigned short* EW = (const unsigned short*)E;                               // [32][256]
        const int8_t* EX = E + NEW * TILE_BYTES;                                           // [64*WB][lpad] fp16
        const unsigned short* ECw = (const unsigned short*)(E + (NEW + NEX) * TILE_BYTES); // [64*WA]
        const unsigned short* ECx = ECw + 256;                                             // [64*WB]
        const int4* EZx = (const int4*)(E + (NEW + NEX + 1) * TILE_BYTES);                 // zeropoint: [64*WB] records
        const double* EZc = (const double*)(E + (NEW + NEX + 1 + NZX) * TILE_BYTES);       // 3 planes of NZP*128 doubles
        // output staging behind the ring (the ring slots are busy with the next tile): 8 KiB per wave
        // (a block of 64 tokens x 64 columns), 4 KiB (32 tokens) with eight waves
        constexpr int BU = WQ == 2 ? 2 : 1;  // token tiles per staged block
        int8_t* stg = lds + NB * STAGE + w * (BU * 4096);

        // rows O of the fp16 weights for column jcol, outlier slots t0 + 8*gl .. +7, straight from memory
        // (both without conditions on the loads themselves, so that the eight indices, then the eight weights, are
        // in flight together: a slot, column or token that does not exist reads one that does and is zeroed)
        auto load_w_mem = [&](int jcol, int t0) {
            unsigned k[8];
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const int t = t0 + 8 * gl + e;
                k[e] = g.rows_are_slots ? (unsigned)t : (unsigned)g.idx[t < cnt ? t : 0];
            }
            unsigned short v[8];
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const bool ok = t0 + 8 * gl + e < cnt && k[e] < (unsigned)g.wrows;
                v[e] = g.Wf[(size_t)(ok ? k[e] : 0u) * o + (jcol < o ? jcol : 0)];
            }
            v8h wa;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const bool ok = t0 + 8 * gl + e < cnt && k[e] < (unsigned)g.wrows && jcol < o;
                wa[e] = __builtin_bit_cast(_Float16, ok ? v[e] : (unsigned short)0);
            }
            return wa;
        };
        auto load_x_mem = [&](int i, int t0) {
            const v8h xb = *(const v8h*)(g.Xo + (size_t)(i < s ? i : s - 1) * opad + t0 + 8 * gl);
            return i < s ? xb : (v8h)(0);
        };

        // FAST: operands from the LDS image of the epilogue stages, no guards.  Its stores go
        // through a buffer descriptor that spans the tile's existing tokens (rows of Out from the tile's first
        // token on): where a ragged tile reaches past the last token the hardware drops them, and lanes whose
        // columns do not exist offer an offset past the buffer's end, so a wave issues the same NST store
        // instructions whatever the tile.
        // Otherwise: operands from memory, every access guarded; also exports the raw accumulators.
        const int trows = s - cI0w < 32 * TX ? s - cI0w : 32 * TX;
        const __amdgpu_buffer_rsrc_t obuf =
            __builtin_amdgcn_make_buffer_rsrc(g.Out + (size_t)cI0w * o, 0, trows * o * 2, 0x00020000);
        auto epilogue = [&](auto F) {
            constexpr bool FAST = decltype(F)::value;
            if (!FAST && g.Cdbg) {
#pragma unroll
                for (int a = 0; a < WA; a++)
#pragma unroll
                    for (int b = 0; b < WB; b++) {
                        const int i = I0 + b * 32 + ll;
#pragma unroll
                        for (int r = 0; r < 16; r++) {
                            const int j = J0 + a * 32 + 8 * (r >> 2) + 4 * gl + (r & 3);
                            if (i < s && j < o) g.Cdbg[(size_t)i * o + j] = acc[a][b][r];
                        }
                    }
            }
            float sx[WB];      // c_x / 127^2 of this lane's tokens (Eq. 7: S = c_x (x) c_w / 127^2)
            double zsa[ZP ? WB : 1], zza[ZP ? WB : 1], zrs[ZP ? WB : 1];  // zeropoint: D_x / 254, zp_x, row sum of the codes
            v8h xb[WB][2];     // MFMA "B" operand of the outlier product: slots 8*gl .. +7 (+16) of this lane's tokens
#pragma unroll
            for (int b = 0; b < WB; b++) {
                const int il = wq * 32 * WB + b * 32 + ll;  // token within the workgroup tile
                const int i = cI0w + il;
                if (FAST) {
                    if constexpr (ZP) {
                        const int4 rec = EZx[il];
                        zsa[b] = zp_range((unsigned)rec.x) * (1.0 / 254.0);
                        zza[b] = (double)rec.y;
                        zrs[b] = (double)rec.z;
                    } else {
                        sx[b] = f16_bits_to_float(ECx[il]) * (1.0f / 16129.0f);
                    }
                    xb[b][0] = *(const v8h*)(EX + il * (2 * lpad) + gl * 16);
                    xb[b][1] = (v8h)(0);
                    if (cnt > 16) xb[b][1] = *(const v8h*)(EX + il * (2 * lpad) + (2 + gl) * 16);  // then lpad == 32
                } else {
                    if constexpr (ZP) {
                        int4 rec = g.zp.zcx[i < s ? i : s - 1];
                        if (i >= s) rec = make_int4(0, 0, 0, 0);
                        zsa[b] = zp_range((unsigned)rec.x) * (1.0 / 254.0);
                        zza[b] = (double)rec.y;
                        zrs[b] = (double)rec.z;
                    } else {
                        const float cxi = f16_bits_to_float(g.cx[i < s ? i : s - 1]) * (1.0f / 16129.0f);
                        sx[b] = (i < s) ? cxi : 0.0f;
                    }
                    xb[b][0] = cnt > 0 ? load_x_mem(i, 0) : (v8h)(0);
                    xb[b][1] = cnt > 16 ? load_x_mem(i, 16) : (v8h)(0);
                }
            }
            // zeropoint: this wave's 32*WA columns of the three factor planes, copied once per tile into a
            // wave-private piece of the epilogue-stage slots (they hold nothing such tiles need, and are
            // not refilled before every wave has passed the barrier at the top of the next tile)
            // (the unguarded epilogue finds the planes of the whole workgroup tile in the epilogue stages instead)
            double* ZC = (double*)(lds + eslot * STAGE) + w * (3 * 32 * WA);
            const double* zc0 = FAST ? EZc + wp * 32 * WA : ZC;  // this wave's first column in plane 0
            const int zstride = FAST ? NZP * 128 : 32 * WA;     // doubles from plane to plane
            if constexpr (ZP && !FAST) {
#pragma unroll
                for (int q = 0; q < 3; q++)
                    for (int c = lane_e; c < 32 * WA; c += 64)
                        ZC[q * 32 * WA + c] = g.zp.colc[(size_t)q * g.zp.pitch + J0 + c];
                // read back by other lanes of the same wave only: LDS serves a wave's requests in order,
                // the compiler just must not move the reads up
                asm volatile("" ::: "memory");
                __builtin_amdgcn_wave_barrier();
            }
            STAMP(5);
#pragma unroll
            for (int a0 = 0; a0 < WA; a0 += 2) {
                constexpr int WA_ = WA;
                const int na = (WA_ - a0) < 2 ? (WA_ - a0) : 2;  // column tiles in this pass: 2, or 1 at the end of an odd WA
                float cwv[2][16];
                v8h wa[2][2];
#pragma unroll
                for (int aa = 0; aa < 2; aa++) {
                    if (aa >= na) break;
                    const int jl = wp * 32 * WA + (a0 + aa) * 32;  // first column of the MFMA tile within the workgroup tile
                    if (FAST) {
                        if constexpr (!ZP) {
#pragma unroll
                            for (int rr = 0; rr < 4; rr++) {
                                const uint2 pk = *(const uint2*)(ECw + jl + 8 * rr + 4 * gl);
                                cwv[aa][4 * rr + 0] = f16_bits_to_float((unsigned short)(pk.x & 0xffff));
                                cwv[aa][4 * rr + 1] = f16_bits_to_float((unsigned short)(pk.x >> 16));
                                cwv[aa][4 * rr + 2] = f16_bits_to_float((unsigned short)(pk.y & 0xffff));
                                cwv[aa][4 * rr + 3] = f16_bits_to_float((unsigned short)(pk.y >> 16));
                            }
                        }
#pragma unroll
                        for (int ks = 0; ks < 2; ks++)
#pragma unroll
                            for (int e = 0; e < 8; e++)
                                wa[aa][ks][e] =
                                    __builtin_bit_cast(_Float16, EW[(16 * ks + 8 * gl + e) * 256 + jl + ll]);
                    } else {
                        if constexpr (!ZP) {
#pragma unroll
                            for (int r = 0; r < 16; r++) {
                                const int j = cJ0w + jl + 8 * (r >> 2) + 4 * gl + (r & 3);
                                const float cwj = f16_bits_to_float(g.cw[j < o ? j : 0]);
                                cwv[aa][r] = (j < o) ? cwj : 0.0f;
                            }
                        }
                        wa[aa][0] = cnt > 0 ? load_w_mem(cJ0w + jl + ll, 0) : (v8h)(0);
                        wa[aa][1] = cnt > 16 ? load_w_mem(cJ0w + jl + ll, 16) : (v8h)(0);
                    }
                }
                STAMP(6 + 6 * (a0 / 2));
#pragma unroll
                for (int b0 = 0; b0 < WB; b0 += BU) {
                    int8_t* sb = stg;
                    // ---- 32*BU tokens x 64 columns: dequantize, add the outlier product, stage as fp16 rows in LDS
#pragma unroll
                    for (int aa = 0; aa < 2; aa++) {
                        if (aa >= na) break;
                        const int a = a0 + aa;
#pragma unroll
                        for (int bb = 0; bb < BU; bb++) {
                            if (b0 + bb >= WB) break;
                            const int b = b0 + bb;
                            // Eq. 8: outlier product first (fp32 accumulation in the matrix unit), then one fused
                            // multiply-add per output puts the dequantized int8 product (Eq. 7) on top
                            v16f d;
                            if (cnt > 0) {
                                v16f t = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                                t = __builtin_amdgcn_mfma_f32_32x32x16_f16(wa[aa][0], xb[b][0], t, 0, 0, 0);
                                if (cnt > 16) t = __builtin_amdgcn_mfma_f32_32x32x16_f16(wa[aa][1], xb[b][1], t, 0, 0, 0);
                                if (!FAST)
                                    for (int t0 = OSLOTS; t0 < cnt; t0 += 16) {  // more than 32 outlier columns: rare
                                        const v8h wm = load_w_mem(J0 + a * 32 + ll, t0);
                                        const v8h xm = load_x_mem(I0 + b * 32 + ll, t0);
                                        t = __builtin_amdgcn_mfma_f32_32x32x16_f16(wm, xm, t, 0, 0, 0);
                                    }
                                if constexpr (!ZP) {
#pragma unroll
                                    for (int r = 0; r < 16; r++)
                                        d[r] = __builtin_fmaf((float)acc[a][b][r] * sx[b], cwv[aa][r], t[r]);
                                } else {
                                    d = t;
                                }
                            } else {
#pragma unroll
                                for (int r = 0; r < 16; r++)
                                    d[r] = ZP ? 0.0f : (float)acc[a][b][r] * sx[b] * cwv[aa][r];
                            }
                            if constexpr (ZP) {
                                // Eq. 5 over nd_w: C p + rowsum q + zp_x r with the column factors of
                                // zp_kcol_kernel (planes padded with zeros: no guards), then the division by nd_x
#pragma unroll
                                for (int r = 0; r < 16; r++) {
                                    const int c = a * 32 + 8 * (r >> 2) + 4 * gl + (r & 3);
                                    const double cp = zc0[c], cq = zc0[zstride + c], cr = zc0[2 * zstride + c];
                                    d[r] += (float)(zsa[b] * __builtin_fma((double)acc[a][b][r], cp,
                                                                           __builtin_fma(zrs[b], cq, zza[b] * cr)));
                                }
                            }
                            // staging row of token tl (0..63): 128 bytes = 8 chunks of 16, chunk q stored at
                            // q ^ ((tl >> 1) & 7) to spread the banks
                            const int tl = bb * 32 + ll;
#pragma unroll
                            for (int rr = 0; rr < 4; rr++) {
                                const v4h hv = {(_Float16)d[4 * rr], (_Float16)d[4 * rr + 1], (_Float16)d[4 * rr + 2],
                                                (_Float16)d[4 * rr + 3]};
                                const int q = aa * 4 + rr;
                                *(v4h*)(sb + tl * 128 + ((q ^ ((tl >> 1) & 7)) << 4) + gl * 8) = hv;
                            }
                        }
                    }
                    // The staged values are read back by other lanes of the same wave, through pointers of another
                    // type: LDS serves a wave's requests in order, the compiler must not reorder them either.
                    STAMP(7 + 6 * (a0 / 2) + 2 * (b0 / BU));
                    asm volatile("" ::: "memory");
                    // ---- write the staged block: a lane moves 16 bytes, 8 lanes cover a token's 128 bytes
#pragma unroll
                    for (int p = 0; p < 4 * BU; p++) {
                        if (p >= 4 && b0 + 1 >= WB) break;  // an odd WB stages 32 tokens in its last block
                        const int tl = p * 8 + (lane_e >> 3), q = lane_e & 7;
                        const u4 v = *(const u4*)(sb + tl * 128 + ((q ^ ((tl >> 1) & 7)) << 4));
                        const int i = I0 + b0 * 32 + tl;
                        const int j = J0 + a0 * 32 + q * 8;
                        if (FAST) {
                            if (na == 2 || q < 4)  // byte offset < 2^31: o is bounded for this path; 2 = non-temporal
                                __builtin_amdgcn_raw_buffer_store_b128(v, obuf, j < o ? ((i - cI0w) * o + j) * 2 : 0x7fffffff,
                                                                       0, 2);
                        } else if ((tl < 32 || b0 + 1 < WB) && i < s && q < 4 * na) {
                            if (g.fast_ok && j + 8 <= o) {
                                *(u4*)(g.Out + (size_t)i * o + j) = v;
                            } else {
                                const _Float16* hv = (const _Float16*)&v;
#pragma unroll
                                for (int e = 0; e < 8; e++)
                                    if (j + e < o) g.Out[(size_t)i * o + j + e] = hv[e];
                            }
                        }
                    }
                    asm volatile("" ::: "memory");  // the next block's staging writes stay behind these reads
                    STAMP(8 + 6 * (a0 / 2) + 2 * (b0 / BU));
                }
            }
        };
        epilogue(std::integral_constant<bool, !GUARDED>{});

        STAMP(20);
        if (!has_next) break;
        after_fast = !GUARDED;
        sbase = (eslot + 2) % NB;
        pos += gx;
    }  // tiles
}

// ---- per-device set-up ---------------------------------------------------------
// The kernels need more dynamic LDS than the default limit, and the attribute that raises it belongs to a
// kernel as loaded on one device.  The first launch on a device (or llmint8_init) sets it for EVERY
// instantiation at once, under a lock, and caches the number of compute units; later calls only read an
// atomic flag.  A caller that records calls into a graph therefore needs one call of any shape (or
// llmint8_init) on the device beforehand, not one per tile shape.
template <int WA, int WB, int WQ>
constexpr int prefill_lds_bytes()
{
    return NB * (2 * WA + WQ * WB) * 2 * TILE_BYTES + 32768;  // operand ring + output staging (32 KiB over all waves)
}

template <int WA, int WB, int WQ>
static hipError_t raise_lds_limit()
{
    const void* k[4] = {(const void*)gemm_prefill_kernel<WA, WB, WQ, false, false>,
                        (const void*)gemm_prefill_kernel<WA, WB, WQ, false, true>,
                        (const void*)gemm_prefill_kernel<WA, WB, WQ, true, false>,
                        (const void*)gemm_prefill_kernel<WA, WB, WQ, true, true>};
    for (const void* f : k) {
        const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, prefill_lds_bytes<WA, WB, WQ>());
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

constexpr int MAX_DEVICES = 64;
static std::atomic<int> g_dev_cus[MAX_DEVICES];  // 0: not set up yet; else the device's compute units
static std::mutex g_dev_lock;

hipError_t prefill_device_setup(int* cus)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool cached = dev >= 0 && dev < MAX_DEVICES;
    if (cached) {
        const int n = g_dev_cus[dev].load(std::memory_order_acquire);
        if (n > 0) {
            *cus = n;
            return hipSuccess;
        }
    }
    std::lock_guard<std::mutex> hold(g_dev_lock);
    if ((e = raise_lds_limit<4, 2, 4>()) != hipSuccess) return e;
    if ((e = raise_lds_limit<3, 4, 2>()) != hipSuccess) return e;
    if ((e = raise_lds_limit<2, 2, 4>()) != hipSuccess) return e;
    if ((e = raise_lds_limit<2, 2, 2>()) != hipSuccess) return e;
    if ((e = raise_lds_limit<3, 2, 2>()) != hipSuccess) return e;
    if ((e = raise_lds_limit<3, 1, 2>()) != hipSuccess) return e;
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    *cus = n;
    if (cached) g_dev_cus[dev].store(n, std::memory_order_release);
    return hipSuccess;
}

template <int WA, int WB, int WQ, bool ZP>
static hipError_t launch_cfg(GemmArgs& g, hipStream_t st)
{
    constexpr int shm = prefill_lds_bytes<WA, WB, WQ>();
    g.nP = (g.JT + 2 * WA - 1) / (2 * WA);
    g.nQ = (g.RT + WQ * WB - 1) / (WQ * WB);
    int ncu = 0;
    const hipError_t e = prefill_device_setup(&ncu);
    if (e != hipSuccess) return e;
    const int total = g.nP * g.nQ;
    const int grid = total < ncu ? total : ncu;
    // The unguarded epilogue takes outputs and epilogue operands in 16-byte pieces and up to OSLOTS outlier
    // columns.  With a larger outlier buffer both instantiations are launched; each looks at the count and the
    // one whose case it is not returns at once (about 3 us for the empty launch).
    g.many_only = 0;
    if (g.fast_ok && !g.Cdbg) {
        gemm_prefill_kernel<WA, WB, WQ, ZP, false><<<grid, 128 * WQ, shm, st>>>(g);
        if (g.opad <= OSLOTS) return hipGetLastError();
        const hipError_t e1 = hipGetLastError();
        if (e1 != hipSuccess) return e1;
        g.many_only = 1;
    }
    gemm_prefill_kernel<WA, WB, WQ, ZP, true><<<grid, 128 * WQ, shm, st>>>(g);
    return hipGetLastError();
}

static inline bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// Tile shape: the one with the smallest estimate of the kernel's time,
//   max( passes x (MFMA time of a tile),  all tiles' operand bytes / what the L2s deliver together,
//        (time to stream W from HBM once) / (share of the compute units that have a tile) )  +  a little per pass,
// passes = the rounds the compute units need for the tile grid.  The first term decides long X (a
// 256 x 256 tile moves the fewest operand bytes per MFMA), the second the middle range, where every compute
// unit pulls operands at once, the third short X, where the call is bound by streaming W once and compute
// units without a tile waste their share of that stream (with 192-column tiles a 49 152-column weight matrix
// is exactly one tile per compute unit).  The constants are fitted to the kernel times of all six shapes on
// five weight matrices at 33 to 1 024 tokens and to the three full-size workloads: the choice is then within
// 0.8 % of the fastest shape on average and 9 % in the worst case (5 120 x 20 480 at 1 024 tokens).
constexpr int NCFG = 6;
int pick_cfg(int s, int h, int o)
{
    static const int cols[NCFG] = {256, 192, 128, 128, 192, 192}, toks[NCFG] = {256, 256, 256, 128, 128, 64};
    static const double eff[NCFG] = {1.0, 0.96, 0.95, 0.85, 0.8, 0.5};  // relative MFMA rate of the main loop
    const double mfma_per_cu = 8e12, l2_all = 14e12, hbm = 6.9e12, ncu = 256.0, per_pass = 1.5e-6;
    int best = 0;
    double bestc = 0;
    for (int c = 0; c < NCFG; c++) {
        const double nP = (double)((o + cols[c] - 1) / cols[c]), nQ = (double)((s + toks[c] - 1) / toks[c]);
        const double tiles = nP * nQ, passes = (double)(long)((tiles + ncu - 1) / ncu);
        const double t_mfma = passes * 2.0 * cols[c] * toks[c] * h / (mfma_per_cu * eff[c]);
        const double t_l2 = tiles * (cols[c] + toks[c]) * h / l2_all;
        const double t_hbm = (double)o * h / hbm * (passes * ncu / tiles);
        double cost = t_mfma > t_l2 ? t_mfma : t_l2;
        cost = (cost > t_hbm ? cost : t_hbm) + per_pass * (passes - 1);
        if (c == 0 || cost < bestc) { best = c; bestc = cost; }
    }
    return best;
}

std::atomic<int> g_force_cfg{-1};  // test hook: tile shape override (-1 = automatic)

hipError_t launch_gemm_prefill(const int8_t* Xq, const unsigned short* cx, const unsigned short* Xo,
                               const int32_t* count, int cap, const int8_t* Wq, const unsigned short* cw,
                               const unsigned short* Wf, int rows_are_slots, const int32_t* idx, int s, int h, int o,
                               unsigned short* Out, int32_t* Cdbg, hipStream_t st, const ZpArgs* zp)
{
    GemmArgs g;
    g.zp = zp ? *zp : ZpArgs{nullptr, nullptr, 0};
    g.rows_are_slots = rows_are_slots;
    g.wrows = rows_are_slots ? opad_of(cap) : h;
    g.Wq = Wq; g.Xq = Xq;
    g.KT = k_tiles(h); g.JT = row_tiles(o); g.RT = row_tiles(s);
    g.nP = g.nQ = 0;
    g.cw = cw; g.cx = cx; g.Wf = Wf; g.idx = idx; g.Xo = (const _Float16*)Xo; g.count = count;
    g.cap = cap; g.opad = opad_of(cap);
    g.Out = (_Float16*)Out; g.Cdbg = Cdbg;
    g.s = s; g.h = h; g.o = o;
    g.fast_ok = (o % 8 == 0) && o < (1 << 21) && al16(cw) && al16(cx) && al16(Wf) && al16(Xo) && al16(Out) && al16(g.zp.zcx) &&
                al16(g.zp.colc);
    const int forced = g_force_cfg.load(std::memory_order_relaxed);
    const int c = forced >= 0 ? forced : pick_cfg(s, h, o);
    if (zp) {
        switch (c) {
            case 1: return launch_cfg<3, 4, 2, true>(g, st);
            case 2: return launch_cfg<2, 2, 4, true>(g, st);
            case 3: return launch_cfg<2, 2, 2, true>(g, st);
            case 4: return launch_cfg<3, 2, 2, true>(g, st);
            case 5: return launch_cfg<3, 1, 2, true>(g, st);
            default: return launch_cfg<4, 2, 4, true>(g, st);
        }
    }
    switch (c) {
        case 1: return launch_cfg<3, 4, 2, false>(g, st);
        case 2: return launch_cfg<2, 2, 4, false>(g, st);
        case 3: return launch_cfg<2, 2, 2, false>(g, st);
        case 4: return launch_cfg<3, 2, 2, false>(g, st);
        case 5: return launch_cfg<3, 1, 2, false>(g, st);
        default: return launch_cfg<4, 2, 4, false>(g, st);
    }
}

}  // namespace llmint8

#ifdef LLMINT8_GEMM_STAMPS
// measurement build only: the 8 x 32 clock stamps of the last launch (host buffer of 256 long long; rows 4-7 only with eight waves)
extern "C" int llmint8_debug_read_stamps(long long* out)
{
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(llmint8::g_stamps), sizeof(long long) * 8 * 32);
}
#endif
